// Row kernels: everything of the step that is not a matrix product or attention.
// One workgroup of 256 threads handles one token row end to end, so the row-wide
// reductions (RMSNorm mean square, cosine dot product and norms) stay inside a workgroup:
// wavefront shuffles first, then a fixed-order sum over the four wavefronts.  They also
// add up the float32 slices the split contraction of the GEMMs leaves behind, round once to
// the storage type, and do the cache scatter, so no value makes an extra trip through HBM.
// All global accesses are 16-byte (or 8-byte for bf16) vectors when the row width allows it
// (V = 4), issued for the whole row before the first use so that one memory round trip
// covers a row; V = 1 is the fallback for widths that are not multiples of four.
#include "common.hpp"

namespace dllmc {

namespace {

constexpr int kThreads = 256;
constexpr int kNW = kThreads / kWave;
constexpr int kRegVecs = 4;  // vectors of a row a thread keeps in registers (rows up to 4096 wide)

template <int V> struct Vec { float v[V]; };

// Row of a cache tensor that holds logical row `row`: the row itself in the flat layout, the
// row map's entry in the paged one.
__device__ __forceinline__ size_t cache_row(const int* __restrict__ rmap, int row) {
  return static_cast<size_t>(rmap ? rmap[row] : row);
}
// The same with the layout known at compile time: the kernels of the adaptive step's critical
// path are instantiated twice, so that the flat layout's code carries no trace of the lookup
// (a run-time test in front of a row's loads cost ~0.3 us per launch).
template <bool PG> __device__ __forceinline__ size_t cache_row_t(const int* __restrict__ rmap, int row) {
  return static_cast<size_t>(PG ? rmap[row] : row);
}

template <int V> __device__ __forceinline__ Vec<V> ld_f32(const float* p);
template <> __device__ __forceinline__ Vec<1> ld_f32<1>(const float* p) { return {{*p}}; }
template <> __device__ __forceinline__ Vec<4> ld_f32<4>(const float* p) {
  const float4 t = *reinterpret_cast<const float4*>(p);
  return {{t.x, t.y, t.z, t.w}};
}
template <int V> __device__ __forceinline__ void st_f32(float* p, const Vec<V>& a);
template <> __device__ __forceinline__ void st_f32<1>(float* p, const Vec<1>& a) { *p = a.v[0]; }
template <> __device__ __forceinline__ void st_f32<4>(float* p, const Vec<4>& a) {
  *reinterpret_cast<float4*>(p) = make_float4(a.v[0], a.v[1], a.v[2], a.v[3]);
}

template <typename T, int V> struct IO;
template <> struct IO<float, 1> {
  static __device__ __forceinline__ Vec<1> ld(const float* p) { return {{*p}}; }
  static __device__ __forceinline__ void st(float* p, const Vec<1>& a) { *p = a.v[0]; }
};
template <> struct IO<float, 4> {
  static __device__ __forceinline__ Vec<4> ld(const float* p) { return ld_f32<4>(p); }
  static __device__ __forceinline__ void st(float* p, const Vec<4>& a) { st_f32<4>(p, a); }
};
template <> struct IO<bf16_t, 1> {
  static __device__ __forceinline__ Vec<1> ld(const bf16_t* p) { return {{bf16_to_f32(*p)}}; }
  static __device__ __forceinline__ void st(bf16_t* p, const Vec<1>& a) { *p = f32_to_bf16(a.v[0]); }
};
template <> struct IO<bf16_t, 4> {
  static __device__ __forceinline__ Vec<4> ld(const bf16_t* p) {
    const uint2 t = *reinterpret_cast<const uint2*>(p);
    return {{__uint_as_float(t.x << 16), __uint_as_float(t.x & 0xffff0000u),
             __uint_as_float(t.y << 16), __uint_as_float(t.y & 0xffff0000u)}};
  }
  static __device__ __forceinline__ void st(bf16_t* p, const Vec<4>& a) {
    uint2 t;
    t.x = static_cast<uint32_t>(f32_to_bf16(a.v[0])) | (static_cast<uint32_t>(f32_to_bf16(a.v[1])) << 16);
    t.y = static_cast<uint32_t>(f32_to_bf16(a.v[2])) | (static_cast<uint32_t>(f32_to_bf16(a.v[3])) << 16);
    *reinterpret_cast<uint2*>(p) = t;
  }
};

// The slice count is a runtime value, but a loop over it (or a load guarded by a per-lane bounds
// test) makes the compiler wait for every load before it issues the next one, and a row kernel
// then spends its time in a chain of memory round trips.  So the count is dispatched to a
// compile-time constant, every load of a row is issued unconditionally (columns past the end
// are clamped to the last valid vector and their values ignored) and only then consumed.
static_assert(kMaxSlices == 8, "DLLMC_SWITCH_SLICES enumerates 1 .. 8 slices");

#define DLLMC_SWITCH_SLICES(S, NS, ...)                   \
  switch (S) {                                            \
    case 1: { constexpr int NS = 1; __VA_ARGS__; } break; \
    case 2: { constexpr int NS = 2; __VA_ARGS__; } break; \
    case 3: { constexpr int NS = 3; __VA_ARGS__; } break; \
    case 4: { constexpr int NS = 4; __VA_ARGS__; } break; \
    case 5: { constexpr int NS = 5; __VA_ARGS__; } break; \
    case 6: { constexpr int NS = 6; __VA_ARGS__; } break; \
    case 7: { constexpr int NS = 7; __VA_ARGS__; } break; \
    default: { constexpr int NS = 8; __VA_ARGS__; } break; \
  }

// column of vector `it` of this thread inside the chunk starting at c0
template <int V> __device__ __forceinline__ int chunk_col(int c0, int it) {
  return c0 + (it * kThreads + static_cast<int>(threadIdx.x)) * V;
}
// same, clamped so that a load from it stays inside a row of `width` columns
template <int V> __device__ __forceinline__ int chunk_col_clamped(int c0, int it, int width) {
  return min(chunk_col<V>(c0, it), width - V);
}

// sums of NS slices at two positions, in slice order
template <int NS>
__device__ __forceinline__ float2 sum_slices_pair(const float* __restrict__ c_part, size_t stride,
                                                  size_t off_a, size_t off_b) {
  float a[NS], b[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    a[s] = c_part[static_cast<size_t>(s) * stride + off_a];
    b[s] = c_part[static_cast<size_t>(s) * stride + off_b];
  }
  float2 r = make_float2(a[0], b[0]);
#pragma unroll
  for (int s = 1; s < NS; ++s) { r.x += a[s]; r.y += b[s]; }
  return r;
}

// Slice sums for the kRegVecs vectors of this thread inside the chunk starting at column c0.
// The additions keep slice order.
template <int V, int NS>
__device__ __forceinline__ void sum_slices_fixed(const float* __restrict__ c_part, size_t stride,
                                                 size_t row_off, int c0, int width,
                                                 Vec<V> (&out)[kRegVecs]) {
  Vec<V> u[NS][kRegVecs];
#pragma unroll
  for (int s = 0; s < NS; ++s)
#pragma unroll
    for (int it = 0; it < kRegVecs; ++it)
      u[s][it] = ld_f32<V>(c_part + static_cast<size_t>(s) * stride + row_off +
                           chunk_col_clamped<V>(c0, it, width));
#pragma unroll
  for (int it = 0; it < kRegVecs; ++it) {
    out[it] = u[0][it];
#pragma unroll
    for (int s = 1; s < NS; ++s)
#pragma unroll
      for (int e = 0; e < V; ++e) out[it].v[e] += u[s][it].v[e];
  }
}
template <int V>
__device__ __forceinline__ void sum_slices_chunk(const float* __restrict__ c_part, int S,
                                                 size_t stride, size_t row_off, int c0, int width,
                                                 Vec<V> (&out)[kRegVecs]) {
  DLLMC_SWITCH_SLICES(S, NS, sum_slices_fixed<V, NS>(c_part, stride, row_off, c0, width, out))
}
constexpr int kChunk(int V) { return kRegVecs * kThreads * V; }

// Second pass of a row: out = x * rstd * gain (or x itself when gain is null), rounded to T,
// to `dst` and optionally `dst2`.  The first chunk comes from registers (`keep`, `gk`); wider
// rows re-read the float32 row this thread stored itself.
template <typename T, int V>
__device__ __forceinline__ void norm_store(const Vec<V> (&keep)[kRegVecs], const Vec<V>* gk,
                                           const float* __restrict__ xr,
                                           const T* __restrict__ gain, float rstd, int d,
                                           T* __restrict__ dst, T* __restrict__ dst2) {
#pragma unroll
  for (int it = 0; it < kRegVecs; ++it) {
    const int c = chunk_col<V>(0, it);
    if (c < d) {
      Vec<V> xv = keep[it];
      if (gain != nullptr) {
#pragma unroll
        for (int e = 0; e < V; ++e) xv.v[e] = xv.v[e] * rstd * gk[it].v[e];
      }
      IO<T, V>::st(dst + c, xv);
      if (dst2) IO<T, V>::st(dst2 + c, xv);
    }
  }
  for (int c = kChunk(V) + static_cast<int>(threadIdx.x) * V; c < d; c += kThreads * V) {
    Vec<V> xv = ld_f32<V>(xr + c);
    if (gain != nullptr) {
      const Vec<V> g = IO<T, V>::ld(gain + c);
#pragma unroll
      for (int e = 0; e < V; ++e) xv.v[e] = xv.v[e] * rstd * g.v[e];
    }
    IO<T, V>::st(dst + c, xv);
    if (dst2) IO<T, V>::st(dst2 + c, xv);
  }
}

// ---- prologue: residual stream from the embedded tokens, first attention norm ----------
template <typename T, int V>
__global__ __launch_bounds__(kThreads) void k_embed_norm(const T* __restrict__ hidden_in,
                                                         const int* __restrict__ rows, int d,
                                                         float eps, const T* __restrict__ gain,
                                                         float* __restrict__ x, T* __restrict__ h) {
  __shared__ float red[kNW];
  const int row = rows[blockIdx.x];
  const T* src = hidden_in + static_cast<size_t>(row) * d;
  float* xr = x + static_cast<size_t>(row) * d;
  T* hr = h + static_cast<size_t>(row) * d;
  float ss = 0.f;
  for (int c = threadIdx.x * V; c < d; c += kThreads * V) {
    const Vec<V> a = IO<T, V>::ld(src + c);
    st_f32<V>(xr + c, a);
#pragma unroll
    for (int e = 0; e < V; ++e) ss += a.v[e] * a.v[e];
  }
  ss = block_sum<kNW>(ss, red);
  const float rstd = 1.0f / sqrtf(ss / static_cast<float>(d) + eps);
  for (int c = threadIdx.x * V; c < d; c += kThreads * V) {
    Vec<V> a = ld_f32<V>(xr + c);  // this thread's own stores
    const Vec<V> g = IO<T, V>::ld(gain + c);
#pragma unroll
    for (int e = 0; e < V; ++e) a.v[e] = a.v[e] * rstd * g.v[e];
    IO<T, V>::st(hr + c, a);
  }
}

// ---- V-verify epilogue: round V_new, score it against the cached row (metric 0: cosine of
// Eq. (cos_sim); 1: minus the Euclidean distance, the paper's L2 variant), overwrite the cache --
template <typename T, int V>
__global__ __launch_bounds__(kThreads) void k_v_finalize(const float* __restrict__ c_part, int S,
                                                         size_t slice_stride, int first,
                                                         int per_seq, int d_kv, int n, int L_p,
                                                         T* __restrict__ v_cache,
                                                         float* __restrict__ score, int metric,
                                                         T* __restrict__ v_stage,
                                                         const int* __restrict__ rmap) {
  __shared__ float red[kNW];
  const int i = blockIdx.x;
  // carried rows are positions first .. first + per_seq - 1 of every sequence (per_seq = 0: row i):
  // computed, not looked up, so the cached row's loads go out together with the slices'
  const int row = per_seq > 0 ? (i / per_seq) * n + first + i % per_seq : i;
  T* vc = v_cache + cache_row(rmap, row) * d_kv;
  const int pos = row % n;
  const bool scored = (score != nullptr) && (pos >= L_p);
  // selected-only update: response rows are parked in v_stage[i] until the selection is known
  T* vdst = (v_stage != nullptr && pos >= L_p) ? v_stage + static_cast<size_t>(i) * d_kv : vc;
  float dot = 0.f, nn = 0.f, no = 0.f;  // metric 1 (distance): dot holds sum (v - o)^2
  for (int c0 = 0; c0 < d_kv; c0 += kChunk(V)) {
    Vec<V> v[kRegVecs], o[kRegVecs];
    if (scored) {
#pragma unroll
      for (int it = 0; it < kRegVecs; ++it) o[it] = IO<T, V>::ld(vc + chunk_col_clamped<V>(c0, it, d_kv));
    }
    sum_slices_chunk<V>(c_part, S, slice_stride, static_cast<size_t>(i) * d_kv, c0, d_kv, v);
#pragma unroll
    for (int it = 0; it < kRegVecs; ++it) {
      const int c = chunk_col<V>(c0, it);
      if (c < d_kv) {
#pragma unroll
        for (int e = 0; e < V; ++e) v[it].v[e] = roundf_to<T>(v[it].v[e]);
        if (scored) {
          if (metric == 0) {
#pragma unroll
            for (int e = 0; e < V; ++e) {
              dot += v[it].v[e] * o[it].v[e];
              nn += v[it].v[e] * v[it].v[e];
              no += o[it].v[e] * o[it].v[e];
            }
          } else {
#pragma unroll
            for (int e = 0; e < V; ++e) {
              const float df = v[it].v[e] - o[it].v[e];
              dot += df * df;
            }
          }
        }
        IO<T, V>::st(vdst + c, v[it]);
      }
    }
  }
  if (scored) {
    dot = block_sum<kNW>(dot, red);
    nn = block_sum<kNW>(nn, red);
    no = block_sum<kNW>(no, red);
    if (threadIdx.x == 0) {
      const int seq = row / n;
      const int L_r = n - L_p;
      score[static_cast<size_t>(seq) * L_r + (pos - L_p)] =
          metric == 0 ? dot / fmaxf(sqrtf(nn) * sqrtf(no), 1e-8f) : -sqrtf(dot);
    }
  }
}

// ---- Q/K epilogue: RoPE at the row's absolute position, Q to the compact buffer, K scatter --
// grid (rows, query heads + kv heads), one wavefront per (row, head), one lane per pair.
template <typename T, bool PG>
__global__ __launch_bounds__(64) void k_qk_finalize(const float* __restrict__ c_part, int S,
                                                    size_t slice_stride,
                                                    const int* __restrict__ rows, int n, int d_q,
                                                    int d_kv, int d_h,
                                                    const float2* __restrict__ rope_tab,
                                                    T* __restrict__ q_out, T* __restrict__ k_cache,
                                                    int rope_second, const int* __restrict__ rmap) {
  const int i = blockIdx.x, head = blockIdx.y;
  const int row = rows[i];
  const int pos = row % n;
  const int half = d_h / 2;
  const int width = d_q + d_kv;
  const float2* tab = rope_tab + static_cast<size_t>(pos) * half;
  const int c0 = head * d_h;  // first column of the head inside [Q | K]
  T* dst = c0 < d_q ? q_out + static_cast<size_t>(i) * d_q + c0
                    : k_cache + cache_row_t<PG>(rmap, row) * d_kv + (c0 - d_q);
  for (int t = threadIdx.x; t < half; t += 64) {
    const size_t off = static_cast<size_t>(i) * width + c0 + t;
    float2 ab;
    DLLMC_SWITCH_SLICES(S, NS, ab = sum_slices_pair<NS>(c_part, slice_stride, off, off + half))
    // the second matrix is W_k (rotated) or, for K-verify, W_v (stored as it is)
    const float2 cs = (c0 < d_q || rope_second) ? tab[t] : make_float2(1.f, 0.f);
    stf(dst + t, ab.x * cs.x - ab.y * cs.y);
    stf(dst + t + half, ab.y * cs.x + ab.x * cs.y);
  }
}

// ---- K-verify epilogue: RoPE at the row's position, round, score against the cached Key row
// (metric as in k_v_finalize), overwrite the cache (or park response rows in k_stage) -------
// One workgroup per row; a thread handles the rotation pairs (t, t + d_h/2) p = tid, tid+256, ...
template <typename T>
__global__ __launch_bounds__(kThreads) void k_k_finalize(const float* __restrict__ c_part, int S,
                                                         size_t slice_stride,
                                                         const int* __restrict__ rows, int d_kv,
                                                         int d_h, int n, int L_p,
                                                         const float2* __restrict__ rope_tab,
                                                         T* __restrict__ k_cache,
                                                         float* __restrict__ score, int metric,
                                                         T* __restrict__ k_stage,
                                                         const int* __restrict__ rmap) {
  __shared__ float red[kNW];
  const int i = blockIdx.x;
  const int row = rows ? rows[i] : i;
  const int pos = row % n;
  const int half = d_h / 2;
  T* kc = k_cache + cache_row(rmap, row) * d_kv;
  T* kdst = (k_stage != nullptr && pos >= L_p) ? k_stage + static_cast<size_t>(i) * d_kv : kc;
  const bool scored = (score != nullptr) && (pos >= L_p);
  const float2* tab = rope_tab + static_cast<size_t>(pos) * half;
  float dot = 0.f, nn = 0.f, no = 0.f;
  for (int p = threadIdx.x; p < d_kv / 2; p += kThreads) {
    const int t = p % half, c = (p / half) * d_h + t;  // columns c and c + half of the row
    const size_t off = static_cast<size_t>(i) * d_kv + c;
    float2 ab;
    DLLMC_SWITCH_SLICES(S, NS, ab = sum_slices_pair<NS>(c_part, slice_stride, off, off + half))
    const float2 cs = tab[t];
    const float v0 = roundf_to<T>(ab.x * cs.x - ab.y * cs.y);
    const float v1 = roundf_to<T>(ab.y * cs.x + ab.x * cs.y);
    if (scored) {
      const float o0 = ldf(kc + c), o1 = ldf(kc + c + half);
      if (metric == 0) {
        dot += v0 * o0 + v1 * o1;
        nn += v0 * v0 + v1 * v1;
        no += o0 * o0 + o1 * o1;
      } else {
        dot += (v0 - o0) * (v0 - o0) + (v1 - o1) * (v1 - o1);
      }
    }
    stf(kdst + c, v0);
    stf(kdst + c + half, v1);
  }
  if (scored) {
    dot = block_sum<kNW>(dot, red);
    nn = block_sum<kNW>(nn, red);
    no = block_sum<kNW>(no, red);
    if (threadIdx.x == 0)
      score[static_cast<size_t>(row / n) * (n - L_p) + (pos - L_p)] =
          metric == 0 ? dot / fmaxf(sqrtf(nn) * sqrtf(no), 1e-8f) : -sqrtf(dot);
  }
}

// ---- output projection epilogue + residual + FFN norm ------------------------------------
// One workgroup per recomputed row.  Rows that are carried but not recomputed are left alone:
// their residual add of the cached attention output happens in k_down_finalize, in the same
// order of additions, so the stream x of such a row is read and written once per layer.
template <typename T, int V, bool PG>
__global__ __launch_bounds__(kThreads) void k_o_finalize(const float* __restrict__ c_part, int S,
                                                         size_t slice_stride,
                                                         const int* __restrict__ rows_R, int d,
                                                         float eps, T* __restrict__ attn_cache,
                                                         float* __restrict__ x,
                                                         const T* __restrict__ gain,
                                                         T* __restrict__ g_out,
                                                         const int* __restrict__ rmap) {
  __shared__ float red[kNW];
  const int ci = blockIdx.x;
  const int row = rows_R[ci];
  T* ac = attn_cache + cache_row_t<PG>(rmap, row) * d;
  float* xr = x + static_cast<size_t>(row) * d;
  Vec<V> keep[kRegVecs];
  float ss = 0.f;
  for (int c0 = 0; c0 < d; c0 += kChunk(V)) {
    Vec<V> a[kRegVecs], xv[kRegVecs];
    sum_slices_chunk<V>(c_part, S, slice_stride, static_cast<size_t>(ci) * d, c0, d, a);
#pragma unroll
    for (int it = 0; it < kRegVecs; ++it) xv[it] = ld_f32<V>(xr + chunk_col_clamped<V>(c0, it, d));
#pragma unroll
    for (int it = 0; it < kRegVecs; ++it) {
      const int c = chunk_col<V>(c0, it);
      if (c < d) {
#pragma unroll
        for (int e = 0; e < V; ++e) a[it].v[e] = roundf_to<T>(a[it].v[e]);
        IO<T, V>::st(ac + c, a[it]);
#pragma unroll
        for (int e = 0; e < V; ++e) {
          xv[it].v[e] += a[it].v[e];
          ss += xv[it].v[e] * xv[it].v[e];
        }
        st_f32<V>(xr + c, xv[it]);
        if (c0 == 0) keep[it] = xv[it];
      }
    }
  }
  // gain vectors of the first chunk: issued before the reduction so they arrive under it
  Vec<V> gk[kRegVecs];
#pragma unroll
  for (int it = 0; it < kRegVecs; ++it) gk[it] = IO<T, V>::ld(gain + chunk_col_clamped<V>(0, it, d));
  ss = block_sum<kNW>(ss, red);
  const float rstd = 1.0f / sqrtf(ss / static_cast<float>(d) + eps);
  T* gr = g_out + static_cast<size_t>(ci) * d;
  norm_store<T, V>(keep, gk, xr, gain, rstd, d, gr, nullptr);
}

// ---- SwiGLU product (only when the fused gate/up kernel does not apply) -------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void k_swiglu(const float* __restrict__ c_part, int S,
                                                     size_t slice_stride, int m,
                                                     T* __restrict__ u) {
  // rows on grid.x (up to 2^31 - 1 of them), column blocks on grid.y
  const int i = blockIdx.x;
  const int j = blockIdx.y * kThreads + threadIdx.x;
  if (j >= m) return;
  const size_t off = static_cast<size_t>(i) * 2 * m + j;
  float2 gu;
  DLLMC_SWITCH_SLICES(S, NS, gu = sum_slices_pair<NS>(c_part, slice_stride, off, off + m))
  stf(u + static_cast<size_t>(i) * m + j, gu.x / (1.0f + expf(-gu.x)) * gu.y);
}

// ---- down projection epilogue + residual + next layer's attention norm / step output ------
template <typename T, int V, bool PG>
__global__ __launch_bounds__(kThreads) void k_down_finalize(
    const float* __restrict__ c_part, int S, size_t slice_stride, int first, int per_seq,
    const int* __restrict__ inv, int d, int n, int L_p, float eps,
    const T* __restrict__ attn_cache, T* __restrict__ ffn_cache, float* __restrict__ x,
    const T* __restrict__ next_gain, T* __restrict__ h, T* __restrict__ hidden_out,
    T* __restrict__ prompt_out, const int* __restrict__ rmap) {
  __shared__ float red[kNW];
  // carried rows are positions first .. first + per_seq - 1 of every sequence: computed, so that
  // the row's loads do not wait for a list entry
  const int i = blockIdx.x;
  const int row = (i / per_seq) * n + first + i % per_seq;
  const size_t crow = cache_row_t<PG>(rmap, row);
  T* fc = ffn_cache + crow * d;
  const T* ac = attn_cache + crow * d;
  float* xr = x + static_cast<size_t>(row) * d;
  Vec<V> keep[kRegVecs];
  float ss = 0.f;
  for (int c0 = 0; c0 < d; c0 += kChunk(V)) {
    // the stream and both cached rows are fetched before the row is known to be recomputed or
    // not (one round trip for a row that is not; a recomputed one drops the cached values and
    // fetches its slices in a second trip)
    Vec<V> f[kRegVecs], a[kRegVecs], xv[kRegVecs];
#pragma unroll
    for (int it = 0; it < kRegVecs; ++it) {
      const int c = chunk_col_clamped<V>(c0, it, d);
      xv[it] = ld_f32<V>(xr + c);
      f[it] = IO<T, V>::ld(fc + c);
      a[it] = IO<T, V>::ld(ac + c);
    }
    const int ci = inv[row];
    if (ci >= 0) {
      sum_slices_chunk<V>(c_part, S, slice_stride, static_cast<size_t>(ci) * d, c0, d, f);
    } else {
      // a row that was not recomputed: the attention residual add that k_o_finalize left out
      // comes first, then the FFN one below, as for a recomputed row
#pragma unroll
      for (int it = 0; it < kRegVecs; ++it)
#pragma unroll
        for (int e = 0; e < V; ++e) xv[it].v[e] += a[it].v[e];
    }
#pragma unroll
    for (int it = 0; it < kRegVecs; ++it) {
      const int c = chunk_col<V>(c0, it);
      if (c < d) {
        if (ci >= 0) {
#pragma unroll
          for (int e = 0; e < V; ++e) f[it].v[e] = roundf_to<T>(f[it].v[e]);
          IO<T, V>::st(fc + c, f[it]);
        }
#pragma unroll
        for (int e = 0; e < V; ++e) {
          xv[it].v[e] += f[it].v[e];
          ss += xv[it].v[e] * xv[it].v[e];
        }
        st_f32<V>(xr + c, xv[it]);
        if (c0 == 0) keep[it] = xv[it];
      }
    }
  }
  if (next_gain != nullptr) {
    Vec<V> gk[kRegVecs];
#pragma unroll
    for (int it = 0; it < kRegVecs; ++it) gk[it] = IO<T, V>::ld(next_gain + chunk_col_clamped<V>(0, it, d));
    ss = block_sum<kNW>(ss, red);
    const float rstd = 1.0f / sqrtf(ss / static_cast<float>(d) + eps);
    norm_store<T, V>(keep, gk, xr, next_gain, rstd, d, h + static_cast<size_t>(row) * d, nullptr);
  } else {
    T* o = hidden_out + static_cast<size_t>(row) * d;
    const int pos = row % n;
    T* po = (prompt_out != nullptr && pos < L_p)
                ? prompt_out + (static_cast<size_t>(row / n) * L_p + pos) * d
                : nullptr;
    norm_store<T, V>(keep, nullptr, xr, nullptr, 1.0f, d, o, po);
  }
}

// Selected-only V update: v_cache[row] = v_stage[carried index of row] for the recomputed
// response rows (prompt rows were written directly).  Carried rows of a sequence are the
// positions first .. n-1, carried_per_seq of them.
template <typename T>
__global__ __launch_bounds__(kThreads) void k_scatter_v(const int* __restrict__ rows_R, int n,
                                                        int L_p, int first, int carried_per_seq,
                                                        int d_kv, const T* __restrict__ v_stage,
                                                        T* __restrict__ v_cache,
                                                        const int* __restrict__ rmap) {
  const int row = rows_R[blockIdx.x];
  const int pos = row % n;
  if (pos < L_p) return;  // uniform over the workgroup
  const size_t i = static_cast<size_t>(row / n) * carried_per_seq + (pos - first);
  const T* src = v_stage + i * d_kv;
  T* dst = v_cache + cache_row(rmap, row) * d_kv;
  for (int c = threadIdx.x; c < d_kv; c += kThreads) dst[c] = src[c];
}

template <typename T>
__global__ __launch_bounds__(kThreads) void k_copy_prompt(const T* __restrict__ prompt_out, int n,
                                                          int L_p, int d,
                                                          T* __restrict__ hidden_out) {
  const int b = blockIdx.y, t = blockIdx.x;
  const T* s = prompt_out + (static_cast<size_t>(b) * L_p + t) * d;
  T* o = hidden_out + (static_cast<size_t>(b) * n + t) * d;
  for (int c = threadIdx.x; c < d; c += kThreads) o[c] = s[c];
}

// out[row][:] = cache[rmap[row]][:]: a cache tensor in logical row order
template <typename T>
__global__ __launch_bounds__(kThreads) void k_gather_rows(const T* __restrict__ cache,
                                                          const int* __restrict__ rmap, int width,
                                                          T* __restrict__ out) {
  const int row = blockIdx.x;
  const T* s = cache + cache_row(rmap, row) * width;
  T* o = out + static_cast<size_t>(row) * width;
  for (int c = threadIdx.x; c < width; c += kThreads) o[c] = s[c];
}

__global__ void k_iota_rows(int* rows, int* inv, int n, int first, int count, int per_seq,
                            int off) {
  const int b = blockIdx.y;
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= count) return;
  const int ci = b * per_seq + off + t;
  const int row = b * n + first + t;
  if (rows) rows[ci] = row;
  if (inv) inv[row] = ci;
}

__global__ void k_fill_i32(int* p, int value, size_t count) {
  const size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i < count) p[i] = value;
}

__global__ void k_fill_sel_identity(int* sel, int L_r) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < L_r) sel[static_cast<size_t>(blockIdx.y) * L_r + j] = j;
}

template <typename T> inline T* P(void* p) { return static_cast<T*>(p); }
template <typename T> inline const T* P(const void* p) { return static_cast<const T*>(p); }

inline bool vec_ok(int width, std::initializer_list<const void*> ptrs) {
  if (width % 4) return false;
  for (const void* p : ptrs)
    if (p && (reinterpret_cast<uintptr_t>(p) & 15u)) return false;
  return true;
}

}  // namespace

// launch KERNEL<T, 4> or KERNEL<T, 1> depending on whether 16-byte vectors apply
// the same for kernels with the paged-layout switch as a third template argument
#define DLLMC_ROW_LAUNCH_PG(KERNEL, T, vec, pg, grid, st, ...)                                       \
  do {                                                                                               \
    if (vec && pg) hipLaunchKernelGGL((KERNEL<T, 4, true>), grid, dim3(kThreads), 0, st, __VA_ARGS__);      \
    else if (vec) hipLaunchKernelGGL((KERNEL<T, 4, false>), grid, dim3(kThreads), 0, st, __VA_ARGS__);      \
    else if (pg) hipLaunchKernelGGL((KERNEL<T, 1, true>), grid, dim3(kThreads), 0, st, __VA_ARGS__);        \
    else hipLaunchKernelGGL((KERNEL<T, 1, false>), grid, dim3(kThreads), 0, st, __VA_ARGS__);               \
  } while (0)

#define DLLMC_ROW_LAUNCH(KERNEL, T, vec, grid, st, ...)                                      \
  do {                                                                                       \
    if (vec) hipLaunchKernelGGL((KERNEL<T, 4>), grid, dim3(kThreads), 0, st, __VA_ARGS__);    \
    else hipLaunchKernelGGL((KERNEL<T, 1>), grid, dim3(kThreads), 0, st, __VA_ARGS__);        \
  } while (0)

void launch_embed_norm(const RowKernelArgs& a, const void* hidden_in, const int* rows, int M,
                       const void* gain, float* x, void* h, hipStream_t st) {
  if (M <= 0) return;
  const bool vec = vec_ok(a.d, {hidden_in, gain, x, h});
  if (a.dtype == 1) {
    DLLMC_ROW_LAUNCH(k_embed_norm, bf16_t, vec, dim3(M), st, P<bf16_t>(hidden_in), rows, a.d, a.eps,
                     P<bf16_t>(gain), x, P<bf16_t>(h));
  } else {
    DLLMC_ROW_LAUNCH(k_embed_norm, float, vec, dim3(M), st, P<float>(hidden_in), rows, a.d, a.eps,
                     P<float>(gain), x, P<float>(h));
  }
}

void launch_v_finalize(const RowKernelArgs& a, const float* c_part, int S, int first, int per_seq,
                       int M, int d_kv, void* v_cache, float* score, int metric, void* v_stage,
                       hipStream_t st, const int* rmap) {
  if (M <= 0) return;
  const size_t stride = static_cast<size_t>(M) * d_kv;
  const bool vec = vec_ok(d_kv, {c_part, v_cache, v_stage});
  if (a.dtype == 1) {
    DLLMC_ROW_LAUNCH(k_v_finalize, bf16_t, vec, dim3(M), st, c_part, S, stride, first, per_seq, d_kv, a.n, a.L_p,
                     P<bf16_t>(v_cache), score, metric, P<bf16_t>(v_stage), rmap);
  } else {
    DLLMC_ROW_LAUNCH(k_v_finalize, float, vec, dim3(M), st, c_part, S, stride, first, per_seq, d_kv, a.n, a.L_p,
                     P<float>(v_cache), score, metric, P<float>(v_stage), rmap);
  }
}

void launch_scatter_v(const RowKernelArgs& a, const int* rows_R, int M_R, int first,
                      int carried_per_seq, int d_kv, const void* v_stage, void* v_cache,
                      hipStream_t st, const int* rmap) {
  if (M_R <= 0) return;
  if (a.dtype == 1)
    hipLaunchKernelGGL(k_scatter_v<bf16_t>, dim3(M_R), dim3(kThreads), 0, st, rows_R, a.n, a.L_p, first,
                       carried_per_seq, d_kv, P<bf16_t>(v_stage), P<bf16_t>(v_cache), rmap);
  else
    hipLaunchKernelGGL(k_scatter_v<float>, dim3(M_R), dim3(kThreads), 0, st, rows_R, a.n, a.L_p, first,
                       carried_per_seq, d_kv, P<float>(v_stage), P<float>(v_cache), rmap);
}

void launch_qk_finalize(const RowKernelArgs& a, const float* c_part, int S, const int* rows, int M,
                        int d_q, int d_kv, int d_h, const float2* rope_tab, void* q_out,
                        void* k_cache, bool rope_second, hipStream_t st, const int* rmap) {
  if (M <= 0) return;
  const size_t stride = static_cast<size_t>(M) * (d_q + d_kv);
  const dim3 grid(M, (d_q + d_kv) / d_h);
#define DLLMC_QK(T, PG)                                                                           \
  hipLaunchKernelGGL((k_qk_finalize<T, PG>), grid, dim3(64), 0, st, c_part, S, stride, rows, a.n, d_q, \
                     d_kv, d_h, rope_tab, P<T>(q_out), P<T>(k_cache), rope_second ? 1 : 0, rmap)
  if (a.dtype == 1 && rmap) DLLMC_QK(bf16_t, true);
  else if (a.dtype == 1) DLLMC_QK(bf16_t, false);
  else if (rmap) DLLMC_QK(float, true);
  else DLLMC_QK(float, false);
#undef DLLMC_QK
}

void launch_k_finalize(const RowKernelArgs& a, const float* c_part, int S, const int* rows, int M,
                       int d_kv, int d_h, const float2* rope_tab, void* k_cache, float* score,
                       int metric, void* k_stage, hipStream_t st, const int* rmap) {
  if (M <= 0) return;
  const size_t stride = static_cast<size_t>(M) * d_kv;
  if (a.dtype == 1)
    hipLaunchKernelGGL(k_k_finalize<bf16_t>, dim3(M), dim3(kThreads), 0, st, c_part, S, stride, rows,
                       d_kv, d_h, a.n, a.L_p, rope_tab, P<bf16_t>(k_cache), score, metric,
                       P<bf16_t>(k_stage), rmap);
  else
    hipLaunchKernelGGL(k_k_finalize<float>, dim3(M), dim3(kThreads), 0, st, c_part, S, stride, rows,
                       d_kv, d_h, a.n, a.L_p, rope_tab, P<float>(k_cache), score, metric,
                       P<float>(k_stage), rmap);
}

void launch_o_finalize(const RowKernelArgs& a, const float* c_part, int S, const int* rows_R,
                       int M_R, void* attn_cache, float* x, const void* gain, void* g_out,
                       hipStream_t st, const int* rmap) {
  if (M_R <= 0) return;
  const size_t stride = static_cast<size_t>(M_R) * a.d;
  const bool vec = vec_ok(a.d, {c_part, attn_cache, x, gain, g_out});
  if (a.dtype == 1) {
    DLLMC_ROW_LAUNCH_PG(k_o_finalize, bf16_t, vec, rmap != nullptr, dim3(M_R), st, c_part, S, stride, rows_R, a.d, a.eps,
                     P<bf16_t>(attn_cache), x, P<bf16_t>(gain), P<bf16_t>(g_out), rmap);
  } else {
    DLLMC_ROW_LAUNCH_PG(k_o_finalize, float, vec, rmap != nullptr, dim3(M_R), st, c_part, S, stride, rows_R, a.d, a.eps,
                     P<float>(attn_cache), x, P<float>(gain), P<float>(g_out), rmap);
  }
}

void launch_swiglu(int dtype, const float* c_part, int S, int M, int m, void* u, hipStream_t st) {
  if (M <= 0) return;
  const size_t stride = static_cast<size_t>(M) * 2 * m;
  const dim3 grid(M, (m + kThreads - 1) / kThreads);
  if (dtype == 1)
    hipLaunchKernelGGL(k_swiglu<bf16_t>, grid, dim3(kThreads), 0, st, c_part, S, stride, m,
                       P<bf16_t>(u));
  else
    hipLaunchKernelGGL(k_swiglu<float>, grid, dim3(kThreads), 0, st, c_part, S, stride, m,
                       P<float>(u));
}

void launch_down_finalize(const RowKernelArgs& a, const float* c_part, int S, int M_R,
                          int first, int per_seq, int Mc, const int* inv, const void* attn_cache,
                          void* ffn_cache, float* x, const void* next_gain, void* h,
                          void* hidden_out, void* prompt_out, hipStream_t st, const int* rmap) {
  if (Mc <= 0) return;
  const size_t stride = static_cast<size_t>(M_R) * a.d;
  const bool vec =
      vec_ok(a.d, {c_part, attn_cache, ffn_cache, x, next_gain, h, hidden_out, prompt_out});
  if (a.dtype == 1) {
    DLLMC_ROW_LAUNCH_PG(k_down_finalize, bf16_t, vec, rmap != nullptr, dim3(Mc), st, c_part, S, stride, first, per_seq, inv, a.d,
                     a.n, a.L_p, a.eps, P<bf16_t>(attn_cache), P<bf16_t>(ffn_cache), x, P<bf16_t>(next_gain), P<bf16_t>(h),
                     P<bf16_t>(hidden_out), P<bf16_t>(prompt_out), rmap);
  } else {
    DLLMC_ROW_LAUNCH_PG(k_down_finalize, float, vec, rmap != nullptr, dim3(Mc), st, c_part, S, stride, first, per_seq, inv, a.d,
                     a.n, a.L_p, a.eps, P<float>(attn_cache), P<float>(ffn_cache), x, P<float>(next_gain), P<float>(h),
                     P<float>(hidden_out), P<float>(prompt_out), rmap);
  }
}

void launch_copy_prompt(const RowKernelArgs& a, int B, const void* prompt_out, void* hidden_out,
                        hipStream_t st) {
  if (a.L_p <= 0 || B <= 0) return;
  const dim3 grid(a.L_p, B);
  if (a.dtype == 1)
    hipLaunchKernelGGL(k_copy_prompt<bf16_t>, grid, dim3(kThreads), 0, st, P<bf16_t>(prompt_out),
                       a.n, a.L_p, a.d, P<bf16_t>(hidden_out));
  else
    hipLaunchKernelGGL(k_copy_prompt<float>, grid, dim3(kThreads), 0, st, P<float>(prompt_out), a.n,
                       a.L_p, a.d, P<float>(hidden_out));
}

void launch_gather_rows(int dtype, const void* cache, const int* rmap, int rows, int width,
                        void* out, hipStream_t st) {
  if (rows <= 0) return;
  if (dtype == 1)
    hipLaunchKernelGGL(k_gather_rows<bf16_t>, dim3(rows), dim3(kThreads), 0, st, P<bf16_t>(cache), rmap,
                       width, P<bf16_t>(out));
  else
    hipLaunchKernelGGL(k_gather_rows<float>, dim3(rows), dim3(kThreads), 0, st, P<float>(cache), rmap,
                       width, P<float>(out));
}

void launch_iota_rows(int* rows, int* inv, int B, int n, int first, int count, int per_seq,
                      int off, hipStream_t st) {
  if (count <= 0 || B <= 0) return;
  hipLaunchKernelGGL(k_iota_rows, dim3((count + 255) / 256, B), dim3(256), 0, st, rows, inv, n,
                     first, count, per_seq, off);
}

void launch_fill_i32(int* p, int value, size_t count, hipStream_t st) {
  if (count == 0) return;
  hipLaunchKernelGGL(k_fill_i32, dim3(static_cast<unsigned>((count + 255) / 256)), dim3(256), 0, st,
                     p, value, count);
}

void launch_fill_sel_identity(int* sel, int layers_times_B, int L_r, hipStream_t st) {
  if (layers_times_B <= 0 || L_r <= 0) return;
  hipLaunchKernelGGL(k_fill_sel_identity, dim3((L_r + 255) / 256, layers_times_B), dim3(256), 0, st,
                     sel, L_r);
}

}  // namespace dllmc
