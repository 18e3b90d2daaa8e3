// Row kernels: everything of the step that is not a matrix product or attention.
// One workgroup of 256 threads handles one token row end to end, so the row-wide
// reductions (RMSNorm mean square, cosine dot product and norms) stay inside a workgroup:
// wavefront shuffles first, then a fixed-order sum over the four wavefronts.  They also
// add up the float32 slices the split contraction of the GEMMs leaves behind, round once to
// the storage type, and do the cache scatter, so no value makes an extra trip through HBM.
#include "common.hpp"

namespace dllmc {

namespace {

constexpr int kThreads = 256;
constexpr int kNW = kThreads / kWave;

__device__ __forceinline__ float sum_slices(const float* __restrict__ c_part, int S, size_t stride,
                                            size_t off) {
  float t = c_part[off];
  for (int s = 1; s < S; ++s) t += c_part[static_cast<size_t>(s) * stride + off];
  return t;
}

// ---- prologue: residual stream from the embedded tokens, first attention norm ----------
template <typename T>
__global__ __launch_bounds__(kThreads) void k_embed_norm(const T* __restrict__ hidden_in,
                                                         const int* __restrict__ rows, int d,
                                                         float eps, const T* __restrict__ gain,
                                                         float* __restrict__ x, T* __restrict__ h) {
  __shared__ float red[kNW];
  const int row = rows[blockIdx.x];
  const T* src = hidden_in + static_cast<size_t>(row) * d;
  float* xr = x + static_cast<size_t>(row) * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += kThreads) {
    const float v = ldf(src + c);
    xr[c] = v;
    ss += v * v;
  }
  ss = block_sum<kNW>(ss, red);
  const float rstd = 1.0f / sqrtf(ss / static_cast<float>(d) + eps);
  T* hr = h + static_cast<size_t>(row) * d;
  for (int c = threadIdx.x; c < d; c += kThreads) stf(hr + c, xr[c] * rstd * ldf(gain + c));
}

// ---- V-verify epilogue: round V_new, cosine against the cached row, overwrite the cache --
template <typename T>
__global__ __launch_bounds__(kThreads) void k_v_finalize(const float* __restrict__ c_part, int S,
                                                         size_t slice_stride,
                                                         const int* __restrict__ rows, int d_kv,
                                                         int n, int L_p, T* __restrict__ v_cache,
                                                         float* __restrict__ score) {
  __shared__ float red[kNW];
  const int i = blockIdx.x;
  const int row = rows ? rows[i] : i;
  T* vc = v_cache + static_cast<size_t>(row) * d_kv;
  const int pos = row % n;
  const bool scored = (score != nullptr) && (pos >= L_p);
  float dot = 0.f, nn = 0.f, no = 0.f;
  for (int c = threadIdx.x; c < d_kv; c += kThreads) {
    const float v = roundf_to<T>(sum_slices(c_part, S, slice_stride, static_cast<size_t>(i) * d_kv + c));
    if (scored) {
      const float o = ldf(vc + c);
      dot += v * o;
      nn += v * v;
      no += o * o;
    }
    stf(vc + c, v);
  }
  if (scored) {
    dot = block_sum<kNW>(dot, red);
    nn = block_sum<kNW>(nn, red);
    no = block_sum<kNW>(no, red);
    if (threadIdx.x == 0) {
      const int seq = row / n;
      const int L_r = n - L_p;
      score[static_cast<size_t>(seq) * L_r + (pos - L_p)] =
          dot / fmaxf(sqrtf(nn) * sqrtf(no), 1e-8f);
    }
  }
}

// ---- Q/K epilogue: RoPE at the row's absolute position, Q to the compact buffer, K scatter --
template <typename T>
__global__ __launch_bounds__(kThreads) void k_qk_finalize(const float* __restrict__ c_part, int S,
                                                          size_t slice_stride,
                                                          const int* __restrict__ rows, int n,
                                                          int d_q, int d_kv, int d_h,
                                                          const float2* __restrict__ rope_tab,
                                                          T* __restrict__ q_out,
                                                          T* __restrict__ k_cache) {
  const int i = blockIdx.x;
  const int row = rows[i];
  const int pos = row % n;
  const int half = d_h / 2;
  const int width = d_q + d_kv;
  const float2* tab = rope_tab + static_cast<size_t>(pos) * half;
  T* qr = q_out + static_cast<size_t>(i) * d_q;
  T* kr = k_cache + static_cast<size_t>(row) * d_kv;
  // one thread per rotation pair
  for (int p = threadIdx.x; p < width / 2; p += kThreads) {
    const int head = p / half, t = p - head * half;
    const int c0 = head * d_h + t;  // column of the pair's first element in [Q | K]
    const size_t off = static_cast<size_t>(i) * width + c0;
    const float a = sum_slices(c_part, S, slice_stride, off);
    const float b = sum_slices(c_part, S, slice_stride, off + half);
    const float2 cs = tab[t];
    const float ra = a * cs.x - b * cs.y;
    const float rb = b * cs.x + a * cs.y;
    if (c0 < d_q) {
      stf(qr + c0, ra);
      stf(qr + c0 + half, rb);
    } else {
      stf(kr + (c0 - d_q), ra);
      stf(kr + (c0 - d_q) + half, rb);
    }
  }
}

// ---- output projection epilogue + residual + FFN norm ------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void k_o_finalize(const float* __restrict__ c_part, int S,
                                                         size_t slice_stride,
                                                         const int* __restrict__ carried,
                                                         const int* __restrict__ inv, int d,
                                                         float eps, T* __restrict__ attn_cache,
                                                         float* __restrict__ x,
                                                         const T* __restrict__ gain,
                                                         T* __restrict__ g_out) {
  __shared__ float red[kNW];
  const int row = carried[blockIdx.x];
  const int ci = inv[row];
  T* ac = attn_cache + static_cast<size_t>(row) * d;
  float* xr = x + static_cast<size_t>(row) * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += kThreads) {
    float a;
    if (ci >= 0) {
      a = roundf_to<T>(sum_slices(c_part, S, slice_stride, static_cast<size_t>(ci) * d + c));
      stf(ac + c, a);
    } else {
      a = ldf(ac + c);
    }
    const float v = xr[c] + a;
    xr[c] = v;
    ss += v * v;
  }
  if (ci < 0) return;  // uniform over the workgroup
  ss = block_sum<kNW>(ss, red);
  const float rstd = 1.0f / sqrtf(ss / static_cast<float>(d) + eps);
  T* gr = g_out + static_cast<size_t>(ci) * d;
  for (int c = threadIdx.x; c < d; c += kThreads) stf(gr + c, xr[c] * rstd * ldf(gain + c));
}

// ---- SwiGLU product ---------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void k_swiglu(const float* __restrict__ c_part, int S,
                                                     size_t slice_stride, int m,
                                                     T* __restrict__ u) {
  const int i = blockIdx.y;
  const int j = blockIdx.x * kThreads + threadIdx.x;
  if (j >= m) return;
  const size_t off = static_cast<size_t>(i) * 2 * m + j;
  const float g = sum_slices(c_part, S, slice_stride, off);
  const float up = sum_slices(c_part, S, slice_stride, off + m);
  stf(u + static_cast<size_t>(i) * m + j, g / (1.0f + expf(-g)) * up);
}

// ---- down projection epilogue + residual + next layer's attention norm / step output ------
template <typename T>
__global__ __launch_bounds__(kThreads) void k_down_finalize(
    const float* __restrict__ c_part, int S, size_t slice_stride, const int* __restrict__ carried,
    const int* __restrict__ inv, int d, int n, int L_p, float eps, T* __restrict__ ffn_cache,
    float* __restrict__ x, const T* __restrict__ next_gain, T* __restrict__ h,
    T* __restrict__ hidden_out, T* __restrict__ prompt_out) {
  __shared__ float red[kNW];
  const int row = carried[blockIdx.x];
  const int ci = inv[row];
  T* fc = ffn_cache + static_cast<size_t>(row) * d;
  float* xr = x + static_cast<size_t>(row) * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += kThreads) {
    float f;
    if (ci >= 0) {
      f = roundf_to<T>(sum_slices(c_part, S, slice_stride, static_cast<size_t>(ci) * d + c));
      stf(fc + c, f);
    } else {
      f = ldf(fc + c);
    }
    const float v = xr[c] + f;
    xr[c] = v;
    ss += v * v;
  }
  if (next_gain != nullptr) {
    ss = block_sum<kNW>(ss, red);
    const float rstd = 1.0f / sqrtf(ss / static_cast<float>(d) + eps);
    T* hr = h + static_cast<size_t>(row) * d;
    for (int c = threadIdx.x; c < d; c += kThreads) stf(hr + c, xr[c] * rstd * ldf(next_gain + c));
  } else {
    T* o = hidden_out + static_cast<size_t>(row) * d;
    const int pos = row % n;
    T* po = (prompt_out != nullptr && pos < L_p)
                ? prompt_out + (static_cast<size_t>(row / n) * L_p + pos) * d
                : nullptr;
    for (int c = threadIdx.x; c < d; c += kThreads) {
      const float v = xr[c];
      stf(o + c, v);
      if (po) stf(po + c, v);
    }
  }
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

}  // namespace

template <typename T> static inline T* P(void* p) { return static_cast<T*>(p); }
template <typename T> static inline const T* P(const void* p) { return static_cast<const T*>(p); }

void launch_embed_norm(const RowKernelArgs& a, const void* hidden_in, const int* rows, int M,
                       const void* gain, float* x, void* h, hipStream_t st) {
  if (M <= 0) return;
  if (a.dtype == 1)
    hipLaunchKernelGGL(k_embed_norm<bf16_t>, dim3(M), dim3(kThreads), 0, st, P<bf16_t>(hidden_in),
                       rows, a.d, a.eps, P<bf16_t>(gain), x, P<bf16_t>(h));
  else
    hipLaunchKernelGGL(k_embed_norm<float>, dim3(M), dim3(kThreads), 0, st, P<float>(hidden_in),
                       rows, a.d, a.eps, P<float>(gain), x, P<float>(h));
}

void launch_v_finalize(const RowKernelArgs& a, const float* c_part, int S, const int* rows, int M,
                       int d_kv, void* v_cache, float* score, hipStream_t st) {
  if (M <= 0) return;
  const size_t stride = static_cast<size_t>(M) * d_kv;
  if (a.dtype == 1)
    hipLaunchKernelGGL(k_v_finalize<bf16_t>, dim3(M), dim3(kThreads), 0, st, c_part, S, stride, rows,
                       d_kv, a.n, a.L_p, P<bf16_t>(v_cache), score);
  else
    hipLaunchKernelGGL(k_v_finalize<float>, dim3(M), dim3(kThreads), 0, st, c_part, S, stride, rows,
                       d_kv, a.n, a.L_p, P<float>(v_cache), score);
}

void launch_qk_finalize(const RowKernelArgs& a, const float* c_part, int S, const int* rows, int M,
                        int d_q, int d_kv, int d_h, const float2* rope_tab, void* q_out,
                        void* k_cache, hipStream_t st) {
  if (M <= 0) return;
  const size_t stride = static_cast<size_t>(M) * (d_q + d_kv);
  if (a.dtype == 1)
    hipLaunchKernelGGL(k_qk_finalize<bf16_t>, dim3(M), dim3(kThreads), 0, st, c_part, S, stride,
                       rows, a.n, d_q, d_kv, d_h, rope_tab, P<bf16_t>(q_out), P<bf16_t>(k_cache));
  else
    hipLaunchKernelGGL(k_qk_finalize<float>, dim3(M), dim3(kThreads), 0, st, c_part, S, stride,
                       rows, a.n, d_q, d_kv, d_h, rope_tab, P<float>(q_out), P<float>(k_cache));
}

void launch_o_finalize(const RowKernelArgs& a, const float* c_part, int S, int M_R,
                       const int* carried, int Mc, const int* inv, void* attn_cache, float* x,
                       const void* gain, void* g_out, hipStream_t st) {
  if (Mc <= 0) return;
  const size_t stride = static_cast<size_t>(M_R) * a.d;
  if (a.dtype == 1)
    hipLaunchKernelGGL(k_o_finalize<bf16_t>, dim3(Mc), dim3(kThreads), 0, st, c_part, S, stride,
                       carried, inv, a.d, a.eps, P<bf16_t>(attn_cache), x, P<bf16_t>(gain),
                       P<bf16_t>(g_out));
  else
    hipLaunchKernelGGL(k_o_finalize<float>, dim3(Mc), dim3(kThreads), 0, st, c_part, S, stride,
                       carried, inv, a.d, a.eps, P<float>(attn_cache), x, P<float>(gain),
                       P<float>(g_out));
}

void launch_swiglu(int dtype, const float* c_part, int S, int M, int m, void* u, hipStream_t st) {
  if (M <= 0) return;
  const size_t stride = static_cast<size_t>(M) * 2 * m;
  const dim3 grid((m + kThreads - 1) / kThreads, M);
  if (dtype == 1)
    hipLaunchKernelGGL(k_swiglu<bf16_t>, grid, dim3(kThreads), 0, st, c_part, S, stride, m,
                       P<bf16_t>(u));
  else
    hipLaunchKernelGGL(k_swiglu<float>, grid, dim3(kThreads), 0, st, c_part, S, stride, m,
                       P<float>(u));
}

void launch_down_finalize(const RowKernelArgs& a, const float* c_part, int S, int M_R,
                          const int* carried, int Mc, const int* inv, void* ffn_cache, float* x,
                          const void* next_gain, void* h, void* hidden_out, void* prompt_out,
                          hipStream_t st) {
  if (Mc <= 0) return;
  const size_t stride = static_cast<size_t>(M_R) * a.d;
  if (a.dtype == 1)
    hipLaunchKernelGGL(k_down_finalize<bf16_t>, dim3(Mc), dim3(kThreads), 0, st, c_part, S, stride,
                       carried, inv, a.d, a.n, a.L_p, a.eps, P<bf16_t>(ffn_cache), x,
                       P<bf16_t>(next_gain), P<bf16_t>(h), P<bf16_t>(hidden_out),
                       P<bf16_t>(prompt_out));
  else
    hipLaunchKernelGGL(k_down_finalize<float>, dim3(Mc), dim3(kThreads), 0, st, c_part, S, stride,
                       carried, inv, a.d, a.n, a.L_p, a.eps, P<float>(ffn_cache), x,
                       P<float>(next_gain), P<float>(h), P<float>(hidden_out), P<float>(prompt_out));
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
