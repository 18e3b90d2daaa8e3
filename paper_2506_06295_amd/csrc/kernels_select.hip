// Bottom-k selection of the V-verify scores (paper Sec. 3.2.2): per sequence, the k rows with
// the lowest score, equal scores lowest index first, emitted ascending by index.
//
// One workgroup per sequence.  Scores are mapped to unsigned keys whose integer order is the
// float order; four 8-bit radix passes over an LDS histogram find the key of the k-th
// smallest element and how many elements equal to it still belong to the set; one ordered
// compaction pass (ballot + popcount prefix sums per wavefront, LDS across wavefronts) then
// writes the indices in ascending order.  Everything is integer work after the key mapping,
// so the result is exact and independent of scheduling.
#include "common.hpp"

namespace dllmc {

namespace {

constexpr int kThreads = 256;
constexpr int kNW = kThreads / kWave;
constexpr int kKeysInLds = 8192;  // response lengths up to this keep their keys in LDS

__device__ __forceinline__ uint32_t order_key(float s) {
  s += 0.0f;  // -0.0 -> +0.0 so that the two zeros tie
  const uint32_t u = __float_as_uint(s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Exclusive prefix sum of v over the workgroup in thread order; total in *total.
// scratch: kNW + 1 uints of LDS.
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* scratch, uint32_t* total) {
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  uint32_t inc = v;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const uint32_t t = __shfl_up(inc, o, kWave);
    if (lane >= o) inc += t;
  }
  __syncthreads();
  if (lane == kWave - 1) scratch[w] = inc;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < kNW; ++i) {
    const uint32_t s = scratch[i];
    if (i < w) base += s;
    tot += s;
  }
  *total = tot;
  return base + inc - v;
}

// part != nullptr: the scores are formed here first, from the sums the fused V-verify kernel left
// per (row, column tile): part[(c * n_ct + tile) * part_stride + b * L + j], c = 0 dot product (or
// squared distance), 1 |new|^2, 2 |old|^2, added in tile order; Eq. (cos_sim) with the
// denominator clamped at 1e-8, or minus the distance (metric 1).  They are written to `scores`.
__global__ __launch_bounds__(kThreads) void k_select(float* scores, int L, int k,
                                                     int* __restrict__ sel_out, int sel_stride,
                                                     int* __restrict__ rows_out, int per_seq,
                                                     int off, int* __restrict__ inv_out, int n,
                                                     int L_p, const float* __restrict__ part,
                                                     int n_ct, int part_stride, int metric) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t scan_scratch[kNW + 1];
  __shared__ uint32_t sh_prefix, sh_need;
  __shared__ __attribute__((aligned(16))) uint32_t keys[kKeysInLds];
  __shared__ __attribute__((aligned(16))) float psum[kNW][3][kThreads];
  const int b = blockIdx.x;
  float* s = scores + static_cast<size_t>(b) * L;
  // The five passes below read every key; one trip to global memory instead of five when the
  // sequence fits the LDS buffer (the visibility of `keys` rides on the first barrier below).
  const bool in_lds = L <= kKeysInLds;
  if (part != nullptr) {
    const size_t comp = static_cast<size_t>(n_ct) * part_stride;
    const bool vec = (L % 4 == 0) && (part_stride % 4 == 0) &&
                     (reinterpret_cast<uintptr_t>(part) & 15u) == 0;
    if (vec) {
      // A lane takes four neighbouring rows (16-byte loads) and a wavefront a quarter of the
      // column tiles, up to 16 tiles x 3 sums requested before the first is added, so that the
      // whole table is in flight at once; the wavefronts' sums meet in LDS and are added in
      // wavefront order (= tile order).
      const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
      const int per = (n_ct + kNW - 1) / kNW;
      const int t0 = w * per, t1 = min(n_ct, t0 + per);
      for (int j0 = 0; j0 < L; j0 += 4 * kWave) {
        const int jl = j0 + 4 * lane;
        const bool rv = jl < L;
        const float* p0 = part + static_cast<size_t>(b) * L + (rv ? jl : 0);
        float4 acc[3];
#pragma unroll
        for (int c = 0; c < 3; ++c) acc[c] = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int c0 = t0; c0 < t1; c0 += 16) {
          float4 v[3][16];
#pragma unroll
          for (int u = 0; u < 16; ++u) {
            const size_t ct = static_cast<size_t>(min(c0 + u, t1 - 1)) * part_stride;
#pragma unroll
            for (int c = 0; c < 3; ++c) v[c][u] = *reinterpret_cast<const float4*>(p0 + c * comp + ct);
          }
#pragma unroll
          for (int u = 0; u < 16; ++u)
            if (c0 + u < t1) {
#pragma unroll
              for (int c = 0; c < 3; ++c) {
                acc[c].x += v[c][u].x;
                acc[c].y += v[c][u].y;
                acc[c].z += v[c][u].z;
                acc[c].w += v[c][u].w;
              }
            }
        }
#pragma unroll
        for (int c = 0; c < 3; ++c) *reinterpret_cast<float4*>(&psum[w][c][4 * lane]) = acc[c];
        __syncthreads();
        const int j = j0 + static_cast<int>(threadIdx.x);
        if (j < L) {
          float dot = psum[0][0][threadIdx.x], nn = psum[0][1][threadIdx.x], no = psum[0][2][threadIdx.x];
#pragma unroll
          for (int ww = 1; ww < kNW; ++ww) {
            dot += psum[ww][0][threadIdx.x];
            nn += psum[ww][1][threadIdx.x];
            no += psum[ww][2][threadIdx.x];
          }
          const float sc = metric == 0 ? dot / fmaxf(sqrtf(nn) * sqrtf(no), 1e-8f) : -sqrtf(dot);
          s[j] = sc;
          if (in_lds) keys[j] = order_key(sc);
        }
        __syncthreads();
      }
    } else {
      for (int j = threadIdx.x; j < L; j += kThreads) {
        const float* p0 = part + static_cast<size_t>(b) * L + j;
        float dot = 0.f, nn = 0.f, no = 0.f;
        for (int ct = 0; ct < n_ct; ++ct) {
          dot += p0[static_cast<size_t>(ct) * part_stride];
          nn += p0[comp + static_cast<size_t>(ct) * part_stride];
          no += p0[2 * comp + static_cast<size_t>(ct) * part_stride];
        }
        const float sc = metric == 0 ? dot / fmaxf(sqrtf(nn) * sqrtf(no), 1e-8f) : -sqrtf(dot);
        s[j] = sc;
        if (in_lds) keys[j] = order_key(sc);
      }
    }
    if (!in_lds) {  // the passes below re-read the scores this workgroup has just written
      __threadfence_block();
      __syncthreads();
    }
  } else if (in_lds) {
    for (int j = threadIdx.x; j < L; j += kThreads) keys[j] = order_key(s[j]);
  }
  if (k <= 0) __syncthreads();

  uint32_t kth = 0, need = 0;
  if (k > 0) {
    uint32_t prefix = 0;
    need = static_cast<uint32_t>(k);
    for (int pass = 3; pass >= 0; --pass) {
      const int shift = pass * 8;
      const uint32_t himask = pass == 3 ? 0u : (0xFFFFFFFFu << (shift + 8));
      hist[threadIdx.x] = 0;
      __syncthreads();
      for (int j = threadIdx.x; j < L; j += kThreads) {
        const uint32_t key = in_lds ? keys[j] : order_key(s[j]);
        if ((key & himask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
      }
      __syncthreads();
      uint32_t total;
      const uint32_t cnt = hist[threadIdx.x];
      const uint32_t excl = block_excl_scan(cnt, scan_scratch, &total);
      // exactly one bucket satisfies excl < need <= excl + cnt
      if (excl < need && need <= excl + cnt) {
        sh_prefix = prefix | (static_cast<uint32_t>(threadIdx.x) << shift);
        sh_need = need - excl;
      }
      __syncthreads();
      prefix = sh_prefix;
      need = sh_need;
      __syncthreads();
    }
    kth = prefix;
  }

  uint32_t base_sel = 0, base_eq = 0;
  for (int j0 = 0; j0 < L; j0 += kThreads) {
    const int j = j0 + threadIdx.x;
    const bool valid = j < L;
    const uint32_t key = valid ? (in_lds ? keys[j] : order_key(s[j])) : 0xFFFFFFFFu;
    const bool less = valid && k > 0 && key < kth;
    const bool eq = valid && k > 0 && key == kth;
    uint32_t tot_eq, tot_take;
    const uint32_t eq_rank = base_eq + block_excl_scan(eq ? 1u : 0u, scan_scratch, &tot_eq);
    const bool take = less || (eq && eq_rank < need);
    const uint32_t pos = base_sel + block_excl_scan(take ? 1u : 0u, scan_scratch, &tot_take);
    if (take) {
      if (sel_out) sel_out[static_cast<size_t>(b) * sel_stride + pos] = j;
      if (rows_out) rows_out[b * per_seq + off + static_cast<int>(pos)] = b * n + L_p + j;
    }
    if (valid && inv_out) inv_out[b * n + L_p + j] = take ? b * per_seq + off + static_cast<int>(pos) : -1;
    base_eq += tot_eq;
    base_sel += tot_take;
  }
}

// MurmurHash3's 32-bit finalizer: a bijective avalanche mix
__device__ __forceinline__ uint32_t fmix32(uint32_t x) {
  x ^= x >> 16;
  x *= 0x85EBCA6Bu;
  x ^= x >> 13;
  x *= 0xC2B2AE35u;
  x ^= x >> 16;
  return x;
}

// Scores of the random-selection baseline (paper Sec. 4.3): a counter-based uniform in [0, 1)
// with 24 bits per (seed, step, layer, sequence, position): h = seed; for each of step, layer,
// sequence, position: h = fmix32(h xor value); score = (h >> 8) * 2^-24.
__global__ __launch_bounds__(kThreads) void k_random_scores(uint32_t seed, uint32_t step,
                                                            uint32_t layer, int B, int L,
                                                            float* __restrict__ out) {
  const int i = blockIdx.x * kThreads + threadIdx.x;
  if (i >= B * L) return;
  const uint32_t b = static_cast<uint32_t>(i / L), j = static_cast<uint32_t>(i % L);
  const uint32_t h = fmix32(fmix32(fmix32(fmix32(seed ^ step) ^ layer) ^ b) ^ j);
  out[i] = static_cast<float>(h >> 8) * 5.9604644775390625e-8f;  // 2^-24
}

}  // namespace

void launch_random_scores(uint32_t seed, int step, int layer, int B, int L, float* out,
                          hipStream_t st) {
  if (B * L <= 0) return;
  hipLaunchKernelGGL(k_random_scores, dim3((B * L + kThreads - 1) / kThreads), dim3(kThreads), 0, st,
                     seed, static_cast<uint32_t>(step), static_cast<uint32_t>(layer), B, L, out);
}

void launch_select(float* scores, int B, int L, int k, int* sel_out, int sel_stride,
                   int* rows_out, int per_seq, int off, int* inv_out, int n, int L_p,
                   hipStream_t st, const float* part, int n_ct, int part_stride, int metric) {
  if (B <= 0 || L <= 0) return;
  hipLaunchKernelGGL(k_select, dim3(B), dim3(kThreads), 0, st, scores, L, k, sel_out, sel_stride,
                     rows_out, per_seq, off, inv_out, n, L_p, part, n_ct, part_stride, metric);
}

}  // namespace dllmc
