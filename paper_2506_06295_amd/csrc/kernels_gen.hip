// Kernels of the closed denoising loop around the cached step (paper Sec. 3.1: greedy estimate
// of the clean sequence, transition to the next state by low-confidence remasking):
//   k_embed_gather    token ids -> embedded rows
//   k_elig_scores     which response positions are still masked inside the current block
//   k_final_norm      RMSNorm with the final gain of the listed rows, compact output
//   k_head_finalize   per row of logits: greedy token (lowest id among equal logits) and its
//                     softmax probability, in one pass (running maximum and rescaled sum)
//   k_apply_tokens    the chosen positions take their greedy token
// The vocabulary projection itself is a gathered linear map (kernels_gemm.hip); the choice of
// the positions is the integer-exact bottom-k selection (kernels_select.hip) on the negated
// confidences.
#include <cmath>

#include "common.hpp"

namespace dllmc {

namespace {

constexpr int kThreads = 256;
constexpr int kNW = kThreads / kWave;

template <typename T>
__global__ __launch_bounds__(kThreads) void k_embed_gather(const T* __restrict__ table,
                                                           const int* __restrict__ tokens, int d,
                                                           int vocab_rows, T* __restrict__ out) {
  const int row = blockIdx.x;
  int tok = tokens[row];
  tok = tok < 0 ? 0 : (tok >= vocab_rows ? vocab_rows - 1 : tok);  // never read outside the table
  const T* src = table + static_cast<size_t>(tok) * d;
  T* dst = out + static_cast<size_t>(row) * d;
  constexpr int V = 16 / sizeof(T);  // elements per 16-byte vector
  if (d % V == 0) {
    const uint4* s4 = reinterpret_cast<const uint4*>(src);
    uint4* d4 = reinterpret_cast<uint4*>(dst);
    for (int c = threadIdx.x; c < d / V; c += kThreads) d4[c] = s4[c];
  } else {
    for (int c = threadIdx.x; c < d; c += kThreads) dst[c] = src[c];
  }
}

// elig[b][j] = 0 if response position j of sequence b holds mask_id and lo <= j < hi, else 1;
// neg_conf[b][j] = +inf and x0[b][j] = -1 (overwritten for the eligible positions later).
__global__ __launch_bounds__(kThreads) void k_elig_scores(const int* __restrict__ tokens, int B,
                                                          int n, int L_p, int lo, int hi,
                                                          int mask_id, float* __restrict__ elig,
                                                          float* __restrict__ neg_conf,
                                                          int* __restrict__ x0) {
  const int L_r = n - L_p;
  const int i = blockIdx.x * kThreads + threadIdx.x;
  if (i >= B * L_r) return;
  const int b = i / L_r, j = i % L_r;
  const bool e = j >= lo && j < hi && tokens[b * n + L_p + j] == mask_id;
  elig[i] = e ? 0.0f : 1.0f;
  neg_conf[i] = INFINITY;
  x0[i] = -1;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void k_final_norm(const T* __restrict__ hidden,
                                                         const int* __restrict__ rows, int d,
                                                         float eps, const T* __restrict__ gain,
                                                         T* __restrict__ z) {
  __shared__ float red[kNW];
  const int i = blockIdx.x;
  const int row = rows ? rows[i] : i;
  const T* src = hidden + static_cast<size_t>(row) * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += kThreads) {
    const float v = ldf(src + c);
    ss += v * v;
  }
  ss = block_sum<kNW>(ss, red);
  const float rstd = 1.0f / sqrtf(ss / static_cast<float>(d) + eps);
  T* dst = z + static_cast<size_t>(i) * d;
  for (int c = threadIdx.x; c < d; c += kThreads) stf(dst + c, ldf(src + c) * rstd * ldf(gain + c));
}

// running (maximum, sum of exp(l - maximum), index of the first maximum)
struct Soft {
  float m, s;
  int a;
};
__device__ __forceinline__ Soft soft_merge(const Soft& p, const Soft& q) {
  Soft r;
  r.m = fmaxf(p.m, q.m);
  r.s = (p.m == -INFINITY ? 0.f : p.s * expf(p.m - r.m)) +
        (q.m == -INFINITY ? 0.f : q.s * expf(q.m - r.m));
  r.a = p.m > q.m ? p.a : (q.m > p.m ? q.a : min(p.a, q.a));
  return r;
}

// One workgroup per row i of logits: greedy token and confidence from logits[i][0..vocab).
// With rows (rows[i] = b*n + L_p + j) the results go to x0[b][j] and conf[b][j], otherwise to
// x0[i] and conf[i]; conf = sign * probability.
__global__ __launch_bounds__(kThreads) void k_head_finalize(const float* __restrict__ logits,
                                                            int vocab,
                                                            const int* __restrict__ rows, int n,
                                                            int L_p, float sign,
                                                            int* __restrict__ x0,
                                                            float* __restrict__ neg_conf) {
  __shared__ Soft part[kNW];
  const int i = blockIdx.x;
  const float* l = logits + static_cast<size_t>(i) * vocab;
  Soft t{-INFINITY, 0.f, 0x7fffffff};
  if (vocab % 4 == 0) {
    for (int c = threadIdx.x * 4; c < vocab; c += kThreads * 4) {
      const float4 v = *reinterpret_cast<const float4*>(l + c);
      const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int k = 0; k < 4; ++k) t = soft_merge(t, Soft{e[k], 1.f, c + k});
    }
  } else {
    for (int c = threadIdx.x; c < vocab; c += kThreads) t = soft_merge(t, Soft{l[c], 1.f, c});
  }
  // lanes, then wavefronts, in a fixed order
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) {
    Soft q;
    q.m = __shfl_xor(t.m, o, kWave);
    q.s = __shfl_xor(t.s, o, kWave);
    q.a = __shfl_xor(t.a, o, kWave);
    t = soft_merge(t, q);
  }
  if ((threadIdx.x & (kWave - 1)) == 0) part[threadIdx.x / kWave] = t;
  __syncthreads();
  if (threadIdx.x == 0) {
    Soft r = part[0];
#pragma unroll
    for (int w = 1; w < kNW; ++w) r = soft_merge(r, part[w]);
    int o = i;
    if (rows) {
      const int row = rows[i];
      o = (row / n) * (n - L_p) + (row % n - L_p);
    }
    x0[o] = r.a;
    neg_conf[o] = sign / r.s;
  }
}

// tokens[b][L_p + chosen[b][t]] = x0[b][chosen[b][t]] for t < n_unmask
__global__ __launch_bounds__(kThreads) void k_apply_tokens(int* __restrict__ tokens, int B, int n,
                                                           int L_p, const int* __restrict__ chosen,
                                                           int chosen_stride, int n_unmask,
                                                           const int* __restrict__ x0) {
  const int L_r = n - L_p;
  const int i = blockIdx.x * kThreads + threadIdx.x;
  if (i >= B * n_unmask) return;
  const int b = i / n_unmask, t = i % n_unmask;
  const int j = chosen[b * chosen_stride + t];
  tokens[b * n + L_p + j] = x0[b * L_r + j];
}

__global__ __launch_bounds__(kThreads) void k_negate_f32(float* __restrict__ p, size_t count) {
  const size_t i = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (i < count) p[i] = -p[i];
}

}  // namespace

void launch_negate_f32(float* p, size_t count, hipStream_t st) {
  if (count == 0) return;
  hipLaunchKernelGGL(k_negate_f32, dim3(static_cast<unsigned>((count + kThreads - 1) / kThreads)),
                     dim3(kThreads), 0, st, p, count);
}

void launch_embed_gather(int dtype, const void* table, int vocab_rows, const int* tokens, int rows,
                         int d, void* out, hipStream_t st) {
  if (rows <= 0) return;
  if (dtype == 1)
    hipLaunchKernelGGL(k_embed_gather<bf16_t>, dim3(rows), dim3(kThreads), 0, st,
                       static_cast<const bf16_t*>(table), tokens, d, vocab_rows,
                       static_cast<bf16_t*>(out));
  else
    hipLaunchKernelGGL(k_embed_gather<float>, dim3(rows), dim3(kThreads), 0, st,
                       static_cast<const float*>(table), tokens, d, vocab_rows,
                       static_cast<float*>(out));
}

void launch_elig_scores(const int* tokens, int B, int n, int L_p, int lo, int hi, int mask_id,
                        float* elig, float* neg_conf, int* x0, hipStream_t st) {
  const int total = B * (n - L_p);
  if (total <= 0) return;
  hipLaunchKernelGGL(k_elig_scores, dim3((total + kThreads - 1) / kThreads), dim3(kThreads), 0, st,
                     tokens, B, n, L_p, lo, hi, mask_id, elig, neg_conf, x0);
}

void launch_final_norm(int dtype, const void* hidden, const int* rows, int M, int d, float eps,
                       const void* gain, void* z, hipStream_t st) {
  if (M <= 0) return;
  if (dtype == 1)
    hipLaunchKernelGGL(k_final_norm<bf16_t>, dim3(M), dim3(kThreads), 0, st,
                       static_cast<const bf16_t*>(hidden), rows, d, eps,
                       static_cast<const bf16_t*>(gain), static_cast<bf16_t*>(z));
  else
    hipLaunchKernelGGL(k_final_norm<float>, dim3(M), dim3(kThreads), 0, st,
                       static_cast<const float*>(hidden), rows, d, eps,
                       static_cast<const float*>(gain), static_cast<float*>(z));
}

void launch_head_finalize(const float* logits, int M, int vocab, const int* rows, int n, int L_p,
                          float sign, int* x0, float* conf, hipStream_t st) {
  if (M <= 0) return;
  hipLaunchKernelGGL(k_head_finalize, dim3(M), dim3(kThreads), 0, st, logits, vocab, rows, n, L_p,
                     sign, x0, conf);
}

void launch_apply_tokens(int* tokens, int B, int n, int L_p, const int* chosen, int chosen_stride,
                         int n_unmask, const int* x0, hipStream_t st) {
  const int total = B * n_unmask;
  if (total <= 0) return;
  hipLaunchKernelGGL(k_apply_tokens, dim3((total + kThreads - 1) / kThreads), dim3(kThreads), 0, st,
                     tokens, B, n, L_p, chosen, chosen_stride, n_unmask, x0);
}

}  // namespace dllmc
