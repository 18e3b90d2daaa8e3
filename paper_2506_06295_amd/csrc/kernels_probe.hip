// Achievable-peak probes: what this GPU actually delivers for a plain stream copy, a plain
// read-only stream and a back-to-back MFMA loop, so that a kernel's roofline fraction can be
// quoted against the measured ceiling as well as against the published one.  None of these is a
// step of the method.
#include "common.hpp"

namespace dllmc {

namespace {

constexpr int kThreads = 256;

// dst[i] = src[i], 16 bytes per lane per trip, four independent trips in flight per lane
__global__ __launch_bounds__(kThreads) void k_probe_copy(const uint4* __restrict__ src,
                                                         uint4* __restrict__ dst, size_t count) {
  const size_t stride = static_cast<size_t>(gridDim.x) * kThreads;
  size_t i = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
  for (; i + 3 * stride < count; i += 4 * stride) {
    const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], e = src[i + 3 * stride];
    dst[i] = a;
    dst[i + stride] = b;
    dst[i + 2 * stride] = c;
    dst[i + 3 * stride] = e;
  }
  for (; i < count; i += stride) dst[i] = src[i];
}

// reads src once; every lane folds what it read into one word, and a store happens only if the
// fold equals one fixed value (a 2^-32 chance per lane; the store is in bounds anyway), so the
// loads cannot be dropped and in practice nothing is written
__global__ __launch_bounds__(kThreads) void k_probe_read(const uint4* __restrict__ src, size_t count,
                                                         uint32_t* __restrict__ sink) {
  const size_t stride = static_cast<size_t>(gridDim.x) * kThreads;
  size_t i = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
  uint32_t acc = 0;
  for (; i + 3 * stride < count; i += 4 * stride) {
    const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], e = src[i + 3 * stride];
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ e.x ^ e.y ^ e.z ^ e.w;
  }
  for (; i < count; i += stride) {
    const uint4 a = src[i];
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
  if (acc == 0x9e3779b9u) sink[0] = acc;
}

// iters trips of eight independent 16x16x32 bf16 MFMAs per wavefront, operands held in registers
__global__ __launch_bounds__(kThreads) void k_probe_mfma(int iters, float* __restrict__ sink) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = static_cast<__bf16>(static_cast<float>((threadIdx.x + i) & 7) * 0.125f);
    b[i] = static_cast<__bf16>(static_cast<float>((threadIdx.x * 3 + i) & 7) * 0.125f);
  }
  f32x4 acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int t = 0; t < iters; ++t) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[j], 0, 0, 0);
  }
  f32x4 s = acc[0];
#pragma unroll
  for (int j = 1; j < 8; ++j) s += acc[j];
  // one wavefront of the grid writes its result (64 lanes x 4 floats): keeps the loop alive
  if (blockIdx.x == 0 && threadIdx.x < kWave)
    *reinterpret_cast<f32x4*>(sink + threadIdx.x * 4) = s;
}

// the same with four independent 32x32x16 bf16 MFMAs per trip (the same flops per trip)
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
__global__ __launch_bounds__(kThreads) void k_probe_mfma32(int iters, float* __restrict__ sink) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = static_cast<__bf16>(static_cast<float>((threadIdx.x + i) & 7) * 0.125f);
    b[i] = static_cast<__bf16>(static_cast<float>((threadIdx.x * 3 + i) & 7) * 0.125f);
  }
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
  for (int t = 0; t < iters; ++t) {
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
  }
  f32x16 s = acc[0];
#pragma unroll
  for (int j = 1; j < 4; ++j) s += acc[j];
  if (blockIdx.x == 0 && threadIdx.x < kWave) {
    float t = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) t += s[e];
    sink[threadIdx.x] = t;
  }
}

int probe_grid() {
  int dev = 0, cus = 256;
  if (hipGetDevice(&dev) == hipSuccess)
    (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  return cus * 8;
}

}  // namespace

void launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t st) {
  if (bytes < 16) return;
  hipLaunchKernelGGL(k_probe_copy, dim3(probe_grid()), dim3(kThreads), 0, st,
                     static_cast<const uint4*>(src), static_cast<uint4*>(dst), bytes / 16);
}

void launch_probe_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t st) {
  if (bytes < 16) return;
  hipLaunchKernelGGL(k_probe_read, dim3(probe_grid()), dim3(kThreads), 0, st,
                     static_cast<const uint4*>(src), bytes / 16, sink);
}

double launch_probe_mfma(int iters, int shape, float* sink, hipStream_t st) {
  const int grid = probe_grid();
  if (shape == 1)
    hipLaunchKernelGGL(k_probe_mfma32, dim3(grid), dim3(kThreads), 0, st, iters, sink);
  else
    hipLaunchKernelGGL(k_probe_mfma, dim3(grid), dim3(kThreads), 0, st, iters, sink);
  // wavefronts x trips x 8 MFMAs x (16 * 16 * 32 multiply-adds, two flops each)
  return static_cast<double>(grid) * (kThreads / kWave) * iters * 8.0 * (2.0 * 16 * 16 * 32);
}

}  // namespace dllmc
