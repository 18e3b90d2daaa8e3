// Gathered linear maps  C[i, :] = A[rows[i], :] * W^T  (W row-major [N, K], K contiguous).
//
// Two kernels:
//  * k_gemm_simple  -- plain LDS-tiled FMA kernel for any storage type and shape (used for
//                      float32 models and as the fallback for shapes the MFMA kernel
//                      does not take).
//  * k_gemm_stream  -- bf16 MFMA kernel built for the cached step's regime: few activation
//                      rows (64 per workgroup tile) against a weight matrix that is read
//                      exactly once from HBM.  The activation tile is staged in LDS, the
//                      weight rows go straight from global memory into the MFMA B operand
//                      (each lane reads 64 contiguous bytes of one weight row, so a
//                      wavefront consumes whole 256-byte row segments), and the contraction
//                      index is split over workgroups to put >= 2 workgroups on every CU.
//                      Partial sums go to float32 slices that the row kernels add up in a
//                      fixed order (no float atomics: results are bit-reproducible).
#include "common.hpp"

namespace dllmc {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int kMaxSlices = 8;
int gemm_max_slices() { return kMaxSlices; }

// ------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_gemm_simple(const T* __restrict__ A, int lda,
                                                     const int* __restrict__ rows, int M,
                                                     const T* __restrict__ W0,
                                                     const T* __restrict__ W1, int N0, int N, int K,
                                                     float* __restrict__ C) {
  __shared__ float As[16][65];
  __shared__ float Ws[16][65];
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int e = threadIdx.x; e < 1024; e += 256) {
      const int r = e / 16, kk = e % 16;
      float a = 0.f, w = 0.f;
      if (k0 + kk < K) {
        const int m = m0 + r;
        if (m < M) {
          const int row = rows ? rows[m] : m;
          a = ldf(A + static_cast<size_t>(row) * lda + k0 + kk);
        }
        const int nn = n0 + r;
        if (nn < N) {
          const T* wp = nn < N0 ? W0 + static_cast<size_t>(nn) * K
                                : W1 + static_cast<size_t>(nn - N0) * K;
          w = ldf(wp + k0 + kk);
        }
      }
      As[kk][r] = a;
      Ws[kk][r] = w;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Ws[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int nn = n0 + tx * 4 + j;
      if (nn < N) C[static_cast<size_t>(m) * N + nn] = acc[i][j];
    }
  }
}

// ------------------------------------------------------------------------------------
// Workgroup = NW wavefronts; tile = 64 activation rows x (16*NW) output columns; wavefront w
// owns 16 columns and all 64 rows (four 16x16 accumulators of v_mfma_f32_16x16x32_bf16).
// Per 128-wide step of the contraction index, lane (n = lane%16, g = lane/16) holds
// W[col n][k0 + 32g .. k0 + 32g + 31]; its c-th 16-byte piece is MFMA step c, and the A
// operand is read from LDS with the same (g, c) -> k mapping, so the order in which the
// contraction index is visited differs from 0..K-1 but is the same for both operands.
template <int NW>
__global__ __launch_bounds__(NW * 64) void k_gemm_stream(
    const bf16_t* __restrict__ A, int lda, const int* __restrict__ rows, int M,
    const bf16_t* __restrict__ W0, const bf16_t* __restrict__ W1, int N0, int N, int K,
    int k_per_slice, int KC, float* __restrict__ C) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem_raw);
  const int lds_stride = KC + 8;  // +16 bytes: consecutive rows start 4 banks apart
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int ln = lane % 16, lg = lane / 16;
  const int m0 = blockIdx.y * 64;
  const int kbeg = blockIdx.z * k_per_slice;
  const int kend = min(K, kbeg + k_per_slice);
  const int ncol = blockIdx.x * (16 * NW) + wave * 16 + ln;  // < N: N % (16*NW) == 0
  const bf16_t* wrow = ncol < N0 ? W0 + static_cast<size_t>(ncol) * K
                                 : W1 + static_cast<size_t>(ncol - N0) * K;
  f32x4 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int kp = kbeg; kp < kend; kp += KC) {
    const int kc = min(KC, kend - kp);  // multiple of 128
    __syncthreads();
    {
      const int cpr = kc / 8;  // 16-byte chunks per row
      for (int e = threadIdx.x; e < 64 * cpr; e += NW * 64) {
        const int r = e / cpr, c = e - r * cpr;
        const int m = m0 + r;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (m < M) {
          const int row = rows ? rows[m] : m;
          v = *reinterpret_cast<const uint4*>(A + static_cast<size_t>(row) * lda + kp + c * 8);
        }
        *reinterpret_cast<uint4*>(As + r * lds_stride + c * 8) = v;
      }
    }
    __syncthreads();

    const bf16_t* wp = wrow + kp + lg * 32;
    const bf16_t* ap = As + ln * lds_stride + lg * 32;
    uint4 bn[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) bn[c] = *reinterpret_cast<const uint4*>(wp + c * 8);
    for (int ks = 0; ks < kc; ks += 128) {
      uint4 b[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) b[c] = bn[c];
      if (ks + 128 < kc) {
#pragma unroll
        for (int c = 0; c < 4; ++c) bn[c] = *reinterpret_cast<const uint4*>(wp + ks + 128 + c * 8);
      }
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bf16x8 bf = __builtin_bit_cast(bf16x8, b[c]);
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) {
          const bf16x8 af =
              *reinterpret_cast<const bf16x8*>(ap + mb * 16 * lds_stride + ks + c * 8);
          acc[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, bf, acc[mb], 0, 0, 0);
        }
      }
    }
  }

  float* Cs = C + static_cast<size_t>(blockIdx.z) * M * N;
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = m0 + mb * 16 + lg * 4 + i;
      if (m < M) Cs[static_cast<size_t>(m) * N + ncol] = acc[mb][i];
    }
}

__global__ __launch_bounds__(256) void k_reduce_slices(const float* __restrict__ c_part, int S,
                                                       size_t MN, float* __restrict__ out) {
  const size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= MN) return;
  float t = c_part[i];
  for (int s = 1; s < S; ++s) t += c_part[static_cast<size_t>(s) * MN + i];
  out[i] = t;
}

void launch_reduce_slices(const float* c_part, int S, int M, int N, float* out, hipStream_t st) {
  const size_t MN = static_cast<size_t>(M) * N;
  if (MN == 0) return;
  hipLaunchKernelGGL(k_reduce_slices, dim3(static_cast<unsigned>((MN + 255) / 256)), dim3(256), 0,
                     st, c_part, S, MN, out);
}

// ------------------------------------------------------------------------------------
namespace {
constexpr int kStreamNW = 8;      // wavefronts per workgroup of the streaming kernel
constexpr int kStreamKC = 512;    // contraction-index extent staged in LDS per phase
bool g_attr_set = false;

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
}  // namespace

int launch_gemm(int dtype, const void* A, int lda, const int* rows, int M, const void* W0,
                const void* W1, int N0, int N, int K, float* c_part, hipStream_t st) {
  if (M <= 0 || N <= 0) return 1;
  const int BN = 16 * kStreamNW;
  const bool stream_ok = dtype == 1 && (K % 128 == 0) && (N % BN == 0) && (N0 % BN == 0) &&
                         (lda % 8 == 0) && aligned16(A) && aligned16(W0) &&
                         (W1 == nullptr || aligned16(W1));
  if (!stream_ok) {
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    if (dtype == 1)
      hipLaunchKernelGGL(k_gemm_simple<bf16_t>, grid, dim3(256), 0, st,
                         static_cast<const bf16_t*>(A), lda, rows, M,
                         static_cast<const bf16_t*>(W0), static_cast<const bf16_t*>(W1), N0, N, K,
                         c_part);
    else
      hipLaunchKernelGGL(k_gemm_simple<float>, grid, dim3(256), 0, st,
                         static_cast<const float*>(A), lda, rows, M, static_cast<const float*>(W0),
                         static_cast<const float*>(W1), N0, N, K, c_part);
    return 1;
  }
  const int mt = (M + 63) / 64, nt = N / BN;
  // enough workgroups for two per CU (256 CUs) when the tile count alone does not give them
  int S = (512 + mt * nt - 1) / (mt * nt);
  S = S < 1 ? 1 : (S > kMaxSlices ? kMaxSlices : S);
  int kps = ((K + S - 1) / S + 127) / 128 * 128;
  if (kps < 256) kps = 256;
  if (kps > K) kps = K;
  S = (K + kps - 1) / kps;
  const int KC = kps < kStreamKC ? kps : kStreamKC;
  const size_t lds = static_cast<size_t>(64) * (KC + 8) * sizeof(bf16_t);
  if (!g_attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_stream<kStreamNW>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 64);
    g_attr_set = true;
  }
  hipLaunchKernelGGL(k_gemm_stream<kStreamNW>, dim3(nt, mt, S), dim3(kStreamNW * 64), lds, st,
                     static_cast<const bf16_t*>(A), lda, rows, M, static_cast<const bf16_t*>(W0),
                     static_cast<const bf16_t*>(W1), N0, N, K, kps, KC, c_part);
  return S;
}

}  // namespace dllmc
