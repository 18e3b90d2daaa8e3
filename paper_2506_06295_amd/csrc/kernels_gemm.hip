// Gathered linear maps  C[i, :] = A[rows[i], :] * W^T  (W row-major [N, K], K contiguous).
//
// Kernels:
//  * k_gemm_simple  -- plain LDS-tiled FMA kernel for any storage type and shape (used for
//                      float32 models and as the fallback for shapes the MFMA kernel
//                      does not take).
//  * k_gemm_stream  -- bf16 MFMA kernel built for the cached step's regime: few activation
//                      rows (64 or 128 per workgroup tile) against a weight matrix that is read
//                      exactly once from HBM.  The activation tile is staged in LDS, the
//                      weight rows go straight from global memory into the MFMA B operand
//                      (each lane reads 64 contiguous bytes of one weight row, so a
//                      wavefront consumes whole 256-byte row segments), and the contraction
//                      index is split over workgroups so that every CU gets one.
//                      Partial sums go to float32 slices that the row kernels add up in a
//                      fixed order (no float atomics: results are bit-reproducible).
//  * k_gemm_fat / k_gemm_mid -- bf16 MFMA kernels with 256 x 256 / 128 x 128 tiles whose
//                      operands both go through LDS by direct global->LDS loads, for
//                      launches with hundreds of activation rows; the same body with paired
//                      gate/up column blocks and SwiGLU in the epilogue (k_gemm_*_swiglu,
//                      k_gemm_tall_swiglu: 256 x 96 for up to 256 rows).
#include <mutex>

#include "common.hpp"

namespace dllmc {


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
// k_gemm_stream<NW, KC, DUAL, KH>
// Workgroup = NW wavefronts; tile = 64 activation rows x (16*NW) output columns; wavefront w
// owns 16 columns and all 64 rows (four 16x16 accumulators of v_mfma_f32_16x16x32_bf16 per
// weight matrix).  The workgroup's slice of the contraction index is walked in phases of KC:
// the activation tile of phase p+1 is fetched into registers while phase p is multiplied and
// is written to the other LDS buffer at the end of the phase (one barrier per phase).  The
// weight stream is prefetched one whole phase ahead and runs across phase boundaries.
// Lane (n = lane%16, g = lane/16) holds, for MFMA step c of a 128-wide step, the eight
// weights W[col n][k0 + 32c + 8g ..+8]; the A operand is read from LDS at the same offsets
// (the 16-byte chunks of an LDS row are XOR-permuted in groups of 16 by row % 16, which keeps
// the fragment reads free of bank conflicts; with a padded row stride, or a permutation by
// row % 8, half of the LDS cycles of the reads were conflicts).
//   DUAL = 0: columns [0,N0) come from W0, [N0,N) from W1; float32 partial sums are stored
//             to slice blockIdx.z of C.
//   DUAL = 1: every lane streams row n of W0 (gate) and row n of W1 (up) and the epilogue
//             stores bf16(silu(gate) * up) to U[M, N] (SwiGLU, complexity appendix of the
//             paper); needs a single slice.
//   KH = 2:   the wavefronts form two groups that walk the two halves of the workgroup's
//             contraction range side by side (tile = 16*NW/2 columns); the second group hands
//             its accumulators over through LDS at the end and the first adds them (its own
//             sum first).  Doubles the wavefronts, and with them the loads in flight, of a
//             launch that cannot split the contraction over workgroups (DUAL).
// N only has to be a multiple of 16: a ragged last tile is allowed, and with it any number of
// column wavefronts.
//   RB:       16-row blocks per workgroup (4: the 64 rows described above).  With RB = 8 / 16 a
//             wavefront keeps the accumulators of 128 / 256 rows, so the weights of a launch
//             with that many rows are streamed once instead of once per 64-row tile (phases of
//             128 then, to fit the activation tiles in LDS).
template <int NW, int KC, int DUAL, int KH, int RB = 4>
__global__ __launch_bounds__(NW * 64) void k_gemm_stream(
    const bf16_t* __restrict__ A, int lda, const int* __restrict__ rows, int M,
    const bf16_t* __restrict__ W0, const bf16_t* __restrict__ W1, int N0, int N, int K,
    int k_per_slice, float* __restrict__ C, bf16_t* __restrict__ U, int n_full) {
  constexpr int LS = KC;                          // LDS row stride; chunk q of row r sits in slot
                                                  // q ^ (r % 16) of its group of 16 (no padding)
  constexpr int CPR = KC / 8;                     // 16-byte chunks per activation row and phase
  constexpr int R = 16 * RB;                      // activation rows per workgroup
  constexpr int TOT = KH * R * CPR;               // chunks of the workgroup's activation tiles
  constexpr int NCH = (TOT + NW * 64 - 1) / (NW * 64);  // chunks staged per thread and phase
  constexpr bool EVEN = TOT % (NW * 64) == 0;     // otherwise the last chunk of some threads is void
  constexpr int NB = DUAL ? 2 : 1;
  constexpr int NWC = NW / KH;                    // wavefronts side by side over the columns
  static_assert(NW % KH == 0, "wavefront groups must be equal");
  __shared__ __attribute__((aligned(16))) bf16_t As[2][KH][R * LS];
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int ln = lane % 16, lg = lane / 16;
  const int wcol = wave % NWC, kh = wave / NWC;
  int col_tile, row_tile;
  xcd_tile_map(col_tile, row_tile);
  const int m0 = row_tile * R;
  const int kbeg = blockIdx.z * k_per_slice;
  const int klen = min(K, kbeg + k_per_slice) - kbeg;  // multiple of KH * KC
  const int hlen = klen / KH;                          // contraction range of one group
  const int nph = hlen / KC;
  // DUAL: the walk starts at a phase that depends on the column tile and wraps around.  The
  // workgroups of such a launch (one per CU, a single slice) run nearly in step, and rows of W
  // are a multiple of 4 KB apart at these widths: unrotated, every load in flight on the chip
  // has the same address bits below the row pitch and the memory channels are loaded unevenly
  // (the launch took 48 to 61 us depending on where the two matrices happened to lie; rotated,
  // 49 to 52 us everywhere).  The split launches already walk different ranges side by side
  // and gain nothing; a single-slice launch with several workgroups per CU (the vocabulary
  // projection) lost 10-35 %, so they keep the plain order.
  const int rot = (DUAL && nph > 1) ? col_tile % nph : 0;
  // This wavefront's block of 16 columns.  The first n_full column tiles own NWC blocks each, the
  // others NWC - 1 (the host evens out the blocks per CU that way when a launch needs more than
  // one round of workgroups); a wavefront without a block, also in a ragged last tile, only
  // helps to stage the activations and keeps the barriers.
  const int cb = col_tile < n_full ? col_tile * NWC + wcol
                                   : n_full * NWC + (col_tile - n_full) * (NWC - 1) + wcol;
  const bool active = (col_tile < n_full || wcol < NWC - 1) && cb * 16 < N;
  const int ncol = (active ? cb : 0) * 16 + ln;
  const bf16_t* wp[NB];
  if (DUAL) {
    wp[0] = W0 + static_cast<size_t>(ncol) * K + kbeg + kh * hlen + lg * 8;
    wp[NB - 1] = W1 + static_cast<size_t>(ncol) * K + kbeg + kh * hlen + lg * 8;
  } else {
    wp[0] = (ncol < N0 ? W0 + static_cast<size_t>(ncol) * K
                       : W1 + static_cast<size_t>(ncol - N0) * K) + kbeg + kh * hlen + lg * 8;
  }
  // the activation chunks this thread stages: same (group, row, chunk) in every phase
  const bf16_t* asrc[NCH];
  int adst[NCH];
  bool aval[NCH], ain[NCH];
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    int e = threadIdx.x + j * NW * 64;
    ain[j] = EVEN || e < TOT;
    if (!ain[j]) e = 0;
    const int h = e / (R * CPR), r = (e / CPR) % R, c = e % CPR;
    const int m = m0 + r;
    aval[j] = ain[j] && m < M;
    const int row = aval[j] ? (rows ? rows[m] : m) : 0;
    asrc[j] = A + static_cast<size_t>(row) * lda + kbeg + h * hlen + c * 8;
    adst[j] = h * R * LS + r * LS + (c ^ (r % 16)) * 8;
  }
  f32x4 acc[NB][RB];
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int i = 0; i < RB; ++i) acc[b][i] = f32x4{0.f, 0.f, 0.f, 0.f};
  // element offsets, within a 128-wide step, of this lane's four fragment chunks 4c + lg after
  // the slot permutation of its row (rows mb*16 + ln share row % 16 = ln)
  int fo[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) fo[c] = ((4 * c + lg) ^ ln) * 8;

#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (aval[j]) v = *reinterpret_cast<const uint4*>(asrc[j] + rot * KC);
    if (ain[j]) *reinterpret_cast<uint4*>(&As[0][0][adst[j]]) = v;
  }
  // weight pieces in flight: one whole phase (KC / 128 steps) ahead of the multiplications
  constexpr int NS = KC / 128;
  uint4 bn[NB][NS][4];
  if (active) {
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int t = 0; t < NS; ++t)
#pragma unroll
        for (int c = 0; c < 4; ++c)
          bn[b][t][c] = *reinterpret_cast<const uint4*>(wp[b] + rot * KC + t * 128 + c * 32);
  }
  __syncthreads();

  for (int ph = 0; ph < nph; ++ph) {
    const bool more = ph + 1 < nph;
    int pn = ph + 1 + rot;  // the phase fetched during this one
    if (pn >= nph) pn -= nph;
    uint4 av[NCH];
    if (more) {
#pragma unroll
      for (int j = 0; j < NCH; ++j) {
        av[j] = make_uint4(0u, 0u, 0u, 0u);
        if (aval[j]) av[j] = *reinterpret_cast<const uint4*>(asrc[j] + pn * KC);
      }
    }
    const bf16_t* ap = &As[ph & 1][kh][ln * LS];
    if (active) {
#pragma unroll
    for (int t = 0; t < NS; ++t) {
      uint4 bc[NB][4];
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int c = 0; c < 4; ++c) bc[b][c] = bn[b][t][c];
      if (more) {
        const int knext = pn * KC + t * 128;
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
          for (int c = 0; c < 4; ++c)
            bn[b][t][c] = *reinterpret_cast<const uint4*>(wp[b] + knext + c * 32);
      }
#pragma unroll
      for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int mb = 0; mb < RB; ++mb) {
          const bf16x8 af =
              *reinterpret_cast<const bf16x8*>(ap + mb * 16 * LS + t * 128 + fo[c]);
#pragma unroll
          for (int b = 0; b < NB; ++b)
            acc[b][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                af, __builtin_bit_cast(bf16x8, bc[b][c]), acc[b][mb], 0, 0, 0);
        }
    }
    }
    if (more) {
#pragma unroll
      for (int j = 0; j < NCH; ++j)
        if (ain[j]) *reinterpret_cast<uint4*>(&As[(ph + 1) & 1][0][adst[j]]) = av[j];
    }
    __syncthreads();
  }

  if (KH > 1) {
    // hand-over of the other groups' sums: [group - 1][column wavefront][matrix][accumulator
    // element][lane] (every LDS read of the activation tiles is behind the barrier that ended the
    // last phase); the first group adds them to its own in group order
    float* red = reinterpret_cast<float*>(&As[0][0][0]);
    static_assert((KH - 1) * NWC * NB * 4 * RB * 64 * sizeof(float) <= sizeof(As), "hand-over fits the tiles");
    if (kh > 0) {
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            red[((((kh - 1) * NWC + wcol) * NB + b) * (4 * RB) + mb * 4 + i) * 64 + lane] = acc[b][mb][i];
    }
    __syncthreads();
    if (kh > 0 || !active) return;
#pragma unroll
    for (int g = 1; g < KH; ++g)
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            acc[b][mb][i] += red[((((g - 1) * NWC + wcol) * NB + b) * (4 * RB) + mb * 4 + i) * 64 + lane];
  }

  if (!active) return;
  if (DUAL) {
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int m = m0 + mb * 16 + lg * 4 + i;
        if (m < M) {
          const float g = acc[0][mb][i], up = acc[NB - 1][mb][i];
          U[static_cast<size_t>(m) * N + ncol] = f32_to_bf16(g / (1.0f + expf(-g)) * up);
        }
      }
  } else {
    float* Cs = C + static_cast<size_t>(blockIdx.z) * M * N;
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int m = m0 + mb * 16 + lg * 4 + i;
        if (m < M) Cs[static_cast<size_t>(m) * N + ncol] = acc[0][mb][i];
      }
  }
}

// ------------------------------------------------------------------------------------
// LDS-direct MFMA kernels for many activation rows (refresh steps, the V projection of all
// response rows, batched sequences), where the work is bound by the matrix cores and by L2
// rather than by the weight stream.  Workgroup = WM x WN wavefronts, each (16*MI) rows x
// (16*NJ) columns of v_mfma_f32_16x16x32_bf16 accumulators.  Both operands reach LDS with
// global_load_lds_dwordx4 (no VGPR staging): a wavefront instruction copies 8 rows x 128
// contiguous bytes (64 values of the contraction index) into 1 KB of LDS in lane order, i.e.
// LDS holds [row][8 slots of 16 bytes]; the slot of chunk c of row r is c ^ (r % 8) so that
// the 16-byte fragment reads of 8 consecutive rows hit 8 different bank groups.  Two LDS
// stages: the loads of step t+1 are in flight while step t is multiplied.
// Rows beyond M read a valid row again and are dropped at the store.
//   fat: 2 x 4 wavefronts of 128 x 64 -> 256 x 256 tile (every byte pulled from L2 feeds 128
//        flops), 128 KB of LDS, one workgroup per CU: M >= fat_min_m.
//   mid: 2 x 2 wavefronts of  64 x 64 -> 128 x 128 tile, 64 KB of LDS, two workgroups per CU:
//        enough tiles to fill the chip when M is a few hundred rows.
constexpr int kFatM = 256, kFatN = 256, kFatK = 64;
constexpr int kMidM = 128, kMidN = 128;

//   PAIR = 1 (fused gate/up + SwiGLU, single slice): the tile's weight rows are BN/2 rows of W0
//        (gate) followed by the same BN/2 rows of W1 (up), so every lane ends up with the gate
//        and the up sum of the same output element and stores bf16(silu(gate) * up) to U[M, N]
//        (N = FFN width; the grid has N / (BN/2) column tiles).
template <int WM, int WN, int MI, int NJ, int PAIR = 0>
__device__ __forceinline__ void gemm_lds_body(const bf16_t* __restrict__ A, int lda,
                                              const int* __restrict__ rows, int M,
                                              const bf16_t* __restrict__ W0,
                                              const bf16_t* __restrict__ W1, int N0, int N, int K,
                                              int k_per_slice, float* __restrict__ C,
                                              bf16_t* __restrict__ U = nullptr) {
  constexpr int NWV = WM * WN;
  constexpr int BM = WM * MI * 16, BN = WN * NJ * 16;
  constexpr int LA = BM / 8 / NWV, LB = BN / 8 / NWV;  // load instructions per wavefront and step
  static_assert(BM % (8 * NWV) == 0 && BN % (8 * NWV) == 0, "loader must divide evenly");
  // [stage][activation rows, then weight rows][8 slots], 16 bytes each
  __shared__ __attribute__((aligned(1024))) uint4 lds[2][(BM + BN) * 8];
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int ln = lane % 16, lg = lane / 16;
  const int wm = wave / WN, wn = wave % WN;
  int col_tile, row_tile;
  xcd_tile_map(col_tile, row_tile);
  static_assert(!PAIR || NJ % 2 == 0, "gate and up column blocks come in pairs");
  const int m0 = row_tile * BM, n0 = col_tile * (PAIR ? BN / 2 : BN);
  const int kbeg = blockIdx.z * k_per_slice;
  const int klen = min(K, kbeg + k_per_slice) - kbeg;  // multiple of kFatK
  const int nkt = klen / kFatK;

  // loader: instruction q of an operand covers rows [8q, 8q+8); wavefront w issues
  // q = L*w .. L*w+L-1.  Lane l: row 8q + l/8, LDS slot l%8, global chunk (l%8) ^ (row%8).
  const bf16_t* asrc[LA];
  const bf16_t* bsrc[LB];
#pragma unroll
  for (int j = 0; j < LA; ++j) {
    const int r = 8 * (LA * wave + j) + lane / 8;
    const int chunk = (lane % 8) ^ (r % 8);
    int m = m0 + r;
    if (m >= M) m = M - 1;
    const int row = rows ? rows[m] : m;
    asrc[j] = A + static_cast<size_t>(row) * lda + kbeg + chunk * 8;
  }
#pragma unroll
  for (int j = 0; j < LB; ++j) {
    const int r = 8 * (LB * wave + j) + lane / 8;
    const int chunk = (lane % 8) ^ (r % 8);
    if (PAIR) {
      // LDS weight rows [0, BN/2): gate rows n0 + r; [BN/2, BN): up rows n0 + r - BN/2
      const int nn = n0 + (r % (BN / 2));  // < N: N % (BN/2) == 0
      bsrc[j] = (r < BN / 2 ? W0 : W1) + static_cast<size_t>(nn) * K + kbeg + chunk * 8;
    } else {
      const int nn = n0 + r;  // < N: N % BN == 0
      bsrc[j] = (nn < N0 ? W0 + static_cast<size_t>(nn) * K
                         : W1 + static_cast<size_t>(nn - N0) * K) + kbeg + chunk * 8;
    }
  }
#define DLLMC_LDS_ISSUE(stage, kt)                                                              \
  {                                                                                             \
    _Pragma("unroll") for (int j = 0; j < LA; ++j) __builtin_amdgcn_global_load_lds(            \
        asrc[j] + (kt) * kFatK, &lds[stage][(LA * wave + j) * 64], 16, 0, 0);                   \
    _Pragma("unroll") for (int j = 0; j < LB; ++j) __builtin_amdgcn_global_load_lds(            \
        bsrc[j] + (kt) * kFatK, &lds[stage][BM * 8 + (LB * wave + j) * 64], 16, 0, 0);          \
  }

  f32x4 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Two ways through a step.  One workgroup per CU (the 256 x 256 tile): a single barrier,
  // behind which everybody's loads of step kt have landed AND everybody has finished the
  // fragment reads of step kt-1, so the loads of step kt+1 are issued right after it into the
  // other stage.  Two workgroups per CU (128 x 128): the loads of step kt+1 go out before the
  // wait for step kt (a longer window for the shorter steps) and a second barrier at the end of
  // the step protects the stage they overwrite.
  constexpr bool ONE_BARRIER = NWV == 8;
  DLLMC_LDS_ISSUE(0, 0)
  for (int kt = 0; kt < nkt; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < nkt;
    if (ONE_BARRIER) {
      wait_vmcnt<0>();  // this wavefront's loads of step kt have landed
      __builtin_amdgcn_s_barrier();
      if (more) DLLMC_LDS_ISSUE(cur ^ 1, kt + 1)
    } else {
      if (more) {
        DLLMC_LDS_ISSUE(cur ^ 1, kt + 1)
        wait_vmcnt<LA + LB>();  // this wavefront's loads of step kt have landed
      } else {
        wait_vmcnt<0>();
      }
      // bare barrier (no memory fence: a fence would wait for the loads of step kt+1 as well)
      __builtin_amdgcn_s_barrier();  // ... and everybody else's
    }
    const uint4* la = &lds[cur][0];
    const uint4* lb = &lds[cur][BM * 8];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      const int c = kk * 4 + lg;  // 16-byte chunk of the 64-wide step this lane group multiplies
      bf16x8 af[MI], bf[NJ];
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const int r = wm * (MI * 16) + i * 16 + ln;
        af[i] = __builtin_bit_cast(bf16x8, la[r * 8 + (c ^ (r % 8))]);
      }
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        // PAIR: column blocks j < NJ/2 are gate, j >= NJ/2 the same columns of up
        const int r = PAIR ? (j / (NJ / 2)) * (BN / 2) + wn * (NJ / 2 * 16) + (j % (NJ / 2)) * 16 + ln
                           : wn * (NJ * 16) + j * 16 + ln;
        bf[j] = __builtin_bit_cast(bf16x8, lb[r * 8 + (c ^ (r % 8))]);
      }
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    // two-barrier scheme: all LDS reads of this stage are complete (their results fed the MFMAs
    // above) before the loads issued at the top of the next iteration overwrite it
    if (!ONE_BARRIER) __builtin_amdgcn_s_barrier();
  }
#undef DLLMC_LDS_ISSUE

  if (PAIR) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int m = m0 + wm * (MI * 16) + i * 16 + lg * 4 + e;
        if (m < M) {
#pragma unroll
          for (int j = 0; j < NJ / 2; ++j) {
            const float g = acc[i][j][e], up = acc[i][j + NJ / 2][e];
            U[static_cast<size_t>(m) * N + n0 + wn * (NJ / 2 * 16) + j * 16 + ln] =
                f32_to_bf16(g / (1.0f + expf(-g)) * up);
          }
        }
      }
    return;
  }
  float* Cs = C + static_cast<size_t>(blockIdx.z) * M * N;
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int m = m0 + wm * (MI * 16) + i * 16 + lg * 4 + e;
      if (m < M) {
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          Cs[static_cast<size_t>(m) * N + n0 + wn * (NJ * 16) + j * 16 + ln] = acc[i][j][e];
      }
    }
}

__global__ __launch_bounds__(512) void k_gemm_fat(const bf16_t* __restrict__ A, int lda,
                                                  const int* __restrict__ rows, int M,
                                                  const bf16_t* __restrict__ W0,
                                                  const bf16_t* __restrict__ W1, int N0, int N,
                                                  int K, int k_per_slice, float* __restrict__ C) {
  gemm_lds_body<2, 4, 8, 4>(A, lda, rows, M, W0, W1, N0, N, K, k_per_slice, C);
}

__global__ __launch_bounds__(256) void k_gemm_mid(const bf16_t* __restrict__ A, int lda,
                                                  const int* __restrict__ rows, int M,
                                                  const bf16_t* __restrict__ W0,
                                                  const bf16_t* __restrict__ W1, int N0, int N,
                                                  int K, int k_per_slice, float* __restrict__ C) {
  gemm_lds_body<2, 2, 4, 4>(A, lda, rows, M, W0, W1, N0, N, K, k_per_slice, C);
}

// fused gate/up + SwiGLU for many rows: N is the FFN width, grid.x = N / 128 (fat) or N / 64 (mid)
__global__ __launch_bounds__(512) void k_gemm_fat_swiglu(const bf16_t* __restrict__ A, int lda,
                                                         const int* __restrict__ rows, int M,
                                                         const bf16_t* __restrict__ Wg,
                                                         const bf16_t* __restrict__ Wu, int N, int K,
                                                         bf16_t* __restrict__ U) {
  gemm_lds_body<2, 4, 8, 4, 1>(A, lda, rows, M, Wg, Wu, N, N, K, K, nullptr, U);
}

__global__ __launch_bounds__(256) void k_gemm_mid_swiglu(const bf16_t* __restrict__ A, int lda,
                                                         const int* __restrict__ rows, int M,
                                                         const bf16_t* __restrict__ Wg,
                                                         const bf16_t* __restrict__ Wu, int N, int K,
                                                         bf16_t* __restrict__ U) {
  gemm_lds_body<2, 2, 4, 4, 1>(A, lda, rows, M, Wg, Wu, N, N, K, K, nullptr, U);
}

// 256 rows x (48 gate + 48 up) columns, four wavefronts of 64 x 96 each: for up to 256 rows and
// an FFN width that is a multiple of 48 the grid is one workgroup per 48 columns (12288 / 48 =
// 256, one per CU), where the 128 x 128 tiles leave half of the CUs with twice the work (a
// response refresh of 256 rows: 80 -> 69 us per layer; two workgroups of 128 x 96 per CU: 73).
__global__ __launch_bounds__(256) void k_gemm_tall_swiglu(const bf16_t* __restrict__ A, int lda,
                                                          const int* __restrict__ rows, int M,
                                                          const bf16_t* __restrict__ Wg,
                                                          const bf16_t* __restrict__ Wu, int N, int K,
                                                          bf16_t* __restrict__ U) {
  gemm_lds_body<4, 1, 4, 6, 1>(A, lda, rows, M, Wg, Wu, N, N, K, K, nullptr, U);
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
// The process default (guarded by a mutex: contexts copy it at creation, dllmc_set_gemm_tuning
// writes it) and the settings in force on this thread: a context's own copy while one of its
// calls runs (TuningScope), else a snapshot of the default taken by the calling launcher.
GemmTuning g_default_tune;
std::mutex g_tune_mu;
thread_local const GemmTuning* t_scope = nullptr;
thread_local GemmTuning t_snapshot;
const GemmTuning& tune() {
  if (t_scope) return *t_scope;
  std::lock_guard<std::mutex> lock(g_tune_mu);
  t_snapshot = g_default_tune;
  return t_snapshot;
}
#define g_tune (tune())

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <int NW, int KC, int DUAL, int KH = 1, int RB = 4>
void launch_stream(dim3 grid, hipStream_t st, const bf16_t* A, int lda, const int* rows, int M,
                   const bf16_t* W0, const bf16_t* W1, int N0, int N, int K, int kps, float* C,
                   bf16_t* U, int n_full = -1) {
  hipLaunchKernelGGL((k_gemm_stream<NW, KC, DUAL, KH, RB>), grid, dim3(NW * 64), 0, st, A, lda, rows, M, W0,
                     W1, N0, N, K, kps, C, U, n_full < 0 ? static_cast<int>(grid.x) : n_full);
}

bool stream_shape_ok(int dtype, const void* A, int lda, const void* W0, const void* W1, int K) {
  return dtype == 1 && (K % 128 == 0) && (lda % 8 == 0) && aligned16(A) && aligned16(W0) &&
         (W1 == nullptr || aligned16(W1));
}
}  // namespace

static thread_local bool t_last_stream = false;
bool gemm_last_was_stream() { return t_last_stream; }
void gemm_clear_last_stream() { t_last_stream = false; }

#undef g_tune
GemmTuning gemm_default_tuning() {
  std::lock_guard<std::mutex> lock(g_tune_mu);
  return g_default_tune;
}
TuningScope::TuningScope(const GemmTuning* t) : prev(t_scope) { t_scope = t; }
TuningScope::~TuningScope() { t_scope = prev; }

void gemm_set_tile_min_m(int m) { std::lock_guard<std::mutex> lock(g_tune_mu); if (m > 0) g_default_tune.tile_min_m = m; }
void gemm_set_tall_max_m(int m) { std::lock_guard<std::mutex> lock(g_tune_mu); if (m >= 0) g_default_tune.tall_max_m = m; }
void gemm_set_fat_min_m(int m) { std::lock_guard<std::mutex> lock(g_tune_mu); if (m > 0) g_default_tune.fat_min_m = m; }

void gemm_set_tuning(int nw, int nw_dual, int force_s, int target_wg) {
  std::lock_guard<std::mutex> lock(g_tune_mu);
  if (nw == 4 || nw == 8) g_default_tune.nw = nw;
  if (nw_dual == 4 || nw_dual == 8 || nw_dual == 104 || nw_dual == 106 || nw_dual == 108)
    g_default_tune.nw_dual = nw_dual;
  if (force_s >= 0) g_default_tune.force_s = force_s;
  if (target_wg > 0) g_default_tune.target_wg = target_wg;
}
#define g_tune (tune())

// Which kernel, how many slices of the contraction index and how long a slice: pure host logic.
struct GemmPlan {
  int kind;  // 0 nothing fits, 1 plain, 2 streaming, 3 256x256 LDS-direct, 4 128x128 LDS-direct,
             // 5 / 6 streaming with 256 / 128 rows per workgroup
  int S, kps, KC, nt, mt;
};

GemmPlan plan_gemm(int dtype, bool operands_aligned, int lda, int M, int N, int N0, int K,
                   size_t c_capacity) {
  GemmPlan p{0, 0, 0, 0, 0, 0};
  const size_t MN = static_cast<size_t>(M) * N;
  if (M <= 0 || N <= 0 || K <= 0 || c_capacity < MN) return p;
  // most slices the caller's buffer can hold
  const int s_cap = static_cast<int>(c_capacity / MN < static_cast<size_t>(kMaxSlices)
                                         ? c_capacity / MN : static_cast<size_t>(kMaxSlices));
  const int NW = g_tune.nw;
  const int BN = 16 * NW;
  const bool mfma_ok = dtype == 1 && operands_aligned && (K % 128 == 0) && (lda % 8 == 0);
  if (!(mfma_ok && N % BN == 0 && N0 % BN == 0)) {
    p.kind = 1; p.S = 1; p.kps = K; p.nt = (N + 63) / 64; p.mt = (M + 63) / 64;
    return p;
  }
  if (M >= g_tune.fat_min_m && N % kFatN == 0 && N0 % kFatN == 0 && K % kFatK == 0) {
    p.kind = 3;
    p.mt = (M + kFatM - 1) / kFatM;
    p.nt = N / kFatN;
    // One workgroup per CU (128 KB of LDS).  Choose the slice count with the lowest estimated
    // time: rounds of tiles over the 256 CUs at the measured ~1.1 PFLOP/s steady rate of this
    // kernel, plus writing and re-reading the float32 partial sums at ~5 TB/s.
    int S = 1;
    if (g_tune.force_s > 0) {
      S = g_tune.force_s;
    } else {
      double best = 1e30;
      for (int sl = 1; sl <= s_cap; ++sl) {
        if (K / sl < 8 * kFatK) break;
        const int kslice = ((K + sl - 1) / sl + kFatK - 1) / kFatK * kFatK;
        const int rounds = (p.mt * p.nt * sl + 255) / 256;
        const double t_tile = 2.0 * kFatM * kFatN * kslice / (1.1e15 / 256.0);
        const double t_part = sl > 1 ? 2.0 * sl * static_cast<double>(MN) * 4.0 / 5e12 : 0.0;
        const double cost = rounds * t_tile + t_part;
        if (cost < best * 0.98) { best = cost; S = sl; }
      }
    }
    S = S < 1 ? 1 : (S > s_cap ? s_cap : S);
    p.kps = ((K + S - 1) / S + kFatK - 1) / kFatK * kFatK;
    if (p.kps > K) p.kps = K;
    p.S = (K + p.kps - 1) / p.kps;
    return p;
  }
  if (M >= g_tune.tile_min_m && M <= g_tune.tall_max_m && g_tune.tall_max_m >= 256) {
    p.kind = 5;
    p.KC = 128;
    p.mt = (M + 255) / 256;
    p.nt = N / BN;
    int S = g_tune.force_s > 0 ? g_tune.force_s : (g_tune.target_wg + p.mt * p.nt - 1) / (p.mt * p.nt);
    S = S < 1 ? 1 : (S > s_cap ? s_cap : S);
    p.kps = ((K + S - 1) / S + p.KC - 1) / p.KC * p.KC;
    if (p.kps > K) p.kps = K;
    p.S = (K + p.kps - 1) / p.kps;
    return p;
  }
  if (M >= g_tune.tile_min_m && N % kMidN == 0 && N0 % kMidN == 0 && K % kFatK == 0) {
    p.kind = 4;
    p.mt = (M + kMidM - 1) / kMidM;
    p.nt = N / kMidN;
    // Slices: as many as keep the launch within one workgroup per CU, rounded down (every
    // slice costs its float32 partial sums twice, written here and read by the row kernel: a
    // slightly underfilled chip is cheaper than a fifth slice), at least 8 steps of 64 each
    // unless that leaves more than a fifth of the CUs without a workgroup
    const int tiles = p.mt * p.nt;
    int S = g_tune.target_wg / tiles;
    if (5 * tiles * S <= 4 * g_tune.target_wg) ++S;
    if (g_tune.force_s > 0) S = g_tune.force_s;
    S = S < 1 ? 1 : (S > s_cap ? s_cap : S);
    p.kps = ((K + S - 1) / S + kFatK - 1) / kFatK * kFatK;
    if (p.kps < 8 * kFatK) p.kps = 8 * kFatK;
    if (p.kps > K) p.kps = K;
    p.S = (K + p.kps - 1) / p.kps;
    return p;
  }
  const bool rows128 = g_tune.tall_max_m >= 128 && M > 64 && NW == 8;
  p.kind = rows128 ? 6 : 2;
  p.KC = (K % 256 == 0) ? 256 : 128;
  p.mt = rows128 ? (M + 127) / 128 : (M + 63) / 64;
  p.nt = N / BN;
  int S = g_tune.force_s > 0 ? g_tune.force_s : (g_tune.target_wg + p.mt * p.nt - 1) / (p.mt * p.nt);
  S = S < 1 ? 1 : (S > s_cap ? s_cap : S);
  p.kps = ((K + S - 1) / S + p.KC - 1) / p.KC * p.KC;
  if (p.kps > K) p.kps = K;
  p.S = (K + p.kps - 1) / p.kps;
  return p;
}

int gemm_plan_slices(int dtype, int M, int N, int N0, int K, size_t c_capacity) {
  return plan_gemm(dtype, true, K, M, N, N0, K, c_capacity).S;
}

int launch_gemm(int dtype, const void* A, int lda, const int* rows, int M, const void* W0,
                const void* W1, int N0, int N, int K, float* c_part, size_t c_capacity,
                hipStream_t st) {
  t_last_stream = false;
  if (M <= 0 || N <= 0) return 1;
  const bool al = aligned16(A) && aligned16(W0) && (W1 == nullptr || aligned16(W1));
  const GemmPlan p = plan_gemm(dtype, al, lda, M, N, N0, K, c_capacity);
  if (p.kind == 0 || static_cast<size_t>(p.S) * M * N > c_capacity) return 0;  // nothing launched
  t_last_stream = p.kind == 2 || p.kind == 5 || p.kind == 6;
  const bf16_t* a = static_cast<const bf16_t*>(A);
  const bf16_t* w0 = static_cast<const bf16_t*>(W0);
  const bf16_t* w1 = static_cast<const bf16_t*>(W1);
  const dim3 grid(p.nt, p.mt, p.S);
  switch (p.kind) {
    case 1:
      if (dtype == 1)
        hipLaunchKernelGGL(k_gemm_simple<bf16_t>, grid, dim3(256), 0, st, a, lda, rows, M, w0, w1, N0,
                           N, K, c_part);
      else
        hipLaunchKernelGGL(k_gemm_simple<float>, grid, dim3(256), 0, st,
                           static_cast<const float*>(A), lda, rows, M,
                           static_cast<const float*>(W0), static_cast<const float*>(W1), N0, N, K,
                           c_part);
      break;
    case 3:
      hipLaunchKernelGGL(k_gemm_fat, grid, dim3(512), 0, st, a, lda, rows, M, w0, w1, N0, N, K, p.kps,
                         c_part);
      break;
    case 4:
      hipLaunchKernelGGL(k_gemm_mid, grid, dim3(256), 0, st, a, lda, rows, M, w0, w1, N0, N, K,
                         p.kps, c_part);
      break;
    case 6:
      if (p.KC == 256)
        launch_stream<8, 256, 0, 1, 8>(grid, st, a, lda, rows, M, w0, w1, N0, N, K, p.kps, c_part, nullptr);
      else
        launch_stream<8, 128, 0, 1, 8>(grid, st, a, lda, rows, M, w0, w1, N0, N, K, p.kps, c_part, nullptr);
      break;
    case 5:
      if (g_tune.nw == 8)
        launch_stream<8, 128, 0, 1, 16>(grid, st, a, lda, rows, M, w0, w1, N0, N, K, p.kps, c_part, nullptr);
      else
        launch_stream<4, 128, 0, 1, 16>(grid, st, a, lda, rows, M, w0, w1, N0, N, K, p.kps, c_part, nullptr);
      break;
    default: {
#define DLLMC_GS(NWv, KCv) \
  launch_stream<NWv, KCv, 0>(grid, st, a, lda, rows, M, w0, w1, N0, N, K, p.kps, c_part, nullptr)
      if (g_tune.nw == 8) {
        if (p.KC == 256) DLLMC_GS(8, 256); else DLLMC_GS(8, 128);
      } else {
        if (p.KC == 256) DLLMC_GS(4, 256); else DLLMC_GS(4, 128);
      }
#undef DLLMC_GS
    }
  }
  return p.S;
}

bool launch_gemm_swiglu(int dtype, const void* A, int lda, const int* rows, int M,
                        const void* w_gate, const void* w_up, int m, int K, void* u,
                        hipStream_t st) {
  if (M <= 0 || m <= 0) return true;
  const int KC = (K % 256 == 0) ? 256 : 128;
  // two wavefront groups over the two halves of K when the halves are whole phases
  const int KH = (g_tune.nw_dual >= 100 && K % (2 * KC) == 0) ? 2 : 1;
  int NW = g_tune.nw_dual % 100;  // wavefronts per workgroup
  if (KH == 1 && NW == 6) NW = 3;  // the two-group shape without the split: one group of its width
  const int BN = 16 * NW / KH;
  if (M >= g_tune.tile_min_m && stream_shape_ok(dtype, A, lda, w_gate, w_up, K) && K % kFatK == 0) {
    // many rows: the LDS-direct tile kernels with paired gate/up column blocks, one slice
    const bool fat = M >= g_tune.fat_min_m && m % (kFatN / 2) == 0;
    const bool tall = !fat && M <= 256 && m % 48 == 0;
    if (fat || tall || m % (kMidN / 2) == 0) {
      t_last_stream = false;
      const bf16_t* a = static_cast<const bf16_t*>(A);
      const bf16_t* w0 = static_cast<const bf16_t*>(w_gate);
      const bf16_t* w1 = static_cast<const bf16_t*>(w_up);
      bf16_t* uo = static_cast<bf16_t*>(u);
      if (tall)
        hipLaunchKernelGGL(k_gemm_tall_swiglu, dim3(m / 48, 1, 1), dim3(256), 0, st, a, lda, rows, M,
                           w0, w1, m, K, uo);
      else if (fat)
        hipLaunchKernelGGL(k_gemm_fat_swiglu, dim3(m / (kFatN / 2), (M + kFatM - 1) / kFatM, 1),
                           dim3(512), 0, st, a, lda, rows, M, w0, w1, m, K, uo);
      else
        hipLaunchKernelGGL(k_gemm_mid_swiglu, dim3(m / (kMidN / 2), (M + kMidM - 1) / kMidM, 1),
                           dim3(256), 0, st, a, lda, rows, M, w0, w1, m, K, uo);
      return true;
    }
  }
  if (!(stream_shape_ok(dtype, A, lda, w_gate, w_up, K) && m % 16 == 0) || M > 128) return false;
  const bool rows128 = g_tune.tall_max_m >= 128 && M > 64 && NW == 6 && KH == 2 && K % 256 == 0;
  dim3 grid((m + BN - 1) / BN, rows128 ? 1 : (M + 63) / 64, 1);
  // More workgroups than CUs (one runs per CU at a time): rather than rounds of full tiles with
  // a last round that leaves CUs idle (FFN width 18944: 395 tiles of 48 columns, 2 x 48 columns
  // on the busiest CU), whole rounds of workgroups of which the first n_full own NWC blocks of
  // 16 columns and the others NWC - 1 (512 workgroups, 160 of them with 3 blocks: 48 + 32
  // columns; 91 -> 86 us).  128-wide phases, which let two such workgroups share a CU, measured
  // slower (90 us).
  int n_full = -1;
  {
    static const int cus = [] {
      int dev = 0, n = 0;
      if (hipGetDevice(&dev) != hipSuccess ||
          hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
        n = 256;
      return n;
    }();
    const int NWC = NW / KH, nblk = m / 16;
    const int G = (static_cast<int>(grid.x) + cus - 1) / cus * cus;
    if (grid.y == 1 && NWC >= 2 && static_cast<int>(grid.x) > cus &&
        static_cast<long long>(G) * (NWC - 1) <= nblk) {
      n_full = nblk - G * (NWC - 1);
      grid.x = G;
    }
  }
  t_last_stream = true;
  const bf16_t* a = static_cast<const bf16_t*>(A);
  const bf16_t* w0 = static_cast<const bf16_t*>(w_gate);
  const bf16_t* w1 = static_cast<const bf16_t*>(w_up);
  bf16_t* uo = static_cast<bf16_t*>(u);
#define DLLMC_GD(NWv, KCv, KHv) \
  launch_stream<NWv, KCv, 1, KHv>(grid, st, a, lda, rows, M, w0, w1, m, m, K, K, nullptr, uo, n_full)
  if (rows128) {
    launch_stream<6, 128, 1, 2, 8>(grid, st, a, lda, rows, M, w0, w1, m, m, K, K, nullptr, uo, n_full);
    return true;
  }
  switch (NW * 10 + KH) {
    case 62: if (KC == 256) DLLMC_GD(6, 256, 2); else DLLMC_GD(6, 128, 2); break;
    case 82: if (KC == 256) DLLMC_GD(8, 256, 2); else DLLMC_GD(8, 128, 2); break;
    case 31: if (KC == 256) DLLMC_GD(3, 256, 1); else DLLMC_GD(3, 128, 1); break;
    case 81: if (KC == 256) DLLMC_GD(8, 256, 1); else DLLMC_GD(8, 128, 1); break;
    case 42: if (KC == 256) DLLMC_GD(4, 256, 2); else DLLMC_GD(4, 128, 2); break;
    default: if (KC == 256) DLLMC_GD(4, 256, 1); else DLLMC_GD(4, 128, 1); break;
  }
#undef DLLMC_GD
  return true;
}

#undef g_tune

}  // namespace dllmc
