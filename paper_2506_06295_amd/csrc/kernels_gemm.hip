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
#include <type_traits>

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
  // (the wavefront index as a scalar: the column block and whether the wavefront has one are
  // then scalar too)
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64), lane = threadIdx.x % 64;
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
  // A wavefront without a block runs the same phases as the others (no branch in the loop: see
  // below), on the first 256 contraction values of block 0 over and over: cache hits.
  const int kmul = active ? 1 : 0;
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
    const int mm = min(m, M - 1);  // chunks without a row of their own read a valid one and are zeroed
    const int row = rows ? rows[mm] : mm;
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

  // The activation chunks of the first phase: every load goes out before the first one is used
  // (rows past M and chunks past the tile read a valid row and are zeroed or dropped afterwards --
  // a load under "if (row < M)" is a basic block of its own, and the store that follows it then
  // waits for it before the next load is issued: one trip to memory per chunk), and so do the
  // first weight pieces, before the activations are waited for.
  uint4 a0[NCH];
#pragma unroll
  for (int j = 0; j < NCH; ++j) a0[j] = *reinterpret_cast<const uint4*>(asrc[j] + rot * KC);
  // Weight pieces in flight: one whole phase (KC / 128 steps) ahead of the multiplications, in
  // two register sets that swap roles from phase to phase; a phase is straight-line code (the
  // last one, which fetches nothing, is a variant of its own; a wavefront without a column block
  // loads and multiplies like the others), and its barrier is a bare s_barrier behind a wait for
  // the LDS operations only.  Each of these matters, because the wait counter counts loads in
  // order and the compiler has to place its waits from what it can prove: (1) with one set,
  // refilled piece by piece behind a copy of the piece being multiplied, it carries the set
  // through the loop by copying the freshly loaded registers into place at the end of the body,
  // and waits for every load of the phase to do so; (2) a __syncthreads() waits for every load in
  // flight; (3) behind a join of paths that issued different numbers of loads (wavefronts
  // without a block, the last phase) the activation chunks, the oldest loads of a phase, are
  // waited for as if no younger load existed.  With any one of the three nothing stayed in
  // flight across a phase boundary and a phase cost a full trip to memory (adaptive step of
  // `llada8b` 5.45 -> 5.29 ms).  Three sets, two phases ahead, measured no better than two; nor
  // did the first weight pieces issued ahead of the row list's wait (the activation chunks,
  // which come from L2, then return behind them).
  constexpr int NS = KC / 128;
  uint4 bset0[NB][NS][4], bset1[NB][NS][4];
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int t = 0; t < NS; ++t)
#pragma unroll
      for (int c = 0; c < 4; ++c)
        bset0[b][t][c] = *reinterpret_cast<const uint4*>(wp[b] + (rot * KC + t * 128) * kmul + c * 32);
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    if (!aval[j]) a0[j] = make_uint4(0u, 0u, 0u, 0u);
    if (ain[j]) *reinterpret_cast<uint4*>(&As[0][0][adst[j]]) = a0[j];
  }
  __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this wavefront's stores are complete
  __builtin_amdgcn_s_barrier();

  // one phase: multiply from `cur`; MORE: fetch the next phase's activation chunks and, as the
  // steps go by, its weight pieces into `nxt`
  auto phase = [&](auto more_tag, int ph, const uint4 (&cur)[NB][NS][4], uint4 (&nxt)[NB][NS][4]) {
    constexpr bool MORE = decltype(more_tag)::value;
    int pn = ph + 1 + rot;  // the phase fetched during this one
    if (pn >= nph) pn -= nph;
    uint4 av[NCH];
    if (MORE) {
#pragma unroll
      for (int j = 0; j < NCH; ++j) av[j] = *reinterpret_cast<const uint4*>(asrc[j] + pn * KC);
    }
    const bf16_t* ap = &As[ph & 1][kh][ln * LS];
#pragma unroll
    for (int t = 0; t < NS; ++t) {
      if (MORE) {
        const int knext = (pn * KC + t * 128) * kmul;
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
          for (int c = 0; c < 4; ++c)
            nxt[b][t][c] = *reinterpret_cast<const uint4*>(wp[b] + knext + c * 32);
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
                af, __builtin_bit_cast(bf16x8, cur[b][t][c]), acc[b][mb], 0, 0, 0);
        }
    }
    if (MORE) {
#pragma unroll
      for (int j = 0; j < NCH; ++j) {
        if (!aval[j]) av[j] = make_uint4(0u, 0u, 0u, 0u);
        if (ain[j]) *reinterpret_cast<uint4*>(&As[(ph + 1) & 1][0][adst[j]]) = av[j];
      }
    }
    // this wavefront's fragment reads of the phase and its stores for the next one are complete
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
  };
  {
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;
    int ph = 0;
    for (; ph + 2 < nph; ph += 2) {
      phase(yes{}, ph, bset0, bset1);
      phase(yes{}, ph + 1, bset1, bset0);
    }
    if (nph - ph == 2) {
      phase(yes{}, ph, bset0, bset1);
      phase(no{}, ph + 1, bset1, bset0);
    } else if (nph - ph == 1) {
      phase(no{}, ph, bset0, bset1);
    }
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
// stages (128-row tiles) or five slots of one operand block (256-row tiles): later steps'
// loads are in flight while step t is multiplied.
// Rows beyond M read a valid row again and are dropped at the store.
//   fat: 2 x 4 wavefronts of 128 x 64 -> 256 x 256 tile (every byte pulled from L2 feeds 128
//        flops), all 160 KB of LDS, one workgroup per CU: M >= fat_min_m.
//   mid: 2 x 2 wavefronts of  64 x 64 -> 128 x 128 tile, 64 KB of LDS, two workgroups per CU:
//        enough tiles to fill the chip when M is a few hundred rows.
constexpr int kFatM = 256, kFatN = 256, kFatK = 64;
constexpr int kMidM = 128, kMidN = 128;

//   PAIR = 1 (fused gate/up + SwiGLU, single slice): the tile's weight rows are BN/2 rows of W0
//        (gate) followed by the same BN/2 rows of W1 (up), so every lane ends up with the gate
//        and the up sum of the same output element and stores bf16(silu(gate) * up) to U[M, N]
//        (N = FFN width; the grid has N / (BN/2) column tiles).
//   EPI = 1 / 2 (single slice): the step's work on the tile is finished in the epilogue, nothing
//        goes through float32 slices and no row kernel follows.
//        1: V-verify (Sec. 3.2.2, Eq. cos_sim).  Activation row i is carried row i of the step
//           (position first + i % per_seq of sequence i / per_seq); the sums are rounded to bf16,
//           scored against the cached row they replace (per row and 64-column block the three
//           sums go to `part`, laid out as for k_vverify_tile) and written to the cache.
//        2: Q | K with RoPE.  A tile column block of 128 is one head, two column wavefronts; the
//           weight rows are dealt so that a lane's accumulators j and j + 2 hold the rotation pair
//           (t, t + 64): rotated in registers, query heads go to the compact q_out[i] and the
//           other heads to cache row rows[i].
struct TileEpilogue {
  // EPI = 1
  int first, per_seq, n, L_p;
  bf16_t* cache;         // V cache [*, N] (EPI 1); K (or V) cache [*, d_kv] (EPI 2)
  float* part;           // tile sums, or nullptr: no scoring
  int part_stride, metric;
  const int* rmap;       // paged layout: cache row of a logical row, or nullptr
  // EPI = 2
  const float2* tab;     // [n][64] (cos, sin)
  bf16_t* q_out;         // [M, N0]
  int d_kv, rope_second;
};

template <int WM, int WN, int MI, int NJ, int PAIR = 0, int EPI = 0>
__device__ __forceinline__ void gemm_lds_body(const bf16_t* __restrict__ A, int lda,
                                              const int* __restrict__ rows, int M,
                                              const bf16_t* __restrict__ W0,
                                              const bf16_t* __restrict__ W1, int N0, int N, int K,
                                              int k_per_slice, float* __restrict__ C,
                                              bf16_t* __restrict__ U = nullptr,
                                              const TileEpilogue* ep = nullptr) {
  constexpr int NWV = WM * WN;
  constexpr int BM = WM * MI * 16, BN = WN * NJ * 16;
  constexpr int LA = BM / 8 / NWV, LB = BN / 8 / NWV;  // load instructions per wavefront and step
  static_assert(BM % (8 * NWV) == 0 && BN % (8 * NWV) == 0, "loader must divide evenly");
  // [stage][activation rows, then weight rows][8 slots], 16 bytes each
  // (EPI: followed by two ints per tile row, see below.  One LDS object on purpose: with a second
  // one the compiler can no longer tell the fragment reads from the loads in flight into the
  // other stage and waits for those before every read.)
  constexpr int kStage = (BM + BN) * 8;
  // Two ways through the contraction.  Two workgroups per CU (128 x 128, four wavefronts): two
  // stages of both operands; the loads of step kt+1 go out before the wait for step kt and a
  // second barrier at the end of the step protects the stage they overwrite (the five-slot loop
  // with 16 KB slots measured 3-8 % slower there).  One workgroup per CU (256-row tiles): five
  // slots of one operand block each (all 160 KB of the CU), one barrier per step, see the main
  // loop.
  constexpr bool ONE_BARRIER = BM == 256;
  constexpr int kSlot = (BM > BN ? BM : BN) * 8;
  constexpr int kLdsTotal = ONE_BARRIER ? 5 * kSlot : 2 * kStage + (EPI ? 2 * BM / 4 : 0);
  static_assert(kLdsTotal * sizeof(uint4) <= 160 * 1024, "LDS of one CU");
  __shared__ __attribute__((aligned(1024))) uint4 lds_all[kLdsTotal];
  uint4 (*lds)[kStage] = reinterpret_cast<uint4 (*)[kStage]>(lds_all);
  // (five slots: the table lives in the last slot, written after the main loop)
  int (*meta)[BM] = reinterpret_cast<int (*)[BM]>(lds_all + (ONE_BARRIER ? 4 * kSlot : 2 * kStage));
  // (the wavefront index as a scalar: the LDS addresses of the loads, which go through M0, are then
  // scalar arithmetic instead of vector instructions and v_readfirstlane in every step)
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64), lane = threadIdx.x % 64;
  const int ln = lane % 16, lg = lane / 16;
  const int wm = wave / WN, wn = wave % WN;
  int col_tile, row_tile;
  xcd_tile_map_blocked(col_tile, row_tile);
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
    int row;
    if (EPI == 1) row = (m / ep->per_seq) * ep->n + ep->first + m % ep->per_seq;
    else row = rows ? rows[m] : m;
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
      // EPI 2: LDS weight row wn*64 + j*16 + c is column (j/2)*64 + (wn%2)*32 + (j%2)*16 + c of head
      // wn/2 of the tile, so that a lane's accumulators j and j + 2 are a rotation pair
      const int rp = EPI == 2 ? (r / 128) * 128 + ((r % 64) / 32) * 64 + ((r / 64) % 2) * 32 + r % 32 : r;
      const int nn = n0 + rp;  // < N: N % BN == 0
      bsrc[j] = (nn < N0 ? W0 + static_cast<size_t>(nn) * K
                         : W1 + static_cast<size_t>(nn - N0) * K) + kbeg + chunk * 8;
    }
  }
  // EPI: what the epilogue needs to know about the tile's rows, looked up here so that the trips
  // to memory pass under the main loop.  EPI 1: cache row, index of the row's score (-1: not
  // scored); EPI 2: position in the sequence, cache row.
  // (with five slots there is no room for the table during the main loop: the thread keeps its
  // row's two entries in registers and writes them to the last slot afterwards)
  int meta_r0 = 0, meta_r1 = 0;
  if (EPI != 0 && threadIdx.x < BM) {
    const int r = threadIdx.x;
    const int m = min(m0 + r, M - 1);
    if (EPI == 1) {
      const int seq = m / ep->per_seq, pos = ep->first + m % ep->per_seq;
      const int row = seq * ep->n + pos;
      meta_r0 = ep->rmap ? ep->rmap[row] : row;
      meta_r1 = (m0 + r < M && ep->part != nullptr && pos >= ep->L_p)
                                 ? seq * (ep->n - ep->L_p) + (pos - ep->L_p) : -1;
    } else {
      const int row = rows ? rows[m] : m;
      meta_r0 = row % ep->n;
      meta_r1 = ep->rmap ? ep->rmap[row] : row;
    }
    if (!ONE_BARRIER) {
      meta[0][r] = meta_r0;
      meta[1][r] = meta_r1;
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

  // The walk over the contraction index starts at a step that depends on the XCD and wraps
  // around: the workgroups of a launch run nearly in step and their rows are a multiple of 4 KB
  // apart, so unrotated every load in flight on the chip has the same address bits below the row
  // pitch and the memory channels are loaded unevenly (4096 x 4096 x 16384: 959 -> 1097 TFLOP/s).
  // The workgroups of one XCD keep a common start, they share operand blocks through its L2.
  const int rot = (((blockIdx.x + gridDim.x * blockIdx.y) & 7) * nkt) >> 3;
  auto kof = [&](int kt) { const int k = kt + rot; return (k < nkt ? k : k - nkt) * kFatK; };
  if (ONE_BARRIER) {
    // Five slots of one operand block (256 rows x 64 contraction values) each.  Blocks are
    // numbered in the order they are needed, A(0), B(0), A(1), B(1), ...; block p lives in slot
    // p % 5.  While step kt multiplies A(kt) and B(kt), A(kt+1), B(kt+1) and A(kt+2) are landing
    // or have landed, and the barrier of step kt -- everybody has finished the fragment reads of
    // step kt, everybody's loads up to B(kt+1) have landed -- makes room for B(kt+2) and A(kt+3):
    // 96 KB in flight per CU instead of the 64 KB of two stages, A(kt+2) stays in flight across
    // the barrier (the memory pipeline never drains), and the new loads go out two per MFMA unit
    // over the following step instead of all behind the barrier, where sixteen wavefronts'
    // worth of address work kept the matrix pipes waiting (the 256 x 256 x 64 step: 1.12 ->
    // 1.38 PFLOP/s on 12288 x 4096 x 12288).
    //
    // The step's MFMAs go in units of 4 activation blocks x NJ weight blocks x 32 contraction
    // values, and the fragments of unit u + 1 are read from LDS into a second register set while
    // the MFMAs of unit u run: the wavefronts of a workgroup leave every barrier together, so
    // without this they all read fragments at the same time and then all multiply, and the
    // matrix pipes idle for an LDS round trip in front of every group of MFMAs.  The barrier
    // sits in front of the step's last unit.
    constexpr int AG = 4;            // activation fragments per unit
    constexpr int UH = MI / AG;      // units per 32 contraction values
    constexpr int NU = 2 * UH;       // units per step
    constexpr int NL = LA + LB;      // loads per wavefront and step: B(kt+2) first, then A(kt+3)
    static_assert(MI % AG == 0, "units of four activation blocks");
    auto issue_a = [&](int slot, int kt, int j0, int j1) {
      const int ko = kof(kt);
#pragma unroll
      for (int j = j0; j < j1; ++j)
        __builtin_amdgcn_global_load_lds(asrc[j] + ko, &lds_all[slot * kSlot + (LA * wave + j) * 64],
                                         16, 0, 0);
    };
    // Weight loads take their address as a scalar base + a 32-bit lane offset (no vector
    // arithmetic per load): the 8 rows of one load instruction are consecutive rows of one
    // matrix (the tile origins and the W0 | W1 boundary are multiples of 8), so the lane offset
    // -- row lane/8, chunk (lane%8) ^ (lane/8) -- is the same for every instruction and the base
    // is lane 0's address.  The scalar sum is re-read as a wavefront constant and the offset
    // passes through an empty asm so that the compiler neither folds the two into per-lane
    // 64-bit pointers outside the loop nor moves the zero-extension away from the load, either
    // of which loses the addressing form.
    const char* bbase[LB];
#pragma unroll
    for (int j = 0; j < LB; ++j) bbase[j] = wave_uniform_ptr(reinterpret_cast<const char*>(bsrc[j]));
    const uint32_t boff =
        static_cast<uint32_t>(reinterpret_cast<const char*>(bsrc[0]) - bbase[0]);
    auto issue_b = [&](int slot, int kt, int j0, int j1) {
      const int ko = kof(kt);
#pragma unroll
      for (int j = j0; j < j1; ++j) {
        const char* bp = wave_uniform_ptr(bbase[j] + ko * static_cast<int>(sizeof(bf16_t)));
        uint32_t o = boff;
        asm volatile("" : "+v"(o));
        __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint4*>(bp + o),
                                         &lds_all[slot * kSlot + (LB * wave + j) * 64], 16, 0, 0);
      }
    };
    // loads [i0, i1) of the NL that the barrier of step kb makes room for (slots sa_b, sb_b of that
    // step's operands)
    auto issue_some = [&](int kb, int sa_b, int sb_b, int i0, int i1) {
      const int b0 = min(i0, LB), b1 = min(i1, LB);
      const int a0 = max(i0, LB) - LB, a1 = max(i1, LB) - LB;
      if (b1 > b0 && kb + 2 < nkt) issue_b(sa_b, kb + 2, b0, b1);
      if (a1 > a0 && kb + 3 < nkt) issue_a(sb_b, kb + 3, a0, a1);
    };
    bf16x8 af[2][AG], bf[2][NJ];
    auto read_a = [&](int slot, int u, bf16x8 (&dst)[AG]) {
      const uint4* la = &lds_all[slot * kSlot];
      const int c = (u / UH) * 4 + lg;
#pragma unroll
      for (int i = 0; i < AG; ++i) {
        const int r = wm * (MI * 16) + ((u % UH) * AG + i) * 16 + ln;
        dst[i] = __builtin_bit_cast(bf16x8, la[r * 8 + (c ^ (r % 8))]);
      }
    };
    auto read_b = [&](int slot, int kk, bf16x8 (&dst)[NJ]) {
      const uint4* lb = &lds_all[slot * kSlot];
      const int c = kk * 4 + lg;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int r = PAIR ? (j / (NJ / 2)) * (BN / 2) + wn * (NJ / 2 * 16) + (j % (NJ / 2)) * 16 + ln
                           : wn * (NJ * 16) + j * 16 + ln;
        dst[j] = __builtin_bit_cast(bf16x8, lb[r * 8 + (c ^ (r % 8))]);
      }
    };
    issue_a(0, 0, 0, LA);
    issue_b(1, 0, 0, LB);
    if (nkt > 1) {
      issue_a(2, 1, 0, LA);
      issue_b(3, 1, 0, LB);
    }
    if (nkt > 2) {
      issue_a(4, 2, 0, LA);
      wait_vmcnt_lds<2 * LA + LB>();
    } else if (nkt > 1) {
      wait_vmcnt_lds<LA + LB>();
    } else {
      wait_vmcnt_lds<0>();
    }
    __builtin_amdgcn_s_barrier();
    read_a(0, 0, af[0]);
    read_b(1, 0, bf[0]);
    int sa = 0;            // slot of A(kt); B(kt) is in the next one (mod 5)
    int sap = 0, sbp = 0;  // the slots of the step before
    for (int kt = 0; kt < nkt; ++kt) {
      const int sb = sa + 1 < 5 ? sa + 1 : sa - 4;
      const int sa1 = sb + 1 < 5 ? sb + 1 : sb - 4;     // A(kt+1)
      const int sb1 = sa1 + 1 < 5 ? sa1 + 1 : sa1 - 4;  // B(kt+1)
#pragma unroll
      for (int u = 0; u < NU; ++u) {
        // The first row of MFMAs of the unit goes first: the compiler waits for every LDS read
        // issued so far (lgkmcnt(0)) in front of a unit's first MFMA whatever the reads are for,
        // so the reads for the next unit are issued behind it and have the rest of the unit.
        auto mfma_rows = [&](int i0, int i1) {
#pragma unroll
          for (int i = i0; i < i1; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
              acc[(u % UH) * AG + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                  af[u & 1][i], bf[(u / UH) & 1][j], acc[(u % UH) * AG + i][j], 0, 0, 0);
        };
        __builtin_amdgcn_sched_barrier(0);
        mfma_rows(0, 1);
        __builtin_amdgcn_sched_barrier(0);
        if (u + 1 < NU) {
          read_a(sa, u + 1, af[(u + 1) & 1]);
          if ((u + 1) % UH == 0) read_b(sb, (u + 1) / UH, bf[((u + 1) / UH) & 1]);
          // this unit's share of what the barrier of the step before made room for
          if (kt > 0) issue_some(kt - 1, sap, sbp, (u + 1) * NL / NU, (u + 2) * NL / NU);
        } else if (kt + 1 < nkt) {
          // this wavefront's loads up to B(kt+1) have landed (A(kt+2), the last LA loads it
          // issued, may be in flight) and its fragment reads of step kt are complete (not merely
          // issued: the loads that follow overwrite their slots)
          if (kt + 2 < nkt) wait_vmcnt_lds<LA>(); else wait_vmcnt_lds<0>();
          __builtin_amdgcn_s_barrier();
          issue_some(kt, sa, sb, 0, NL / NU);
          read_a(sa1, 0, af[0]);
          read_b(sb1, 0, bf[0]);
        }
        __builtin_amdgcn_sched_barrier(0);
        mfma_rows(1, AG);
        __builtin_amdgcn_sched_barrier(0);
      }
      sap = sa;
      sbp = sb;
      sa = sa1;
    }
  } else {
  DLLMC_LDS_ISSUE(0, rot)
  for (int kt = 0; kt < nkt; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < nkt;
    {
      if (more) {
        DLLMC_LDS_ISSUE(cur ^ 1, kt + 1 + rot < nkt ? kt + 1 + rot : kt + 1 + rot - nkt)
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
    // all fragment reads of this stage are complete before the loads issued at the top of the
    // next iteration overwrite it.  The explicit wait matters: without it the compiler puts the
    // wait for the last reads (and the MFMAs they feed) behind the barrier, and a load that hits
    // in L1 (the neighbouring workgroup on the CU reads the same activation rows) can land
    // before those reads execute.
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
  }
  }
#undef DLLMC_LDS_ISSUE

  if (EPI != 0) {
    // Epilogues that finish the step's work on the tile.  A wavefront's 16-row x 64-column block of
    // results (rounded to bf16) is staged through a private piece of LDS so that it leaves, and
    // the cached rows it is compared with arrive, as 16-byte pieces of contiguous row segments:
    // lane l then holds columns 8*(l%8) .. +8 of block rows l/8 and l/8 + 8.
    static_assert(EPI == 0 || NJ == 4, "a wavefront's block is 64 columns wide");
    static_assert(EPI != 2 || WN % 2 == 0, "a head is two column wavefronts");
    constexpr int kStg = 72;  // staging row stride in elements: 64 columns + 16 bytes
    static_assert(NWV * 16 * kStg * sizeof(bf16_t) <= kStage * sizeof(uint4), "staging fits a stage");
    __syncthreads();  // everybody has finished the fragment reads of the last step
    if (ONE_BARRIER) {
      static_assert(!ONE_BARRIER || NWV * 16 * kStg * sizeof(bf16_t) <= 4 * kSlot * sizeof(uint4),
                    "staging stays clear of the table");
      if (threadIdx.x < BM) {
        meta[0][threadIdx.x] = meta_r0;
        meta[1][threadIdx.x] = meta_r1;
      }
      __syncthreads();
    }
    uint32_t* stg32 = reinterpret_cast<uint32_t*>(&lds[0][0]) + wave * (16 * kStg / 2);
    const bf16_t* stg = reinterpret_cast<const bf16_t*>(stg32);
    const int rr = lane / 8, ch = lane % 8;
    const int odd = ln & 1;
    // EPI 2: the wavefront's columns are pairs (t, t + 64) of one head, t = tb .. tb + 31 (see the
    // weight loader), staged as two runs of 32
    const int tb = (wn % 2) * 32;
    const int head0 = n0 + (wn / 2) * 128;  // first column of the head in [W0; W1]
    const bool is_q = head0 < N0;
    const bool rot = is_q || ep->rope_second != 0;
    const int run = (ch / 4) * 64 + tb + (ch % 4) * 8;  // column inside the head of this lane's piece
    const int n_ct = N / 64, ct = col_tile * WN + wn;
    // rotation factors of block i for this lane's rows lg*4 + e and pairs tb + j*16 + ln, or the old
    // rows of block i (EPI 1): requested one block ahead
    float2 cs[2][4];
    uint4 old[2];
    auto request = [&](int i) {
      const int rb = wm * (MI * 16) + i * 16;  // first row of the block inside the tile
      if (EPI == 2) {
        if (rot) {
          const int4 pos = *reinterpret_cast<const int4*>(&meta[0][rb + lg * 4]);
          const int p4[4] = {pos.x, pos.y, pos.z, pos.w};
#pragma unroll
          for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int j = 0; j < 2; ++j)
              cs[j][e] = ep->tab[static_cast<size_t>(p4[e]) * 64 + tb + j * 16 + ln];
        }
      } else {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          old[h] = make_uint4(0u, 0u, 0u, 0u);
          const int r = rb + rr + 8 * h;
          if (meta[1][r] >= 0)
            old[h] = *reinterpret_cast<const uint4*>(ep->cache + static_cast<size_t>(meta[0][r]) * N + n0 +
                                                     wn * 64 + ch * 8);
        }
      }
    };
    if (!rot) {
#pragma unroll
      for (int e = 0; e < 4; ++e) cs[0][e] = cs[1][e] = make_float2(1.f, 0.f);
    }
    request(0);
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int rb = wm * (MI * 16) + i * 16;
      // final values of the lane's accumulator elements
      float val[NJ][4];
      uint4 old_i[2] = {old[0], old[1]};
      if (EPI == 2) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            const float x0 = acc[i][j][e], x1 = acc[i][j + 2][e];
            val[j][e] = x0 * cs[j][e].x - x1 * cs[j][e].y;
            val[j + 2][e] = x1 * cs[j][e].x + x0 * cs[j][e].y;
          }
      } else {
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
          for (int e = 0; e < 4; ++e) val[j][e] = acc[i][j][e];
      }
      if (i + 1 < MI) request(i + 1);
      // Neighbouring lanes hold neighbouring columns of the same four rows: they trade one value
      // of each row pair, after which the even lane owns columns (ln, ln + 1) of row e and the odd
      // lane columns (ln - 1, ln) of row e + 1, one 32-bit store each.
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int e = 0; e < 4; e += 2) {
          const float got = dpp_xor1(odd ? val[j][e] : val[j][e + 1]);
          const float lo = odd ? got : val[j][e];
          const float hi = odd ? val[j][e + 1] : got;
          const int r = lg * 4 + e + odd;
          stg32[(r * kStg + j * 16 + (ln & ~1)) / 2] = pack_bf16x2(lo, hi);
        }
      // the wavefront's own stores have completed before its loads are issued
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int r = rb + rr + 8 * h;  // row inside the tile
        const uint4 nv = *reinterpret_cast<const uint4*>(stg + (rr + 8 * h) * kStg + ch * 8);
        const int crow = meta[EPI == 1 ? 0 : 1][r];
        if (EPI == 1) {
          const int sidx = meta[1][r];
          if (ep->part != nullptr) {  // uniform
            const uint32_t nw4[4] = {nv.x, nv.y, nv.z, nv.w};
            const uint32_t ow4[4] = {old_i[h].x, old_i[h].y, old_i[h].z, old_i[h].w};
            float dot = 0.f, nn = 0.f, no = 0.f;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
              const float a0 = __uint_as_float(nw4[t] << 16), a1 = __uint_as_float(nw4[t] & 0xffff0000u);
              const float b0 = __uint_as_float(ow4[t] << 16), b1 = __uint_as_float(ow4[t] & 0xffff0000u);
              if (ep->metric == 0) {
                dot += a0 * b0; nn += a0 * a0; no += b0 * b0;
                dot += a1 * b1; nn += a1 * a1; no += b1 * b1;
              } else {
                const float d0 = a0 - b0, d1 = a1 - b1;
                dot += d0 * d0;
                dot += d1 * d1;
              }
            }
            // the eight lanes of a row: pairs, quads, then the two quads
            dot += dpp_xor1(dot); nn += dpp_xor1(nn); no += dpp_xor1(no);
            dot += dpp_xor2(dot); nn += dpp_xor2(nn); no += dpp_xor2(no);
            dot += dpp_half_mirror(dot); nn += dpp_half_mirror(nn); no += dpp_half_mirror(no);
            if (sidx >= 0 && ch == 0) {
              ep->part[(static_cast<size_t>(0) * n_ct + ct) * ep->part_stride + sidx] = dot;
              ep->part[(static_cast<size_t>(1) * n_ct + ct) * ep->part_stride + sidx] = nn;
              ep->part[(static_cast<size_t>(2) * n_ct + ct) * ep->part_stride + sidx] = no;
            }
          }
          if (m0 + r < M)
            *reinterpret_cast<uint4*>(ep->cache + static_cast<size_t>(crow) * N + n0 + wn * 64 + ch * 8) = nv;
        } else if (m0 + r < M) {
          bf16_t* dst = is_q ? ep->q_out + static_cast<size_t>(m0 + r) * N0 + head0 + run
                             : ep->cache + static_cast<size_t>(crow) * ep->d_kv + (head0 - N0) + run;
          *reinterpret_cast<uint4*>(dst) = nv;
        }
      }
      // ... and the loads before the next block's stores
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_s_waitcnt(0xC07F);
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
    return;
  }
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

// Tile kernels that finish the step's work in their epilogue (single slice): V-verify and Q | K
// with RoPE (see EPI above).
__global__ __launch_bounds__(512) void k_gemm_fat_vverify(const bf16_t* __restrict__ A, int lda, int M,
                                                          const bf16_t* __restrict__ W, int N, int K,
                                                          TileEpilogue ep) {
  gemm_lds_body<2, 4, 8, 4, 0, 1>(A, lda, nullptr, M, W, nullptr, N, N, K, K, nullptr, nullptr, &ep);
}
__global__ __launch_bounds__(256) void k_gemm_mid_vverify(const bf16_t* __restrict__ A, int lda, int M,
                                                          const bf16_t* __restrict__ W, int N, int K,
                                                          TileEpilogue ep) {
  gemm_lds_body<2, 2, 4, 4, 0, 1>(A, lda, nullptr, M, W, nullptr, N, N, K, K, nullptr, nullptr, &ep);
}
__global__ __launch_bounds__(512) void k_gemm_fat_qk(const bf16_t* __restrict__ A, int lda,
                                                     const int* __restrict__ rows, int M,
                                                     const bf16_t* __restrict__ W0,
                                                     const bf16_t* __restrict__ W1, int N0, int N, int K,
                                                     TileEpilogue ep) {
  gemm_lds_body<2, 4, 8, 4, 0, 2>(A, lda, rows, M, W0, W1, N0, N, K, K, nullptr, nullptr, &ep);
}
__global__ __launch_bounds__(256) void k_gemm_mid_qk(const bf16_t* __restrict__ A, int lda,
                                                     const int* __restrict__ rows, int M,
                                                     const bf16_t* __restrict__ W0,
                                                     const bf16_t* __restrict__ W1, int N0, int N, int K,
                                                     TileEpilogue ep) {
  gemm_lds_body<2, 2, 4, 4, 0, 2>(A, lda, rows, M, W0, W1, N0, N, K, K, nullptr, nullptr, &ep);
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

// 256 rows x (96 gate + 96 up) columns, 4 x 2 wavefronts of 64 x 96 each, one workgroup per CU: the
// column count that makes whole rounds of workgroups when the 256 x (128 + 128) tiles do not
// (1024 rows x FFN width 12288: 384 tiles of the latter are a full round and a half-empty one,
// 512 of these are two full rounds of tiles three quarters the size).
__global__ __launch_bounds__(512) void k_gemm_fat96_swiglu(const bf16_t* __restrict__ A, int lda,
                                                           const int* __restrict__ rows, int M,
                                                           const bf16_t* __restrict__ Wg,
                                                           const bf16_t* __restrict__ Wu, int N, int K,
                                                           bf16_t* __restrict__ U) {
  gemm_lds_body<4, 2, 4, 6, 1>(A, lda, rows, M, Wg, Wu, N, N, K, K, nullptr, U);
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
  // (phases of 128: the two register sets of gate and up pieces of a 256-wide phase do not fit
  // beside the activation chunks)
  const int KC = 128;
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
      // 96-column tiles when their rounds over the CUs finish sooner (a tile's time goes with its
      // columns; the narrower tile pulls a few per cent more operand bytes per flop)
      bool fat96 = false;
      if (fat && m % 96 == 0) {
        const int mt = (M + kFatM - 1) / kFatM, cus = 256;
        const double c128 = static_cast<double>((mt * (m / 128) + cus - 1) / cus) * 128.0;
        const double c96 = static_cast<double>((mt * (m / 96) + cus - 1) / cus) * 96.0 * 1.05;
        fat96 = c96 < c128;
      }
      if (tall)
        hipLaunchKernelGGL(k_gemm_tall_swiglu, dim3(m / 48, 1, 1), dim3(256), 0, st, a, lda, rows, M,
                           w0, w1, m, K, uo);
      else if (fat96)
        hipLaunchKernelGGL(k_gemm_fat96_swiglu, dim3(m / 96, (M + kFatM - 1) / kFatM, 1), dim3(512), 0, st, a,
                           lda, rows, M, w0, w1, m, K, uo);
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
    case 62: DLLMC_GD(6, 128, 2); break;
    case 82: DLLMC_GD(8, 128, 2); break;
    case 31: DLLMC_GD(3, 128, 1); break;
    case 81: DLLMC_GD(8, 128, 1); break;
    case 42: DLLMC_GD(4, 128, 2); break;
    default: DLLMC_GD(4, 128, 1); break;
  }
#undef DLLMC_GD
  return true;
}

// Which tile kernel finishes a launch of M rows x N columns in one slice: 2 = 256 x 256, 1 = 128 x
// 128, 0 = neither (the launch would leave more than a quarter of the CUs without a workgroup, or
// the shape does not fit the tiles).
static int direct_tile_kind(int M, int N, int N0, int K) {
  if (K % kFatK) return 0;
  const int cus = 256;
  if (M >= g_tune.fat_min_m && N % kFatN == 0 && N0 % kFatN == 0 &&
      ((M + kFatM - 1) / kFatM) * (N / kFatN) >= 3 * cus / 4)
    return 2;
  if (M >= g_tune.tile_min_m && N % kMidN == 0 && N0 % kMidN == 0 &&
      ((M + kMidM - 1) / kMidM) * (N / kMidN) >= 3 * cus / 4)
    return 1;
  return 0;
}

bool launch_gemm_vverify_tiles(int dtype, const void* A, int lda, int M, int first, int per_seq, int n,
                               int L_p, const void* W, int N, int K, void* v_cache, float* part,
                               int part_stride, int metric, const int* rmap, hipStream_t st) {
  if (M <= 0) return true;
  if (dtype != 1 || per_seq <= 0 || lda % 8 || !aligned16(A) || !aligned16(W)) return false;
  const int kind = direct_tile_kind(M, N, N, K);
  if (kind == 0) return false;
  TileEpilogue ep{};
  ep.first = first; ep.per_seq = per_seq; ep.n = n; ep.L_p = L_p;
  ep.cache = static_cast<bf16_t*>(v_cache);
  ep.part = part; ep.part_stride = part_stride; ep.metric = metric; ep.rmap = rmap;
  t_last_stream = false;
  const bf16_t* a = static_cast<const bf16_t*>(A);
  const bf16_t* w = static_cast<const bf16_t*>(W);
  if (kind == 2)
    hipLaunchKernelGGL(k_gemm_fat_vverify, dim3(N / kFatN, (M + kFatM - 1) / kFatM, 1), dim3(512), 0, st, a,
                       lda, M, w, N, K, ep);
  else
    hipLaunchKernelGGL(k_gemm_mid_vverify, dim3(N / kMidN, (M + kMidM - 1) / kMidM, 1), dim3(256), 0, st, a,
                       lda, M, w, N, K, ep);
  return true;
}

bool launch_gemm_qk_tiles(int dtype, const void* A, int lda, const int* rows, int M, const void* wq,
                          const void* w2, int d_q, int d_kv, int d_h, int K, const float2* rope_tab,
                          int n, void* q_out, void* cache, bool rope_second, const int* rmap,
                          hipStream_t st) {
  if (M <= 0) return true;
  if (dtype != 1 || d_h != 128 || lda % 8 || !aligned16(A) || !aligned16(wq) || !aligned16(w2)) return false;
  const int N = d_q + d_kv;
  const int kind = direct_tile_kind(M, N, d_q, K);
  if (kind == 0) return false;
  TileEpilogue ep{};
  ep.n = n; ep.cache = static_cast<bf16_t*>(cache); ep.rmap = rmap; ep.tab = rope_tab;
  ep.q_out = static_cast<bf16_t*>(q_out); ep.d_kv = d_kv; ep.rope_second = rope_second ? 1 : 0;
  t_last_stream = false;
  const bf16_t* a = static_cast<const bf16_t*>(A);
  const bf16_t* w0 = static_cast<const bf16_t*>(wq);
  const bf16_t* w1 = static_cast<const bf16_t*>(w2);
  if (kind == 2)
    hipLaunchKernelGGL(k_gemm_fat_qk, dim3(N / kFatN, (M + kFatM - 1) / kFatM, 1), dim3(512), 0, st, a, lda,
                       rows, M, w0, w1, d_q, N, K, ep);
  else
    hipLaunchKernelGGL(k_gemm_mid_qk, dim3(N / kMidN, (M + kMidM - 1) / kMidM, 1), dim3(256), 0, st, a, lda,
                       rows, M, w0, w1, d_q, N, K, ep);
  return true;
}

#undef g_tune

}  // namespace dllmc
