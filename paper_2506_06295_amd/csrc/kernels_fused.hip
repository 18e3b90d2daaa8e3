// Matrix products whose epilogue finishes the step's work in place, so that no float32 partial
// sums travel through HBM and no row kernel follows:
//
//  * k_vverify_tile -- V-verify of paper Sec. 3.2.2 in one launch (bf16): V_new = h W_v^T for
//                      every carried row, rounded to bf16; per row and 64-column tile the three
//                      sums of Eq. (cos_sim) (dot(V_new, V_cached), |V_new|^2, |V_cached|^2; or
//                      |V_new - V_cached|^2 for the L2 variant) against the cached row it is
//                      about to replace; the cached row overwritten.  The selection kernel adds
//                      the tile sums of a row in tile order and forms the score.
//                      64 x 64 output tile per workgroup over the whole contraction range (256
//                      workgroups for 256 response rows x 4096 columns: one per CU), four
//                      wavefronts of 32 x 32, both operands global -> LDS with
//                      global_load_lds_dwordx4 through a ring of four 64-wide stages (three
//                      steps in flight), v_mfma_f32_16x16x32_bf16.
#include "common.hpp"

namespace dllmc {

namespace {

constexpr int kVT = 64;       // tile edge: rows and columns
constexpr int kVK = 64;       // contraction values per stage
constexpr int kVStages = 4;
constexpr int kVnStride = 72; // bf16 elements per row of the epilogue tile (64 + 8 pad)

__device__ __forceinline__ void unpack8(const uint4& u, float (&f)[8]) {
  const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = __uint_as_float(w[i] << 16);
    f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}

// Carried row i of the step is position first + i % per_seq of sequence i / per_seq (per_seq = 0:
// row i itself).  A row is scored when part != nullptr and its position is a response position.
// part[(c * gridDim.x + column tile) * part_stride + seq * (n - L_p) + pos - L_p], c = 0 dot (or
// squared distance), 1 |new|^2, 2 |old|^2.
// KH = 2: eight wavefronts in two groups that walk the two halves of the contraction range side by
// side, each through its own ring (two wavefronts per SIMD cover each other's LDS and MFMA
// latencies, twice the loads in flight); the second group hands its sums over through LDS and
// the first adds them to its own (fixed order).
template <int KH>
__global__ __launch_bounds__(256 * KH) void k_vverify_tile(
    const bf16_t* __restrict__ A, int lda, int M, int first, int per_seq, int n, int L_p,
    const bf16_t* __restrict__ W, int N, int K, bf16_t* __restrict__ v_cache,
    float* __restrict__ part, int part_stride, int metric, const int* __restrict__ rmap) {
  // [group][stage][activation rows, then weight rows][8 slots of 16 bytes]; slot = chunk ^ (row % 8)
  __shared__ __attribute__((aligned(1024))) uint4 lds_all[KH][kVStages][(kVT + kVT) * 8];
  __shared__ __attribute__((aligned(16))) bf16_t Vn[kVT * kVnStride];
  const int kh = threadIdx.x / 256;                 // wavefront group
  const int wave = (threadIdx.x / 64) % 4, lane = threadIdx.x % 64;
  const int ln = lane % 16, lg = lane / 16;
  const int wm = wave / 2, wn = wave % 2;
  uint4 (*lds)[(kVT + kVT) * 8] = lds_all[kh];
  int col_tile, row_tile;
  xcd_tile_map(col_tile, row_tile);
  const int m0 = row_tile * kVT, n0 = col_tile * kVT;
  const int nkt = K / kVK / KH;                     // steps of one group
  const int kbase = kh * nkt * kVK;

  // epilogue role of this thread: row er of the tile, columns ECOLS eq .. ECOLS eq + ECOLS - 1
  constexpr int EPR = 4 * KH;        // threads per row
  constexpr int ECOLS = kVT / EPR;   // columns per thread: 16 or 8
  constexpr int EV = ECOLS / 8;      // 16-byte vectors per thread
  const int er = threadIdx.x / EPR, eq = threadIdx.x % EPR;
  const int em = m0 + er;
  const bool evalid = em < M;
  int erow = 0, epos = 0, eseq = 0;
  if (evalid) {
    if (per_seq > 0) {
      eseq = em / per_seq;
      epos = first + em % per_seq;
      erow = eseq * n + epos;
    } else {
      erow = em;
      eseq = em / n;
      epos = em % n;
    }
  }
  const bool scored = evalid && part != nullptr && epos >= L_p;
  // paged layout: the cache row that holds logical row erow
  const size_t crow = static_cast<size_t>((rmap != nullptr && evalid) ? rmap[erow] : erow);
  bf16_t* vrow = v_cache + crow * N + n0 + eq * ECOLS;
  // the cached values this thread scores against: requested first, they arrive under the loop
  uint4 vo[EV];
#pragma unroll
  for (int h = 0; h < EV; ++h) {
    vo[h] = make_uint4(0u, 0u, 0u, 0u);
    if (scored) vo[h] = *reinterpret_cast<const uint4*>(vrow + 8 * h);
  }

  // loader: instruction q of an operand covers tile rows [8q, 8q + 8); wavefront w issues q = 2w
  // and 2w + 1 of both operands.  Lane l: row 8q + l/8, LDS slot l%8, global chunk (l%8) ^ (row%8).
  const bf16_t* asrc[2];
  const bf16_t* bsrc[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int r = 8 * (2 * wave + j) + lane / 8;
    const int chunk = (lane % 8) ^ (r % 8);
    int m = m0 + r;
    if (m >= M) m = M - 1;  // rows past the end repeat the last one and are dropped at the store
    const int row = per_seq > 0 ? (m / per_seq) * n + first + m % per_seq : m;
    asrc[j] = A + static_cast<size_t>(row) * lda + kbase + chunk * 8;
    bsrc[j] = W + static_cast<size_t>(n0 + r) * K + kbase + chunk * 8;  // n0 + r < N: N % 64 == 0
  }
#define DLLMC_VV_ISSUE(stage, kt)                                                              \
  {                                                                                            \
    _Pragma("unroll") for (int j = 0; j < 2; ++j) {                                            \
      __builtin_amdgcn_global_load_lds(asrc[j] + (kt) * kVK, &lds[stage][(2 * wave + j) * 64], \
                                       16, 0, 0);                                              \
      __builtin_amdgcn_global_load_lds(bsrc[j] + (kt) * kVK,                                   \
                                       &lds[stage][kVT * 8 + (2 * wave + j) * 64], 16, 0, 0);  \
    }                                                                                          \
  }

  f32x4 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

#pragma unroll
  for (int s = 0; s < kVStages - 1; ++s)
    if (s < nkt) DLLMC_VV_ISSUE(s, s)

  for (int kt = 0; kt < nkt; ++kt) {
    // this wavefront's loads of step kt have landed: the younger steps in flight are
    // min(steps left, kVStages - 2), four loads each
    const int rem = nkt - 1 - kt;
    // (with every LDS read of this wavefront complete: see wait_vmcnt_lds)
    if (rem >= 2) wait_vmcnt_lds<8>();
    else if (rem == 1) wait_vmcnt_lds<4>();
    else wait_vmcnt_lds<0>();
    // everybody's loads of step kt have landed, and everybody has finished reading step kt - 1,
    // whose stage the loads of step kt + 3 overwrite
    __builtin_amdgcn_s_barrier();
    if (kt + kVStages - 1 < nkt) DLLMC_VV_ISSUE((kt + kVStages - 1) % kVStages, kt + kVStages - 1)
    const uint4* la = &lds[kt % kVStages][0];
    const uint4* lb = &lds[kt % kVStages][kVT * 8];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      const int c = kk * 4 + lg;
      bf16x8 af[2], bf[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int r = wm * 32 + i * 16 + ln;
        af[i] = __builtin_bit_cast(bf16x8, la[r * 8 + (c ^ (r % 8))]);
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int r = wn * 32 + j * 16 + ln;
        bf[j] = __builtin_bit_cast(bf16x8, lb[r * 8 + (c ^ (r % 8))]);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
  }
#undef DLLMC_VV_ISSUE

  if (KH > 1) {
    // hand-over of the second group's sums: [accumulator element][thread of the group]; its own
    // ring is free once the group has passed its last step
    float* red = reinterpret_cast<float*>(&lds_all[KH - 1][0][0]);
    const int t4 = threadIdx.x % 256;
    __syncthreads();
    if (kh > 0) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int e = 0; e < 4; ++e) red[((i * 2 + j) * 4 + e) * 256 + t4] = acc[i][j][e];
    }
    __syncthreads();
    if (kh == 0) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[i][j][e] += red[((i * 2 + j) * 4 + e) * 256 + t4];
    }
  }
  // the tile, rounded to bf16, through LDS: accumulator layout -> whole row segments per thread
  if (kh == 0) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          Vn[(wm * 32 + i * 16 + lg * 4 + e) * kVnStride + wn * 32 + j * 16 + ln] =
              f32_to_bf16(acc[i][j][e]);
  }
  __syncthreads();
  uint4 vn[EV];
#pragma unroll
  for (int h = 0; h < EV; ++h)
    vn[h] = *reinterpret_cast<const uint4*>(&Vn[er * kVnStride + eq * ECOLS + 8 * h]);
  if (part != nullptr) {  // uniform over the launch
    float dot = 0.f, nn = 0.f, no = 0.f;
    float a[8], o[8];
#pragma unroll
    for (int h = 0; h < EV; ++h) {
      unpack8(vn[h], a);
      unpack8(vo[h], o);
      if (metric == 0) {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          dot += a[t] * o[t];
          nn += a[t] * a[t];
          no += o[t] * o[t];
        }
      } else {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          const float df = a[t] - o[t];
          dot += df * df;
        }
      }
    }
    // the threads of a row are neighbouring lanes; fixed combination order
#pragma unroll
    for (int o2 = 1; o2 < EPR; o2 <<= 1) {
      dot += __shfl_xor(dot, o2, 64);
      nn += __shfl_xor(nn, o2, 64);
      no += __shfl_xor(no, o2, 64);
    }
    if (scored && eq == 0) {
      const size_t sidx = static_cast<size_t>(eseq) * (n - L_p) + (epos - L_p);
      const size_t nct = gridDim.x;
      part[(0 * nct + col_tile) * part_stride + sidx] = dot;
      part[(1 * nct + col_tile) * part_stride + sidx] = nn;
      part[(2 * nct + col_tile) * part_stride + sidx] = no;
    }
  }
  if (evalid) {
#pragma unroll
    for (int h = 0; h < EV; ++h) *reinterpret_cast<uint4*>(vrow + 8 * h) = vn[h];
  }
}

// score[i] from the tile sums, for callers without a selection (dllmc_op_vverify)
__global__ __launch_bounds__(256) void k_scores_from_part(const float* __restrict__ part, int n_ct,
                                                          int count, int metric,
                                                          float* __restrict__ score) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  float dot = 0.f, nn = 0.f, no = 0.f;
  for (int ct = 0; ct < n_ct; ++ct) {
    dot += part[(static_cast<size_t>(0) * n_ct + ct) * count + i];
    nn += part[(static_cast<size_t>(1) * n_ct + ct) * count + i];
    no += part[(static_cast<size_t>(2) * n_ct + ct) * count + i];
  }
  score[i] = metric == 0 ? dot / fmaxf(sqrtf(nn) * sqrtf(no), 1e-8f) : -sqrtf(dot);
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

bool vverify_fused_ok(int dtype, const void* A, int lda, int M, const void* W, int N, int K,
                      const void* v_cache) {
  if (dtype != 1 || M < 1 || N % kVT || K % kVK || lda % 8) return false;
  if (!aligned16(A) || !aligned16(W) || !aligned16(v_cache)) return false;
  // Up to two tiles per CU.  Beyond that (refresh steps with many rows) the 128 x 128 and 256 x 256
  // tiles of the split kernels pull half as many operand bytes into a CU per flop and win in
  // spite of their float32 round trip (768 rows x 4096 columns: 57 us here against ~45 there).
  const long long tiles = static_cast<long long>((M + kVT - 1) / kVT) * (N / kVT);
  return tiles <= 512;
}

size_t vverify_part_floats(int N, size_t scored_rows) {
  return static_cast<size_t>(3) * ((N + kVT - 1) / kVT) * scored_rows;
}

int vverify_col_tiles(int N) { return N / kVT; }

void launch_vverify_fused(const void* A, int lda, int M, int first, int per_seq, int n, int L_p,
                          const void* W, int N, int K, void* v_cache, float* part, int part_stride,
                          int metric, hipStream_t st, const int* rmap) {
  if (M <= 0) return;
  const dim3 grid(N / kVT, (M + kVT - 1) / kVT);
  // two wavefront groups when the halves of the contraction range are whole steps
  if ((K / kVK) % 2 == 0 && K / kVK >= 8)
    hipLaunchKernelGGL(k_vverify_tile<2>, grid, dim3(512), 0, st, static_cast<const bf16_t*>(A), lda,
                       M, first, per_seq, n, L_p, static_cast<const bf16_t*>(W), N, K,
                       static_cast<bf16_t*>(v_cache), part, part_stride, metric, rmap);
  else
    hipLaunchKernelGGL(k_vverify_tile<1>, grid, dim3(256), 0, st, static_cast<const bf16_t*>(A), lda,
                       M, first, per_seq, n, L_p, static_cast<const bf16_t*>(W), N, K,
                       static_cast<bf16_t*>(v_cache), part, part_stride, metric, rmap);
}

void launch_scores_from_part(const float* part, int n_ct, int count, int metric, float* score,
                             hipStream_t st) {
  if (count <= 0) return;
  hipLaunchKernelGGL(k_scores_from_part, dim3((count + 255) / 256), dim3(256), 0, st, part, n_ct,
                     count, metric, score);
}

}  // namespace dllmc
