// Shared device helpers and the host-side launch interface of the dllmc kernels (gfx950).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dllmc {

constexpr int kWave = 64;  // CDNA wavefront width

// ---- storage types -------------------------------------------------------------------
// bf16 values are handled as raw 16-bit patterns; conversion is round-to-nearest-even.
typedef uint16_t bf16_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t h) {
  return __uint_as_float(static_cast<uint32_t>(h) << 16);
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<bf16_t>((u >> 16) | 0x40u);  // NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<bf16_t>(u >> 16);
}

// two floats -> two bf16 (round to nearest even; the hardware's packed conversion), `lo` in the
// low half
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}
// value of lane (l ^ 1) / (l ^ 2) of the same quad, and of lane 7 - (l % 8) of the same group of
// eight (data-parallel-primitive moves: no LDS traffic)
__device__ __forceinline__ float dpp_xor1(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, false));
}
__device__ __forceinline__ float dpp_xor2(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, false));
}
__device__ __forceinline__ float dpp_half_mirror(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, false));
}

template <typename T> __device__ __forceinline__ float ldf(const T* p);
template <> __device__ __forceinline__ float ldf<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ldf<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }

template <typename T> __device__ __forceinline__ void stf(T* p, float v);
template <> __device__ __forceinline__ void stf<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void stf<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// value after a round trip through the storage type
template <typename T> __device__ __forceinline__ float roundf_to(float v);
template <> __device__ __forceinline__ float roundf_to<float>(float v) { return v; }
template <> __device__ __forceinline__ float roundf_to<bf16_t>(float v) { return bf16_to_f32(f32_to_bf16(v)); }

// ---- wavefront / workgroup reductions ------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
// Sum over a workgroup of NW wavefronts; `red` is NW floats of LDS.  Every thread gets the
// total, summed in wave order (deterministic).
template <int NW>
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x / kWave;
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) red[w] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < NW; ++i) t += red[i];
  return t;
}

// a pointer that is the same in every lane, re-read from lane 0 (lands in scalar registers)
__device__ __forceinline__ const char* wave_uniform_ptr(const char* p) {
  const uint64_t b = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b >> 32));
  return reinterpret_cast<const char*>((static_cast<uint64_t>(hi) << 32) | lo);
}

// ---- MFMA operand types, tile-to-XCD mapping, explicit waits ----------------------------
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

// Workgroups are handed to the 8 XCDs round-robin in launch order (x fastest), and each XCD has
// its own L2.  With several row tiles per column tile, remap (blockIdx.x, blockIdx.y) so that
// all row tiles of one column tile run back to back on the same XCD: the weight tile is then
// fetched from HBM once and the other row tiles hit in that XCD's L2.  The column tiles beyond
// the last multiple of 8 are walked column by column after the remapped part.
__device__ __forceinline__ void xcd_tile_map(int& col_tile, int& row_tile) {
  const int nt = gridDim.x, mt = gridDim.y;
  col_tile = blockIdx.x;
  row_tile = blockIdx.y;
  if (mt > 1 && nt >= 8) {
    const int nt8 = nt & ~7;
    const int lin = blockIdx.x + nt * blockIdx.y;
    if (lin < nt8 * mt) {
      const int xcd = lin & 7, slot = lin >> 3;
      row_tile = slot % mt;
      col_tile = (slot / mt) * 8 + xcd;
    } else {
      const int rest = lin - nt8 * mt;
      row_tile = rest % mt;
      col_tile = nt8 + rest / mt;
    }
  }
}
// Tile order of the LDS-direct tile kernels.  What matters for them is how many DIFFERENT operand
// blocks the workgroups that run at the same time on one XCD pull into its L2: 32 workgroups (one
// per CU) that share one weight tile and differ in their activation rows -- what dealing column
// tiles to the XCDs round-robin gives a tall problem -- fetch 33 blocks per step between them, all
// but one of them used once, and a 12288-row projection then reads its activations from memory
// once per column tile (1.7 GB for 130 MB of operands) and runs at the speed of that traffic.  Here
// the tiles are put in an order of bands of kBand row tiles, walked column by column with the rows
// of the band innermost, and every XCD takes a contiguous piece of that order: its concurrent
// workgroups then form a patch of about kBand x (32 / kBand) tiles, 12 blocks per step for 32
// tiles.  The map is a bijection of the grid for any mt, nt.
constexpr int kBand = 8;
__device__ __forceinline__ void xcd_tile_map_blocked(int& col_tile, int& row_tile) {
  const int nt = gridDim.x, mt = gridDim.y;
  const int T = nt * mt;
  const int lin = blockIdx.x + nt * blockIdx.y;
  if (T < 16) {  // nothing to arrange
    col_tile = blockIdx.x;
    row_tile = blockIdx.y;
    return;
  }
  // XCD x runs the workgroups lin = x, x + 8, ...: (T - x + 7) / 8 of them; its piece of the order
  // starts where the pieces of the XCDs before it end
  const int xcd = lin & 7, slot = lin >> 3;
  const int g = xcd * (T >> 3) + min(xcd, T & 7) + slot;
  const int band = g / (kBand * nt);
  const int rows_in_band = min(kBand, mt - band * kBand);
  const int within = g - band * kBand * nt;
  row_tile = band * kBand + within % rows_in_band;
  col_tile = within / rows_in_band;
}
// s_waitcnt with only vmcnt set: vmcnt[3:0] -> bits 3:0, vmcnt[5:4] -> bits 15:14
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
// ... and lgkmcnt(0): at most N vector-memory operations outstanding AND every LDS operation of
// this wavefront complete.  Needed in front of a barrier that hands an LDS stage back to
// global_load_lds: a fragment read that has been issued but not executed when the wavefront
// passes the barrier can be overtaken by the data of the next load into that stage (which does
// not queue behind LDS instructions), and the compiler is free to place the wait for such a read
// behind the barrier.
template <int N> __device__ __forceinline__ void wait_vmcnt_lds() {
  __builtin_amdgcn_s_waitcnt(0x0070 | (N & 15) | ((N >> 4) << 14));
}

// ---- host-side launchers (defined in the kernels_*.hip files) --------------------------
// dtype: 0 = float32 storage, 1 = bf16 storage.  All pointers are device pointers.

// C_part[s][i][:] (float32, s < S) = partial products of A[rows[i], :] * [W0; W1]^T over the
// s-th slice of the contraction index.  W0 holds output columns [0, N0), W1 columns [N0, N)
// (W1 may be null when N0 == N).  rows == nullptr means the identity.  Returns the number
// of slices S it used (>= 1) so that consumers sum c_part[0..S) in order.  c_part holds
// c_capacity floats; S is chosen so that S * M * N fits, and 0 is returned (nothing launched)
// if not even M * N floats fit.
// most float32 slices of the contraction index a GEMM launch may produce; the row kernels
// dispatch their slice count to a compile-time constant in 1 .. kMaxSlices
constexpr int kMaxSlices = 8;
int gemm_max_slices();
// Kernel choice and slice planning knobs of the matrix products.  Every context owns a copy (taken
// from the process default when it is created); the launchers use the copy of the context whose
// call is running on this thread (TuningScope), the process default otherwise.
struct GemmTuning {
  int nw = 8;          // wavefronts per workgroup (4 or 8) of the single-matrix kernel
  int nw_dual = 106;   // fused gate/up kernel: 6 wavefronts in two groups over the contraction
                       // range (+100), i.e. 48 columns of each matrix per workgroup: the
                       // narrowest tile that still amortises the activation tile measured
                       // fastest at both FFN widths (12288: one workgroup per CU)
  int force_s = 0;     // > 0: number of slices of the contraction index
  int target_wg = 256; // workgroups the automatic slice count aims for
  int fat_min_m = 512;      // activation rows from which the 256 x 256 LDS-direct kernel is used
  int tall_max_m = 128;     // most rows the streaming kernel covers with one workgroup tile:
                            // 65..128 rows run with 128 rows per workgroup when it is >= 128
                            // (weights streamed once instead of once per 64-row tile); from
                            // 256 on, launches of tile_min_m..tall_max_m rows use 256 rows per
                            // workgroup instead of the 128 x 128 tiles (slower where measured)
  int tile_min_m = 192;     // activation rows from which the 128 x 128 LDS-direct kernel is used
                            // (off by default: the streaming kernel is faster at the sizes measured)
};
GemmTuning gemm_default_tuning();
struct TuningScope {
  const GemmTuning* prev;
  explicit TuningScope(const GemmTuning* t);
  ~TuningScope();
  TuningScope(const TuningScope&) = delete;
  TuningScope& operator=(const TuningScope&) = delete;
};
// slices launch_gemm would use for 16-byte aligned operands (0: capacity too small); host only
int gemm_plan_slices(int dtype, int M, int N, int N0, int K, size_t c_capacity);
void gemm_set_tuning(int nw, int nw_dual, int force_s, int target_wg);
void gemm_set_tile_min_m(int m);
void gemm_set_fat_min_m(int m);
void gemm_set_tall_max_m(int m);
// True when the most recent launch_gemm / launch_gemm_swiglu of this thread ran k_gemm_stream.
bool gemm_last_was_stream();
void gemm_clear_last_stream();  // a matrix product launched by another launcher follows
int launch_gemm(int dtype, const void* A, int lda, const int* rows, int M, const void* W0,
                const void* W1, int N0, int N, int K, float* c_part, size_t c_capacity,
                hipStream_t st);

// Fused gate/up projection with the SwiGLU product: u[i][j] = T(silu(a_i . w_gate_j) *
// (a_i . w_up_j)), no slices, nothing but u written.  Returns false (and launches nothing)
// when the shape or type is not handled; the caller then uses launch_gemm + launch_swiglu.
bool launch_gemm_swiglu(int dtype, const void* A, int lda, const int* rows, int M,
                        const void* w_gate, const void* w_up, int m, int K, void* u,
                        hipStream_t st);

// out[i][:] = sum_s c_part[s][i][:]
void launch_reduce_slices(const float* c_part, int S, int M, int N, float* out, hipStream_t st);

// Paged cache layout: wherever a launcher takes `rmap` (device int32, one entry per logical row
// b * n + position, or nullptr for the flat layout), logical row r of a cache tensor lives in row
// rmap[r] of that tensor's storage.
// out[r][:] = cache[rmap[r]][:] for r < rows
void launch_gather_rows(int dtype, const void* cache, const int* rmap, int rows, int width,
                        void* out, hipStream_t st);

struct RowKernelArgs {
  int dtype;
  int n;            // rows per sequence (L_p + L_r)
  int L_p;
  int d;            // model width
  float eps;
};

// x[row] = hidden_in[row]; h[row] = T(rmsnorm(x[row]) * g) for row in rows[0..M)
void launch_embed_norm(const RowKernelArgs& a, const void* hidden_in, const int* rows, int M,
                       const void* gain, float* x, void* h, hipStream_t st);

// V finalize: for i < M: row = (i / per_seq) * n + first + i % per_seq, the carried rows of a
// step (row = i when per_seq == 0); v = T(sum_s c_part[s][i][:]);
// if score != nullptr and row is a response row: score[seq][j] = cos(v, v_cache[row]) (metric
// 0) or -|v - v_cache[row]| (metric 1); then v_cache[row] = v, except that response rows go
// to v_stage[i] instead when v_stage != nullptr (selected-only update, see launch_scatter_v).
void launch_v_finalize(const RowKernelArgs& a, const float* c_part, int S, int first, int per_seq,
                       int M, int d_kv, void* v_cache, float* score, int metric, void* v_stage,
                       hipStream_t st, const int* rmap = nullptr);
// v_cache[row] = v_stage[(row / n) * carried_per_seq + row % n - first] for the response rows
// among rows_R[0..M_R)
void launch_scatter_v(const RowKernelArgs& a, const int* rows_R, int M_R, int first,
                      int carried_per_seq, int d_kv, const void* v_stage, void* v_cache,
                      hipStream_t st, const int* rmap = nullptr);
// score[b][j] = 24-bit uniform in [0, 1) keyed by (seed, step, layer, b, j)
void launch_random_scores(uint32_t seed, int step, int layer, int B, int L, float* out,
                          hipStream_t st);

// Q/K finalize: for i < M: row = rows[i], pos = row % n; c = sum_s c_part[s][i][0..d_q+d_kv);
// q_out[i] = T(rope(c[0..d_q))), k_cache[row] = T(rope(c[d_q..))).  rope_tab[pos][t] =
// (cos, sin) of pos * theta^(-2t/d_h).
// rope_second = false: the second matrix' columns are stored unrotated (K-verify: they are the
// Values of the selected rows and k_cache is the V cache).
void launch_qk_finalize(const RowKernelArgs& a, const float* c_part, int S, const int* rows, int M,
                        int d_q, int d_kv, int d_h, const float2* rope_tab, void* q_out,
                        void* k_cache, bool rope_second, hipStream_t st, const int* rmap = nullptr);
// K finalize (K-verify): like launch_v_finalize on the Key projection, with RoPE at the row's
// position before rounding, scoring and the cache write.
void launch_k_finalize(const RowKernelArgs& a, const float* c_part, int S, const int* rows, int M,
                       int d_kv, int d_h, const float2* rope_tab, void* k_cache, float* score,
                       int metric, void* k_stage, hipStream_t st, const int* rmap = nullptr);

// Output-projection finalize over the recomputed rows: for ci < M_R: row = rows_R[ci];
// attn_cache[row] = T(sum_s c_part[s][ci][:]) (c_part slices hold M_R rows);
// x[row] += attn_cache[row]; g_out[ci] = T(rmsnorm(x[row]) * gain).  The carried rows that are
// not recomputed get their x[row] += attn_cache[row] in launch_down_finalize.
void launch_o_finalize(const RowKernelArgs& a, const float* c_part, int S, const int* rows_R,
                       int M_R, void* attn_cache, float* x, const void* gain, void* g_out,
                       hipStream_t st, const int* rmap = nullptr);

// SwiGLU: u[i][j] = T(silu(c[i][j]) * c[i][m + j]) with c = sum_s c_part[s] of width 2m.
void launch_swiglu(int dtype, const float* c_part, int S, int M, int m, void* u, hipStream_t st);

// Down-projection finalize over the Mc carried rows (row = (i / per_seq) * n + first + i % per_seq,
// ci = inv[row]): if ci >= 0
// the ffn_cache update as in launch_o_finalize, else first x[row] += attn_cache[row];
// x[row] += ffn_cache[row]; then either h[row] = T(rmsnorm(x[row]) * next_gain) (next_gain
// != nullptr) or, for the last layer, hidden_out[row] = T(x[row]) and, for prompt rows when
// prompt_out != nullptr, prompt_out[seq][row % n] = T(x[row]).
void launch_down_finalize(const RowKernelArgs& a, const float* c_part, int S, int M_R,
                          int first, int per_seq, int Mc, const int* inv, const void* attn_cache,
                          void* ffn_cache, float* x, const void* next_gain, void* h,
                          void* hidden_out, void* prompt_out, hipStream_t st,
                          const int* rmap = nullptr);

// hidden_out[b][t] = prompt_out[b][t] for all prompt rows
void launch_copy_prompt(const RowKernelArgs& a, int B, const void* prompt_out, void* hidden_out,
                        hipStream_t st);

// Bottom-k selection per sequence.  scores: [B, L] float32.  Writes, for sequence b and the
// pos-th selected index j (ascending):
//   sel_out[b*sel_stride + pos] = j                          (if sel_out != nullptr)
//   rows_out[b*per_seq + off + pos] = b*n + L_p + j          (if rows_out != nullptr)
//   inv_out[b*n + L_p + j] = b*per_seq + off + pos, and -1 for rows not selected
// part != nullptr: the scores are formed first (and written to `scores`) from the sums the
// fused V-verify launch left per row and column tile (n_ct tiles, see launch_vverify_fused).
void launch_select(float* scores, int B, int L, int k, int* sel_out, int sel_stride,
                   int* rows_out, int per_seq, int off, int* inv_out, int n, int L_p,
                   hipStream_t st, const float* part = nullptr, int n_ct = 0, int part_stride = 0,
                   int metric = 0);

// Fused V-verify (bf16): v = bf16(A[row(i)] W^T) for the M carried rows (row(i) = (i / per_seq) * n
// + first + i % per_seq, or i when per_seq == 0); when part != nullptr, for every response row
// (position >= L_p) and 64-column tile t the sums (v . old, |v|^2, |old|^2) (metric 1: (|v -
// old|^2, 0, 0)) over the tile's columns go to part[(c * n_ct + t) * part_stride + seq * (n -
// L_p) + pos - L_p]; then v_cache[row] = v.  vverify_fused_ok says whether the shape is handled.
bool vverify_fused_ok(int dtype, const void* A, int lda, int M, const void* W, int N, int K,
                      const void* v_cache);
size_t vverify_part_floats(int N, size_t scored_rows);
int vverify_col_tiles(int N);
void launch_vverify_fused(const void* A, int lda, int M, int first, int per_seq, int n, int L_p,
                          const void* W, int N, int K, void* v_cache, float* part, int part_stride,
                          int metric, hipStream_t st, const int* rmap = nullptr);
// The same V-verify, and the Q | K projection with RoPE and the cache scatter, finished in the
// epilogue of the 128 x 128 / 256 x 256 tile kernels (one slice, no float32 partial sums, no row
// kernel) for launches with enough rows to fill the chip that way.  Arguments as for
// launch_vverify_fused / launch_gemm + launch_qk_finalize.  Return false (nothing launched) when
// the shape is not handled.
bool launch_gemm_vverify_tiles(int dtype, const void* A, int lda, int M, int first, int per_seq, int n,
                               int L_p, const void* W, int N, int K, void* v_cache, float* part,
                               int part_stride, int metric, const int* rmap, hipStream_t st);
bool launch_gemm_qk_tiles(int dtype, const void* A, int lda, const int* rows, int M, const void* wq,
                          const void* w2, int d_q, int d_kv, int d_h, int K, const float2* rope_tab,
                          int n, void* q_out, void* cache, bool rope_second, const int* rmap,
                          hipStream_t st);
// score[i] = cosine (metric 0) or minus distance (metric 1) from the tile sums, i < count
void launch_scores_from_part(const float* part, int n_ct, int count, int metric, float* score,
                             hipStream_t st);

// Attention of Mq compact queries per sequence over all n keys of that sequence.
// q, out: [B, Mq, H_q*d_h]; k_cache, v_cache: [B, n, H_kv*d_h].
// The float32 / odd-head-width kernel keeps one row of n scores in LDS.
bool attention_supported(int dtype, int d_h, int n);
// scratch (may be null): attention_scratch_floats() floats for the split-key partial results.
size_t attention_scratch_floats();
// rmap (paged layout): key row j of sequence b is row rmap[b * n + j] of k_cache / v_cache.
void launch_attention(int dtype, const void* q, int B, int Mq, const void* k_cache,
                      const void* v_cache, int n, int H_q, int H_kv, int d_h, void* out,
                      float* scratch, hipStream_t st, const int* rmap = nullptr);

// Row lists: for b < B, t < count: ci = b*per_seq + off + t, row = b*n + first + t;
// rows[ci] = row (if rows), inv[row] = ci (if inv).
void launch_iota_rows(int* rows, int* inv, int B, int n, int first, int count, int per_seq,
                      int off, hipStream_t st);
void launch_fill_i32(int* p, int value, size_t count, hipStream_t st);
// ---- closed denoising loop (kernels_gen.hip) --------------------------------------------
// out[r][:] = table[tokens[r]][:] for r < rows; table has vocab_rows rows of width d
void launch_embed_gather(int dtype, const void* table, int vocab_rows, const int* tokens, int rows,
                         int d, void* out, hipStream_t st);
// elig[b][j] = 0 if response position j of sequence b holds mask_id and lo <= j < hi, else 1;
// neg_conf[b][j] = +inf, x0[b][j] = -1.  tokens: [B, n].
void launch_elig_scores(const int* tokens, int B, int n, int L_p, int lo, int hi, int mask_id,
                        float* elig, float* neg_conf, int* x0, hipStream_t st);
// z[i][:] = T(rmsnorm(hidden[rows[i]]) * gain) for i < M (rows == nullptr: identity)
void launch_final_norm(int dtype, const void* hidden, const int* rows, int M, int d, float eps,
                       const void* gain, void* z, hipStream_t st);
// for i < M: token = first argmax of logits[i][0..vocab), p = softmax(logits[i])[token]; with
// rows (rows[i] = b*n + L_p + j): x0[b][j] = token, conf[b][j] = sign * p; rows == nullptr:
// x0[i], conf[i]
void launch_head_finalize(const float* logits, int M, int vocab, const int* rows, int n, int L_p,
                          float sign, int* x0, float* conf, hipStream_t st);
void launch_negate_f32(float* p, size_t count, hipStream_t st);
// tokens[b][L_p + chosen[b*chosen_stride + t]] = x0[b][...] for t < n_unmask
void launch_apply_tokens(int* tokens, int B, int n, int L_p, const int* chosen, int chosen_stride,
                         int n_unmask, const int* x0, hipStream_t st);

// achievable-peak probes (not steps of the method): plain copy, plain read, MFMA loop; the last
// returns the flops its launch performs
void launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t st);
void launch_probe_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t st);
double launch_probe_mfma(int iters, int shape, float* sink, hipStream_t st);

// sel[r][j] = j for r < rows, j < L_r
void launch_fill_sel_identity(int* sel, int rows, int L_r, hipStream_t st);

}  // namespace dllmc
