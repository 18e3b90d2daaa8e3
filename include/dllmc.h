/*
 * dllmc -- cached bidirectional-transformer denoising step (dLLM-Cache) for MI355X.
 *
 * C ABI of libdllmc.so.  All pointers named "device" are HIP device memory owned by the
 * caller; the library never allocates or frees device memory.  All calls return 0 on
 * success or a negative DLLMC_E* code; nothing aborts or throws across this boundary.
 * Work is enqueued on the HIP stream given at creation and the calls do not wait for it:
 * outputs are valid once the caller has synchronised that stream.
 *
 * The method (paper Sec. 3.2): per transformer layer the library keeps K (after RoPE), V,
 * AttnOut (after the output projection) and FFNOut (after the down projection) for every
 * token, split into a prompt cache (rows [0, L_p)) and a response cache (rows [L_p, n)).
 * Step i (counted up from 0) refreshes the prompt features iff i % K_p == 0, refreshes the
 * whole response iff i % K_r == 0, and otherwise performs the adaptive partial update of
 * Sec. 3.2.2: project V for all response rows, score each row by the cosine similarity to
 * its cached V (Eq. cos_sim), overwrite the cached V, and recompute Q/K, attention over all
 * n cached keys, the output projection and the SwiGLU FFN only for the floor(rho*L_r) rows
 * with the lowest score (ties: lower index), scattering K, AttnOut and FFNOut back.
 */
#ifndef DLLMC_H
#define DLLMC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dllmc_ctx dllmc_ctx; /* opaque host object */

enum { DLLMC_F32 = 0, DLLMC_BF16 = 1 };

enum {
  DLLMC_OK = 0,
  DLLMC_EINVAL = -1, /* bad dimension, rho outside [0,1], K_p/K_r < 1, null or misaligned pointer */
  DLLMC_ESTATE = -2, /* first step is not step 0, or a non-zero step_idx that does not increase */
  DLLMC_EHIP = -3,   /* a HIP runtime call failed (see dllmc_last_hip_error) */
  DLLMC_ENOMEM = -4, /* workspace smaller than dllmc_workspace_bytes() */
  DLLMC_ETOOBIG = -5 /* dllmc_op_linear_static: M * N beyond the static scratch buffer */
};

/* Architecture of the bidirectional transformer (pre-RMSNorm, rotate-half RoPE with pairs
 * (t, t + head_dim/2), softmax scale 1/sqrt(head_dim), SwiGLU FFN, no biases).  The paper
 * names only "bidirectional attention" and the three SwiGLU matmuls (complexity appendix);
 * the rest comes from the LLaDA-8B / Dream-7B shaped workloads. */
typedef struct {
  int32_t n_layers;   /* T */
  int32_t d_model;    /* d */
  int32_t n_q_heads;  /* H_q */
  int32_t n_kv_heads; /* H_kv, divides H_q */
  int32_t head_dim;   /* d_h, even; n_q_heads*head_dim is the attention width d_q */
  int32_t d_ffn;      /* m */
  int32_t batch;      /* B independent sequences, each with its own caches and selection */
  int32_t dtype;      /* DLLMC_F32 or DLLMC_BF16: type of weights, hidden states and caches */
  float rms_eps;
  float rope_theta;
} dllmc_model;

/* One layer's weights: device pointers, borrowed for the life of the context, read-only,
 * row-major [out, in] (the contraction index is contiguous), element type = model dtype,
 * 16-byte aligned. */
typedef struct {
  const void* attn_norm_g; /* [d]        */
  const void* wq;          /* [d_q, d]   */
  const void* wk;          /* [d_kv, d]  */
  const void* wv;          /* [d_kv, d]  */
  const void* wo;          /* [d, d_q]   */
  const void* ffn_norm_g;  /* [d]        */
  const void* w_gate;      /* [m, d]     */
  const void* w_up;        /* [m, d]     */
  const void* w_down;      /* [d, m]     */
} dllmc_layer_weights;

/* Bytes of device workspace a context needs (caches of Sec. 3.2 plus scratch); 0 if the
 * arguments are invalid.  Caches take 2*(d_kv + d)*n*B*T elements, the paper's 4*T*d per
 * token and layer (storage-overhead proof) with d_kv in place of d for grouped KV heads. */
size_t dllmc_workspace_bytes(const dllmc_model* model, int32_t L_p, int32_t L_r);

/* Create a context.  `layers` is a host array of n_layers entries (copied).  `workspace`
 * is device memory of at least dllmc_workspace_bytes(), 256-byte aligned, owned by the
 * caller and used exclusively by this context until dllmc_destroy.  `hip_stream` is a
 * hipStream_t (NULL = the default stream).  rho in [0,1]; K_p, K_r >= 1 (Sec. 3.2). */
int dllmc_create(dllmc_ctx** out, const dllmc_model* model, const dllmc_layer_weights* layers,
                 int32_t L_p, int32_t L_r, float rho, int32_t K_p, int32_t K_r,
                 void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---- paged cache layout ------------------------------------------------------------------
 * The paper's Limitations paragraph names the growth of the feature caches with the sequence
 * length as its open problem and points at memory management as the remedy.  Here the four
 * per-layer cache tensors of Sec. 3.2 may live in a POOL of equally sized pages instead of one
 * flat [B, n, width] block per layer: a page holds page_rows consecutive token positions of one
 * sequence, in every layer and in all four tensors (one page id addresses the same slot
 * everywhere), and a page table maps (sequence b, logical page p) to a pool page:
 *     row (b, pos) of a layer's cache tensor  ->  row page_table[b][pos / page_rows] * page_rows
 *                                                     + pos % page_rows of that tensor's pool block.
 * Results are bit-identical to the flat layout.  The pool may be carved from the context's own
 * workspace (pool == NULL) or be caller-owned device memory of dllmc_pool_bytes() bytes shared
 * by several contexts of the same model, page_rows and pool_pages, each using its own, disjoint
 * pages: when a generation is over its pages can serve another context (eviction is the
 * caller's policy; dllmc_pool_* below is a host-side allocator for the ids).
 * Pool block layout: regions K, V, AttnOut, FFNOut in this order; a region holds n_layers
 * blocks of pool_pages * page_rows rows of the tensor's width, each block 256-byte aligned. */
typedef struct {
  int32_t page_rows;          /* token positions per page, >= 1 */
  int32_t pool_pages;         /* pages in the pool */
  const int32_t* page_table;  /* HOST [B][ceil((L_p + L_r) / page_rows)], copied; entries in
                                 [0, pool_pages), no page listed twice */
  void* pool;                 /* device, 256-byte aligned, or NULL: inside the workspace */
  size_t pool_bytes;          /* size of `pool` (ignored when pool == NULL) */
} dllmc_paging;

/* Bytes of a pool block for this model (0: invalid arguments). */
size_t dllmc_pool_bytes(const dllmc_model* model, int32_t page_rows, int32_t pool_pages);
/* dllmc_workspace_bytes / dllmc_create for the paged layout.  With paging->pool == NULL the
 * workspace also holds the pool.  DLLMC_EINVAL on a malformed page table. */
size_t dllmc_workspace_bytes_paged(const dllmc_model* model, int32_t L_p, int32_t L_r,
                                   const dllmc_paging* paging);
int dllmc_create_paged(dllmc_ctx** out, const dllmc_model* model, const dllmc_layer_weights* layers,
                       int32_t L_p, int32_t L_r, float rho, int32_t K_p, int32_t K_r,
                       const dllmc_paging* paging, void* workspace, size_t workspace_bytes,
                       void* hip_stream);
/* Replace the page table of a paged context (HOST array as above, copied; waits for the
 * context's stream).  Page contents are not moved: the caches are void afterwards and the next
 * dllmc_step must be step 0 (DLLMC_ESTATE otherwise).  DLLMC_EINVAL for a flat context or a
 * malformed table (nothing changes then). */
int dllmc_set_page_table(dllmc_ctx* ctx, const int32_t* page_table);

/* Host-side allocator of page ids (no device memory involved; thread-safe).  alloc hands out
 * `count` ids, lowest free ids first, all or nothing (DLLMC_ENOMEM); free takes ids back and
 * rejects, without freeing anything, a list with an id that is out of range, not allocated or
 * listed twice (DLLMC_EINVAL). */
typedef struct dllmc_page_pool dllmc_page_pool;
int dllmc_pool_create(dllmc_page_pool** out, int32_t pool_pages);
int32_t dllmc_pool_available(dllmc_page_pool* pool);
int dllmc_pool_alloc(dllmc_page_pool* pool, int32_t count, int32_t* ids_out);
int dllmc_pool_free(dllmc_page_pool* pool, const int32_t* ids, int32_t count);
int dllmc_pool_destroy(dllmc_page_pool* pool);

/* floor(rho * L_r): rows recomputed per sequence and layer on an adaptive step (Sec. 3.2.2). */
int32_t dllmc_num_selected(const dllmc_ctx* ctx);

/* Variants the paper compares with its default (cosine V-verify with whole-V overwrite);
 * take effect at the next dllmc_step, normally set before step 0.
 *   source     0: V-verify; 1: K-verify (Sec. 4.3), taken as its mirror image: on an adaptive step
 *              the Key rows (after RoPE) of all response rows are computed, scored against the
 *              cached Keys and written back, the Values are recomputed and scattered for the
 *              selected rows only; dllmc_read_scores then returns the Key scores
 *   metric     0: cosine of Eq. (cos_sim); 1: minus the Euclidean distance between the current
 *              and the cached Value row (appendix "Impact of Similarity Metric")
 *   selection  0: the floor(rho*L_r) lowest scores; 1: random rows (Sec. 4.3): the scores are
 *              24-bit uniforms h >> 8 scaled by 2^-24, h = seed, then for each of step_idx,
 *              layer, sequence, position: h = fmix32(h xor value), fmix32 being the 32-bit
 *              finalizer of MurmurHash3; dllmc_read_scores returns them
 *   v_update   0: the whole verified tensor of the response is overwritten on an adaptive step;
 *              1: only the selected rows are written back (appendix "Design Choice Between Full
 *              V-Cache Overwrite and Selective Update") */
int dllmc_set_policy(dllmc_ctx* ctx, int32_t source, int32_t metric, int32_t selection,
                     int32_t v_update, uint32_t seed);

/* Update ratio per layer (appendix "Layer-wise token selection": the selection is local to a
 * layer; its cross-layer study gives layers different ratios under one average budget): on an
 * adaptive step layer l recomputes floor(rho_layers[l] * L_r) response rows per sequence.
 * rho_layers: HOST array of n_layers floats in [0, 1], copied; NULL returns to the single ratio
 * given at dllmc_create.  n_layers must equal the model's.  Takes effect at the next
 * dllmc_step.  With it, dllmc_step's n_sel reports the largest count over the layers and the
 * first dllmc_layer_num_selected(ctx, l) entries of sel_idx[l][b][:] are valid on an adaptive
 * step.  DLLMC_EINVAL on a ratio outside [0, 1] (nothing is changed then) or a wrong count. */
int dllmc_set_layer_rho(dllmc_ctx* ctx, const float* rho_layers, int32_t n_layers);
int32_t dllmc_layer_num_selected(const dllmc_ctx* ctx, int32_t layer);

/* One denoising step (Sec. 3.2 "Iterative Steps").
 *   hidden_in  device [B, L_p+L_r, d], model dtype: embedded tokens of this step.
 *   step_idx   0 for the first call (fills both caches), then strictly increasing; passing 0
 *              again starts a new generation (a full refresh).
 *   hidden_out device [B, L_p+L_r, d], model dtype: residual stream after the last layer
 *              (no final norm).  Prompt rows are the values of the last prompt refresh.
 *   sel_idx    device [n_layers, B, L_r] int32, may be NULL.  For each layer and sequence the
 *              first *n_sel entries are the response-row indices (0-based inside the
 *              response) that were recomputed, ascending; the rest is left untouched.
 *   n_sel      host out, may be NULL: floor(rho*L_r) on adaptive steps, L_r on refresh steps.
 * hidden_in and hidden_out may alias. */
int dllmc_step(dllmc_ctx* ctx, const void* hidden_in, int32_t step_idx, void* hidden_out,
               int32_t* sel_idx, int32_t* n_sel);

/* Copy one layer's cache tensor to `dst_device`, laid out [B, L_p+L_r, width] in the model
 * dtype.  which: 0 = K (width d_kv), 1 = V (d_kv), 2 = AttnOut (d), 3 = FFNOut (d). */
int dllmc_read_cache(dllmc_ctx* ctx, int32_t layer, int32_t which, void* dst_device);

/* Copy the V-verify scores s_j (Eq. cos_sim) of the most recent adaptive step to
 * `dst_device`, float32 [n_layers, B, L_r]. */
int dllmc_read_scores(dllmc_ctx* ctx, float* dst_device);

/* Optional per-kernel timing.  While enabled, dllmc_step records one HIP event on the context's
 * stream after every kernel launch (and one when the step starts); a kernel's time is the
 * interval between the events before and after it, so it includes the dispatch gap.  dllmc_profile_read waits for the stream, adds the
 * elapsed times to running totals per kernel class and copies the totals to `out`
 * (DLLMC_NUM_KERNEL_CLASSES entries); reset != 0 clears the totals afterwards.  alg_bytes and
 * flops are the algorithmic figures of the launches (for a gathered linear map: weights and
 * activation rows read once, float32 result written once; 2*M*N*K flops). */
enum {
  DLLMC_KC_GEMM_V = 0, DLLMC_KC_GEMM_QK, DLLMC_KC_GEMM_O, DLLMC_KC_GEMM_GATE_UP,
  DLLMC_KC_GEMM_DOWN, DLLMC_KC_ATTENTION, DLLMC_KC_SELECT, DLLMC_KC_ROW, DLLMC_KC_LISTS,
  DLLMC_KC_EVENT_OVERHEAD, /* an empty span per step: what one event record adds to a span */
  DLLMC_KC_STREAM_KERNEL,  /* the launches of the five gemm classes that ran the weight-streaming
                              kernel (k_gemm_stream), counted here a second time: one kernel's
                              figures, comparable with a profiler's per-kernel average */
  DLLMC_KC_HEAD_GEMM,      /* closed loop: vocabulary projection of the masked rows */
  DLLMC_KC_GEN_OTHER,      /* closed loop: final norm, greedy token + confidence, eligibility,
                              the two selections, token update (the embedding gather runs before
                              the step's first event and is not timed) */
  DLLMC_NUM_KERNEL_CLASSES
};
typedef struct {
  int64_t launches;
  double ms;
  double alg_bytes;
  double flops;
} dllmc_kernel_stat;
int dllmc_profile_enable(dllmc_ctx* ctx, int32_t on);
int dllmc_profile_read(dllmc_ctx* ctx, dllmc_kernel_stat* out, int32_t reset);
const char* dllmc_kernel_class_name(int32_t cls);

int dllmc_destroy(dllmc_ctx* ctx);

const char* dllmc_strerror(int code);
/* hipError_t value of the most recent failed HIP call made by the library on the calling thread,
 * 0 if none. */
int dllmc_last_hip_error(void);

/* ---- closed denoising loop around the cached step -------------------------------------
 * Paper Sec. 3.1: the response starts fully masked; every step embeds the current tokens, runs
 * the (cached) mask predictor, takes the greedy estimate of the clean sequence (per-position
 * argmax) and applies the transition S of Eq. (transition_step).  S is low-confidence remasking
 * (appendix "Experimental Details"): the response is cut into blocks of block_len positions
 * completed left to right, steps / (L_r / block_len) steps per block; a step reveals, among the
 * still masked positions of the current block, those whose greedy token has the highest softmax
 * probability (equal probabilities: lower position first; equal logits: lower token id); the
 * block's positions are spread evenly over its steps, the first block_len % steps_per_block
 * steps reveal one more.  Revealed tokens never change.  The predictor's head is RMSNorm with
 * final_norm_g followed by the vocabulary projection lm_head.
 * All pointers are device pointers, borrowed for the life of the object.  Token ids are int32
 * in [0, vocab]; vocab is the id of [MASK] and the index of its row in `embed`. */
typedef struct {
  const void* embed;        /* [vocab + 1, d_model], model dtype */
  const void* final_norm_g; /* [d_model] */
  const void* lm_head;      /* [vocab, d_model], row-major */
  int32_t vocab;
  int32_t steps;            /* denoising steps of one generation */
  int32_t block_len;        /* 0 = L_r; must divide L_r, and L_r / block_len must divide steps */
} dllmc_gen_config;
typedef struct dllmc_gen dllmc_gen;

/* Bytes of device workspace a generation loop on `ctx` needs (0: invalid arguments). */
size_t dllmc_gen_workspace_bytes(const dllmc_ctx* ctx, const dllmc_gen_config* cfg);
/* Creates the loop object on an existing context (whose stream it uses; the context must
 * outlive it and must not be stepped by anyone else in between).  workspace: 256-byte aligned,
 * caller-owned. */
int dllmc_gen_create(dllmc_gen** out, dllmc_ctx* ctx, const dllmc_gen_config* cfg, void* workspace,
                     size_t workspace_bytes);
/* One step of the loop, enqueued on the context's stream: tokens [B, L_p + L_r] (in/out) are
 * embedded, dllmc_step(step_idx) runs (sel_idx and n_sel as there, both may be null), the still
 * masked positions of the current block get their greedy token and confidence, and
 * *n_revealed (host, may be null) of them per sequence are revealed in `tokens`.  step_idx
 * follows dllmc_step's rules and must be < steps.  `tokens` must be the state this loop
 * produced (step 0: the whole response is [MASK]): the number of masked positions per block is
 * taken from the schedule, not counted. */
int dllmc_gen_step(dllmc_gen* gen, int32_t* tokens, int32_t step_idx, int32_t* sel_idx,
                   int32_t* n_sel, int32_t* n_revealed);
/* Results of the most recent dllmc_gen_step, copied on the stream (each destination may be
 * null): x0 [B, L_r] greedy tokens and conf [B, L_r] their probabilities, valid at the positions
 * that were masked inside the step's block (-1 / -inf elsewhere); chosen [B, L_r]: the first
 * n_revealed entries of each row are the revealed positions, ascending; hidden_out
 * [B, L_p + L_r, d_model] the step's output rows. */
int dllmc_gen_read(dllmc_gen* gen, int32_t* x0, float* conf, int32_t* chosen, void* hidden_out);
int dllmc_gen_destroy(dllmc_gen* gen);

/* Head of the mask predictor as a single operation: for i < M, row r = rows[i] (i if rows is
 * null) of hidden [*, d]: x0[i] = first argmax and conf[i] = softmax maximum of
 * rmsnorm(hidden[r]) * final_norm_g projected by lm_head [vocab, d].  scratch: at least
 * dllmc_op_head_scratch_bytes(dtype, M, vocab, d) bytes, 256-byte aligned. */
size_t dllmc_op_head_scratch_bytes(int32_t dtype, int32_t M, int32_t vocab, int32_t d);
int dllmc_op_head(int32_t dtype, const void* hidden, const int32_t* rows, int32_t M,
                  const void* final_norm_g, float eps, const void* lm_head, int32_t vocab, int32_t d,
                  void* scratch, int32_t* x0, float* conf, void* hip_stream);

/* Tuning knobs of the bf16 matrix products, for tests and measurements.  The call changes the
 * process default (thread-safe); a context copies the default when it is created and keeps its
 * copy for life, so live contexts are not affected; the single operations (dllmc_op_*) and the
 * closed loop's head use the default in force when they are called.  An argument outside its
 * range leaves that knob unchanged: nw wavefronts per workgroup (4|8) of the single-matrix kernel; nw_dual
 * shape of the fused gate/up kernel: 4|8 wavefronts in one group, or 100 + (4|6|8): the
 * wavefronts form two groups that each walk one half of the contraction range (default 106:
 * 48 columns of each matrix per workgroup); force_s number of contraction slices
 * (0 = automatic), target_wg
 * workgroups the automatic choice aims for, tile_min_m / fat_min_m number of activation rows
 * (defaults 192 / 512) from which the 128 x 128 / the 256 x 256 LDS-direct tile kernel replaces
 * the weight-streaming kernel; tall_max_m (default 128; 0 = off): from 128 on, launches of 65..128
 * rows run the weight-streaming kernel with 128 rows per workgroup (weights streamed once
 * instead of once per 64-row tile); from 256 on, launches of tile_min_m .. tall_max_m rows use
 * it with 256 rows per workgroup instead of the 128 x 128 tiles.
 * Results are
 * bit-reproducible for fixed settings; different settings change the float32 summation order
 * only. */
int dllmc_set_gemm_tuning(int32_t nw, int32_t nw_dual, int32_t force_s, int32_t target_wg,
                          int32_t tile_min_m, int32_t fat_min_m, int32_t tall_max_m);

/* Host-only: the number of contraction-index slices the library would use for a gathered
 * linear map of M rows, N columns (the first N0 from one matrix), contraction length K, given a
 * float32 slice buffer of capacity_floats elements and 16-byte aligned operands; 0 if M*N
 * floats do not fit.  slices * M * N never exceeds capacity_floats. */
int32_t dllmc_plan_gemm_slices(int32_t dtype, int32_t M, int32_t N, int32_t N0, int32_t K,
                               size_t capacity_floats);

/* ---- single operations of the step, exposed for unit parity tests and micro-benchmarks ---- */

/* Bottom-k selection (Sec. 3.2.2): for each of B rows of `scores` (device float32 [B, L]),
 * write the indices of the k lowest values, ascending by index, to idx_out (device int32
 * [B, k]); equal values are taken lowest index first.  0 <= k <= L. */
int dllmc_op_select(const float* scores, int32_t B, int32_t L, int32_t k, int32_t* idx_out,
                    void* hip_stream);

/* V-verify (Sec. 3.2.2, Eq. cos_sim): V_new = h * Wv^T for `rows` rows, rounded to the model
 * dtype; scores[r] = cos(V_new[r], v_cache[r]) with the denominator clamped at 1e-8; then
 * v_cache[r] <- V_new[r].  h: device [rows, d]; wv: [d_kv, d]; v_cache: [rows, d_kv];
 * scores: float32 [rows]; scratch: device float32 [rows * d_kv * 8]. */
int dllmc_op_vverify(int32_t dtype, const void* h, const void* wv, void* v_cache, float* scores,
                     int32_t rows, int32_t d, int32_t d_kv, float* scratch, void* hip_stream);

/* Gathered linear map: out[i, :] = a[row_idx[i], :] * w^T in float32, i < M.  a: device
 * [*, K] model dtype; row_idx: device int32 [M] or NULL for the identity; w: [N, K];
 * out: float32 [M, N]; scratch: device float32 [M * N * 8]. */
int dllmc_op_linear(int32_t dtype, const void* a, const int32_t* row_idx, int32_t M, const void* w,
                    int32_t N, int32_t K, float* out, float* scratch, void* hip_stream);

/* dllmc_op_linear for callers that cannot allocate device memory or pass a scratch buffer
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the
 * float32 slices of the split contraction go to a buffer that is part of the library's device
 * image, 32 MiB on every GPU the library runs on, held until the process ends.  Same arguments
 * and results as dllmc_op_linear without `scratch`; the call allocates nothing.
 * M * N must not exceed dllmc_op_linear_static_max_elements() (8 Mi elements), else
 * DLLMC_ETOOBIG and nothing is launched; up to 1 Mi elements the slices, and with them every
 * bit of the result, are those of dllmc_op_linear.  All calls on one GPU share the one buffer:
 * calls that may overlap on a GPU (different streams or host threads) race and must be
 * serialised by the caller; calls on one stream are ordered. */
size_t dllmc_op_linear_static_max_elements(void);
int dllmc_op_linear_static(int32_t dtype, const void* a, const int32_t* row_idx, int32_t M,
                           const void* w, int32_t N, int32_t K, float* out, void* hip_stream);

/* Bidirectional attention of Mq query rows per sequence over all n cached keys of that
 * sequence, no mask (complexity appendix: the 4*r^*n*d term).  q, out: device [B, Mq, H_q*d_h];
 * k_cache, v_cache: device [B, n, H_kv*d_h]; all in the model dtype.  Query head a reads
 * key/value head a / (H_q/H_kv).  scratch: device memory of dllmc_op_attention_scratch_bytes()
 * bytes, or NULL; with it, small query sets have their key range split over workgroups. */
size_t dllmc_op_attention_scratch_bytes(void);
int dllmc_op_attention(int32_t dtype, const void* q, int32_t B, int32_t Mq, const void* k_cache,
                       const void* v_cache, int32_t n, int32_t H_q, int32_t H_kv, int32_t d_h,
                       void* out, float* scratch, void* hip_stream);

/* ---- achievable-peak probes (measurement aids, not steps of the method) ----
 * What this GPU delivers for the plainest kernels of each kind, so that a roofline fraction
 * can be quoted against a measured ceiling beside the published one.  All three only enqueue
 * one kernel on hip_stream; the caller times them.
 *   dllmc_probe_copy  dst[0..bytes) = src[0..bytes); device pointers, 16-byte aligned, bytes a
 *                     multiple of 16; moves bytes in and bytes out.
 *   dllmc_probe_read  reads src[0..bytes) once and writes nothing (sink: device, 4 bytes, is
 *                     only there to keep the loads alive).
 *   dllmc_probe_mfma  every wavefront of a grid that fills the chip issues, from registers,
 *                     iters * 8 independent 16x16x32 bf16 MFMAs (shape 0) or iters * 4
 *                     independent 32x32x16 ones (shape 1; the same flops); *flops_out (host,
 *                     may be NULL) = the flops of the launch; sink: device float32 [256],
 *                     16-byte aligned, overwritten. */
int dllmc_probe_copy(const void* src, void* dst, size_t bytes, void* hip_stream);
int dllmc_probe_read(const void* src, size_t bytes, void* sink, void* hip_stream);
int dllmc_probe_mfma(int32_t iters, int32_t shape, float* sink, double* flops_out, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DLLMC_H */
