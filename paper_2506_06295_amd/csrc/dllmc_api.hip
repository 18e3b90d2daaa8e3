// Host side of libdllmc.so: the C ABI, the context (workspace carving, cache schedule of
// paper Sec. 3.2) and the per-layer launch sequence of one denoising step.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/dllmc.h"
#include "common.hpp"
#include "paging_host.hpp"

using namespace dllmc;

namespace {

thread_local int g_last_hip_error = 0;

inline int hip_fail(hipError_t e) {
  g_last_hip_error = static_cast<int>(e);
  return DLLMC_EHIP;
}
#define HIP_TRY(expr)                             \
  do {                                            \
    hipError_t e__ = (expr);                      \
    if (e__ != hipSuccess) return hip_fail(e__);  \
  } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

bool model_ok(const dllmc_model* m, int L_p, int L_r) {
  if (!m) return false;
  if (m->n_layers < 1 || m->d_model < 1 || m->n_q_heads < 1 || m->n_kv_heads < 1 ||
      m->head_dim < 2 || m->d_ffn < 1 || m->batch < 1)
    return false;
  if (m->head_dim % 2 || m->n_q_heads % m->n_kv_heads) return false;
  if (m->dtype != DLLMC_F32 && m->dtype != DLLMC_BF16) return false;
  if (!(m->rms_eps >= 0.f) || !(m->rope_theta > 0.f)) return false;
  if (L_p < 0 || L_r < 1) return false;
  const long long rows = static_cast<long long>(m->batch) * (static_cast<long long>(L_p) + L_r);
  if (rows > (1ll << 24)) return false;  // row ids and compact indices are int32 with headroom
  if (!attention_supported(m->dtype, m->head_dim, L_p + L_r)) return false;
  return true;
}

// Carving of the caller's workspace.  Every region starts 256-byte aligned.
struct Layout {
  size_t esz;
  size_t cws_floats;  // capacity of the GEMM slice buffer
  size_t cache_k, cache_v, cache_ao, cache_fo;  // per-layer strides inside their regions
  size_t off_k, off_v, off_ao, off_fo, off_prompt_out, off_x, off_h, off_q, off_a, off_g, off_u,
      off_cws, off_attn, off_scores, off_part, off_carried, off_rows, off_inv, off_rope, off_rmap,
      pool_total, total;
};

// cache_rows: rows of a layer's cache tensors (B * n flat, pool_pages * page_rows paged);
// caches_inside: whether the workspace holds them (false: a caller-owned pool does).
Layout make_layout(const dllmc_model& m, int L_p, int L_r, size_t cache_rows = 0,
                   bool caches_inside = true, bool paged = false) {
  Layout L{};
  const size_t esz = m.dtype == DLLMC_BF16 ? 2 : 4;
  const size_t B = m.batch, n = static_cast<size_t>(L_p) + L_r, T = m.n_layers;
  const size_t d = m.d_model, d_q = static_cast<size_t>(m.n_q_heads) * m.head_dim,
               d_kv = static_cast<size_t>(m.n_kv_heads) * m.head_dim, mf = m.d_ffn;
  const size_t rows = B * n;
  if (cache_rows == 0) cache_rows = rows;
  L.esz = esz;
  L.cache_k = L.cache_v = align_up(cache_rows * d_kv * esz, 256);
  L.cache_ao = L.cache_fo = align_up(cache_rows * d * esz, 256);
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o += align_up(bytes, 256); return r; };
  L.off_k = take(L.cache_k * T);
  L.off_v = take(L.cache_v * T);
  L.off_ao = take(L.cache_ao * T);
  L.off_fo = take(L.cache_fo * T);
  L.pool_total = o;
  if (!caches_inside) o = 0;  // the four regions above are offsets into the caller's pool
  L.off_rmap = paged ? take(rows * sizeof(int)) : 0;
  L.off_prompt_out = take(B * L_p * d * esz);
  L.off_x = take(rows * d * sizeof(float));
  L.off_h = take(rows * d * esz);
  L.off_q = take(rows * d_q * esz);
  L.off_a = take(rows * d_q * esz);
  L.off_g = take(rows * d * esz);
  L.off_u = take(rows * mf * esz);
  size_t n_max = 2 * mf;
  if (d_q + d_kv > n_max) n_max = d_q + d_kv;
  if (d > n_max) n_max = d;
  // GEMM output slices: the slice count S is chosen so that S*tiles < 512 + tiles workgroup
  // tiles (of at most 128 x 128 floats), and S*M*N <= S*tiles*tile
  const size_t cws_floats = align_up(rows, 128) * n_max + static_cast<size_t>(640) * 128 * 128;
  L.cws_floats = cws_floats;
  L.off_cws = take(cws_floats * sizeof(float));
  // split-key attention partials: only small query sets are split, the bound is the launcher's
  L.off_attn = take(attention_scratch_floats() * sizeof(float));
  L.off_scores = take(T * B * L_r * sizeof(float));
  // per (response row, column tile) sums of the fused V-verify launch
  L.off_part = take(vverify_part_floats(static_cast<int>(d_kv), B * L_r) * sizeof(float));
  L.off_carried = take(rows * sizeof(int));
  L.off_rows = take(rows * sizeof(int));
  L.off_inv = take(rows * sizeof(int));
  L.off_rope = take(n * (m.head_dim / 2) * sizeof(float2));
  L.total = o;
  return L;
}

}  // namespace

struct dllmc_ctx {
  dllmc_model m;
  std::vector<dllmc_layer_weights> layers;
  int L_p, L_r, n, k_sel, K_p, K_r;
  float rho;
  hipStream_t st;
  int last_step;
  Layout lay;
  char* ws;
  char* cache_base;          // where the four cache regions start: the workspace or a caller's pool
  bool have_scores;
  // paged layout (page_rows == 0: flat)
  int page_rows = 0, pool_pages = 0;
  const int* rmap = nullptr; // device: cache row of every logical row b * n + position
  // variants of the paper's ablations (dllmc_set_policy); defaults are the paper's method
  int metric = 0;          // 0 cosine, 1 minus L2 distance
  bool source_k = false;   // K-verify: Keys are scored and overwritten, Values follow the selection
  bool random_sel = false;
  bool v_selected_only = false;
  uint32_t seed = 0;
  std::vector<int> k_layer;  // rows recomputed per sequence on adaptive steps, per layer
  GemmTuning tune;           // kernel-choice knobs, copied from the process default at creation

  // optional per-kernel timing with HIP events on the context's stream
  bool profiling = false;
  struct Span { hipEvent_t a, b; int cls; double bytes, flops; bool stream_kernel; };
  std::vector<Span> spans;           // recorded, not yet read back
  std::vector<hipEvent_t> free_events;
  std::vector<hipEvent_t> step_open_events;  // opening events of profiled steps, not yet recycled
  hipEvent_t last_event = nullptr;           // event that closed the most recent span
  dllmc_kernel_stat totals[DLLMC_NUM_KERNEL_CLASSES] = {};

  hipEvent_t get_event() {
    if (!free_events.empty()) { hipEvent_t e = free_events.back(); free_events.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }

  template <typename T> T* at(size_t off) const { return reinterpret_cast<T*>(ws + off); }
  void* cache(int which, int layer) const {
    switch (which) {
      case 0: return cache_base + lay.off_k + lay.cache_k * layer;
      case 1: return cache_base + lay.off_v + lay.cache_v * layer;
      case 2: return cache_base + lay.off_ao + lay.cache_ao * layer;
      default: return cache_base + lay.off_fo + lay.cache_fo * layer;
    }
  }
};

namespace {
// Times the launches issued while it is alive: the span runs from the event that closed the
// previous span (or the step's opening event) to an event recorded when this object dies, so
// consecutive kernels are separated by a single event and the spans of a step add up to the
// step's duration.  Only active while profiling is on.
struct Timed {
  dllmc_ctx* c;
  int cls; double bytes, flops;
  Timed(dllmc_ctx* c_, int cls_, double bytes_, double flops_) : c(c_), cls(cls_), bytes(bytes_), flops(flops_) {}
  ~Timed() {
    if (!c->profiling || !c->last_event) return;
    hipEvent_t b = c->get_event();
    if (!b) return;
    (void)hipEventRecord(b, c->st);
    const bool is_gemm = (cls >= DLLMC_KC_GEMM_V && cls <= DLLMC_KC_GEMM_DOWN) || cls == DLLMC_KC_HEAD_GEMM;
    c->spans.push_back({c->last_event, b, cls, bytes, flops, is_gemm && gemm_last_was_stream()});
    c->last_event = b;
  }
};
}  // namespace

extern "C" {

}  // extern "C"

namespace {

bool paging_shape_ok(const dllmc_model* m, const dllmc_paging* pg) {
  if (!pg || pg->page_rows < 1 || pg->pool_pages < 1) return false;
  const long long rows = static_cast<long long>(pg->page_rows) * pg->pool_pages;
  return m && rows <= (1ll << 30);
}

Layout layout_for(const dllmc_model& m, int L_p, int L_r, const dllmc_paging* pg) {
  if (!pg) return make_layout(m, L_p, L_r);
  return make_layout(m, L_p, L_r, static_cast<size_t>(pg->page_rows) * pg->pool_pages,
                     pg->pool == nullptr, true);
}

int create_impl(dllmc_ctx** out, const dllmc_model* model, const dllmc_layer_weights* layers,
                int32_t L_p, int32_t L_r, float rho, int32_t K_p, int32_t K_r,
                const dllmc_paging* pg, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!out) return DLLMC_EINVAL;
  *out = nullptr;
  if (!model_ok(model, L_p, L_r) || !layers || !workspace) return DLLMC_EINVAL;
  if (!(rho >= 0.f && rho <= 1.f) || K_p < 1 || K_r < 1) return DLLMC_EINVAL;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return DLLMC_EINVAL;
  for (int l = 0; l < model->n_layers; ++l) {
    const void* ps[9] = {layers[l].attn_norm_g, layers[l].wq, layers[l].wk, layers[l].wv,
                         layers[l].wo, layers[l].ffn_norm_g, layers[l].w_gate, layers[l].w_up,
                         layers[l].w_down};
    for (const void* p : ps)
      if (!p || (reinterpret_cast<uintptr_t>(p) & 15u)) return DLLMC_EINVAL;
  }
  std::vector<int> row_map;
  if (pg) {
    if (!paging_shape_ok(model, pg) || !pg->page_table) return DLLMC_EINVAL;
    if (pg->pool && (reinterpret_cast<uintptr_t>(pg->pool) & 255u)) return DLLMC_EINVAL;
    row_map = build_row_map(model->batch, L_p + L_r, pg->page_rows, pg->pool_pages, pg->page_table);
    if (row_map.empty()) return DLLMC_EINVAL;
  }
  const Layout lay = layout_for(*model, L_p, L_r, pg);
  if (workspace_bytes < lay.total) return DLLMC_ENOMEM;
  if (pg && pg->pool && pg->pool_bytes < lay.pool_total) return DLLMC_ENOMEM;

  dllmc_ctx* c = new (std::nothrow) dllmc_ctx();
  if (!c) return DLLMC_ENOMEM;
  c->m = *model;
  c->layers.assign(layers, layers + model->n_layers);
  c->L_p = L_p;
  c->L_r = L_r;
  c->n = L_p + L_r;
  c->rho = rho;
  c->K_p = K_p;
  c->K_r = K_r;
  // floor(rho * |y|), |y| = response length (Sec. 3.2.2)
  c->k_sel = static_cast<int>(std::floor(static_cast<double>(rho) * L_r + 1e-6));
  if (c->k_sel > L_r) c->k_sel = L_r;
  c->k_layer.assign(model->n_layers, c->k_sel);
  c->tune = gemm_default_tuning();
  c->st = static_cast<hipStream_t>(hip_stream);
  c->last_step = -1;
  c->lay = lay;
  c->ws = static_cast<char*>(workspace);
  c->cache_base = (pg && pg->pool) ? static_cast<char*>(pg->pool) : c->ws;
  c->have_scores = false;
  if (pg) {
    c->page_rows = pg->page_rows;
    c->pool_pages = pg->pool_pages;
    c->rmap = c->at<int>(lay.off_rmap);
  }

  // RoPE table in double on the host: (cos, sin)(pos * theta^(-2t/d_h))
  const int half = model->head_dim / 2;
  std::vector<float2> tab(static_cast<size_t>(c->n) * half);
  for (int pos = 0; pos < c->n; ++pos)
    for (int t = 0; t < half; ++t) {
      const double w = std::pow(static_cast<double>(model->rope_theta),
                                -2.0 * t / static_cast<double>(model->head_dim));
      const double ang = pos * w;
      tab[static_cast<size_t>(pos) * half + t] =
          make_float2(static_cast<float>(std::cos(ang)), static_cast<float>(std::sin(ang)));
    }
  hipError_t e = hipMemcpyAsync(c->ws + lay.off_rope, tab.data(), tab.size() * sizeof(float2),
                                hipMemcpyHostToDevice, c->st);
  if (e == hipSuccess && pg)
    e = hipMemcpyAsync(c->ws + lay.off_rmap, row_map.data(), row_map.size() * sizeof(int),
                       hipMemcpyHostToDevice, c->st);
  if (e == hipSuccess) e = hipStreamSynchronize(c->st);
  if (e != hipSuccess) {
    delete c;
    return hip_fail(e);
  }
  *out = c;
  return DLLMC_OK;
}

}  // namespace

extern "C" {

size_t dllmc_workspace_bytes(const dllmc_model* model, int32_t L_p, int32_t L_r) {
  if (!model_ok(model, L_p, L_r)) return 0;
  return make_layout(*model, L_p, L_r).total;
}

size_t dllmc_pool_bytes(const dllmc_model* model, int32_t page_rows, int32_t pool_pages) {
  dllmc_paging pg{page_rows, pool_pages, nullptr, nullptr, 0};
  if (!model_ok(model, 0, 1) || !paging_shape_ok(model, &pg)) return 0;
  return make_layout(*model, 0, 1, static_cast<size_t>(page_rows) * pool_pages, false, true).pool_total;
}

size_t dllmc_workspace_bytes_paged(const dllmc_model* model, int32_t L_p, int32_t L_r,
                                   const dllmc_paging* paging) {
  if (!model_ok(model, L_p, L_r) || !paging_shape_ok(model, paging)) return 0;
  return layout_for(*model, L_p, L_r, paging).total;
}

int dllmc_create(dllmc_ctx** out, const dllmc_model* model, const dllmc_layer_weights* layers,
                 int32_t L_p, int32_t L_r, float rho, int32_t K_p, int32_t K_r, void* workspace,
                 size_t workspace_bytes, void* hip_stream) {
  return create_impl(out, model, layers, L_p, L_r, rho, K_p, K_r, nullptr, workspace, workspace_bytes,
                     hip_stream);
}

int dllmc_create_paged(dllmc_ctx** out, const dllmc_model* model, const dllmc_layer_weights* layers,
                       int32_t L_p, int32_t L_r, float rho, int32_t K_p, int32_t K_r,
                       const dllmc_paging* paging, void* workspace, size_t workspace_bytes,
                       void* hip_stream) {
  if (!paging) return DLLMC_EINVAL;
  return create_impl(out, model, layers, L_p, L_r, rho, K_p, K_r, paging, workspace, workspace_bytes,
                     hip_stream);
}

int dllmc_set_page_table(dllmc_ctx* c, const int32_t* page_table) {
  if (!c || !page_table || c->page_rows == 0) return DLLMC_EINVAL;
  const std::vector<int> row_map = build_row_map(c->m.batch, c->n, c->page_rows, c->pool_pages, page_table);
  if (row_map.empty()) return DLLMC_EINVAL;
  HIP_TRY(hipStreamSynchronize(c->st));  // nothing in flight may still read the old map
  HIP_TRY(hipMemcpyAsync(c->ws + c->lay.off_rmap, row_map.data(), row_map.size() * sizeof(int),
                         hipMemcpyHostToDevice, c->st));
  HIP_TRY(hipStreamSynchronize(c->st));
  c->last_step = -1;  // the caches are void: a full refresh (step 0) comes next
  c->have_scores = false;
  return DLLMC_OK;
}

int32_t dllmc_num_selected(const dllmc_ctx* ctx) { return ctx ? ctx->k_sel : DLLMC_EINVAL; }

int32_t dllmc_layer_num_selected(const dllmc_ctx* ctx, int32_t layer) {
  if (!ctx || layer < 0 || layer >= ctx->m.n_layers) return DLLMC_EINVAL;
  return ctx->k_layer[layer];
}

int dllmc_set_layer_rho(dllmc_ctx* c, const float* rho_layers, int32_t n_layers) {
  if (!c) return DLLMC_EINVAL;
  if (!rho_layers) {
    c->k_layer.assign(c->m.n_layers, c->k_sel);
    return DLLMC_OK;
  }
  if (n_layers != c->m.n_layers) return DLLMC_EINVAL;
  for (int l = 0; l < n_layers; ++l)
    if (!(rho_layers[l] >= 0.f && rho_layers[l] <= 1.f)) return DLLMC_EINVAL;
  for (int l = 0; l < n_layers; ++l) {
    int k = static_cast<int>(std::floor(static_cast<double>(rho_layers[l]) * c->L_r + 1e-6));
    c->k_layer[l] = k > c->L_r ? c->L_r : k;
  }
  return DLLMC_OK;
}

int dllmc_set_policy(dllmc_ctx* c, int32_t source, int32_t metric, int32_t selection,
                     int32_t v_update, uint32_t seed) {
  if (!c || source < 0 || source > 1 || metric < 0 || metric > 1 || selection < 0 || selection > 1 ||
      v_update < 0 || v_update > 1)
    return DLLMC_EINVAL;
  c->source_k = source == 1;
  c->metric = metric;
  c->random_sel = selection == 1;
  c->v_selected_only = v_update == 1;
  c->seed = seed;
  return DLLMC_OK;
}

int dllmc_step(dllmc_ctx* c, const void* hidden_in, int32_t step_idx, void* hidden_out,
               int32_t* sel_idx, int32_t* n_sel) {
  if (!c || !hidden_in || !hidden_out || step_idx < 0) return DLLMC_EINVAL;
  if (step_idx != 0 && (c->last_step < 0 || step_idx <= c->last_step)) return DLLMC_ESTATE;
  (void)hipGetLastError();  // do not inherit a stale error
  const TuningScope tuning(&c->tune);

  const dllmc_model& m = c->m;
  const int B = m.batch, n = c->n, L_p = c->L_p, L_r = c->L_r, T = m.n_layers;
  const int d = m.d_model, d_h = m.head_dim, d_q = m.n_q_heads * d_h, d_kv = m.n_kv_heads * d_h;
  const int mf = m.d_ffn, dt = m.dtype;
  hipStream_t st = c->st;

  // Sec. 3.2 "Iterative Steps": which caches are refreshed at this step
  const bool P = (step_idx % c->K_p == 0) && L_p > 0;
  const bool Rf = (step_idx % c->K_r == 0);
  const int carried_per_seq = (P ? L_p : 0) + L_r;
  const int Mc = B * carried_per_seq;
  const int sel_off = P ? L_p : 0;
  // response rows recomputed per sequence at layer l, and with the refreshed prompt rows
  auto sel_of = [&](int l) { return Rf ? L_r : c->k_layer[l]; };
  auto per_seq_of = [&](int l) { return sel_off + sel_of(l); };
  if (n_sel) {
    int mx = 0;
    for (int l = 0; l < T; ++l) mx = std::max(mx, sel_of(l));
    *n_sel = mx;
  }

  const RowKernelArgs ra{dt, n, L_p, d, m.rms_eps};
  int* carried = c->at<int>(c->lay.off_carried);
  int* rows_R = c->at<int>(c->lay.off_rows);
  int* inv = c->at<int>(c->lay.off_inv);
  float* x = c->at<float>(c->lay.off_x);
  void* h = c->ws + c->lay.off_h;
  void* qbuf = c->ws + c->lay.off_q;
  void* abuf = c->ws + c->lay.off_a;
  void* gbuf = c->ws + c->lay.off_g;
  void* ubuf = c->ws + c->lay.off_u;
  float* cws = c->at<float>(c->lay.off_cws);
  const size_t cws_cap = c->lay.cws_floats;
  float* scores = c->at<float>(c->lay.off_scores);
  float* part = c->at<float>(c->lay.off_part);
  void* prompt_out = c->ws + c->lay.off_prompt_out;
  const float2* rope_tab = c->at<float2>(c->lay.off_rope);
  const int* rmap = c->rmap;  // paged layout: cache row of every logical row (nullptr: flat)

  c->last_event = nullptr;
  if (c->profiling) {
    c->last_event = c->get_event();
    if (c->last_event) {
      (void)hipEventRecord(c->last_event, st);
      c->step_open_events.push_back(c->last_event);
      Timed empty(c, DLLMC_KC_EVENT_OVERHEAD, 0, 0);  // nothing launched inside this span
    }
  }
  const double esz = static_cast<double>(c->lay.esz);
  // algorithmic bytes / flops of one gathered linear map: weights, activations in, float32 out
  auto gemm_bytes = [&](double M, double N, double K) { return (N * K + M * K) * esz + M * N * 4.0; };
  auto gemm_flops = [&](double M, double N, double K) { return 2.0 * M * N * K; };

  // row lists of this step
  {
    Timed t(c, DLLMC_KC_LISTS, 0, 0);
    launch_iota_rows(carried, nullptr, B, n, P ? 0 : L_p, carried_per_seq, carried_per_seq, 0, st);
    if (P) launch_iota_rows(rows_R, inv, B, n, 0, L_p, per_seq_of(0), 0, st);
    if (Rf) {
      launch_iota_rows(rows_R, inv, B, n, L_p, L_r, per_seq_of(0), sel_off, st);
      if (sel_idx) launch_fill_sel_identity(sel_idx, T * B, L_r, st);
    }
  }
  {
    Timed t(c, DLLMC_KC_ROW, Mc * d * (2.0 * esz + 4.0), 0);
    launch_embed_norm(ra, hidden_in, carried, Mc, c->layers[0].attn_norm_g, x, h, st);
  }

  for (int l = 0; l < T; ++l) {
    const dllmc_layer_weights& w = c->layers[l];
    const int k_l = sel_of(l), per_seq = per_seq_of(l), M_R = B * per_seq;
    if (P && l > 0 && per_seq != per_seq_of(l - 1)) {
      // the compact list of recomputed rows is laid out with this layer's row count per
      // sequence: the refreshed prompt rows move to their new places
      Timed t(c, DLLMC_KC_LISTS, 0, 0);
      launch_iota_rows(rows_R, inv, B, n, 0, L_p, per_seq, 0, st);
    }
    void* Kc = c->cache(0, l);
    void* Vc = c->cache(1, l);
    // Verify: the verified projection (V; K for the K-verify variant) for every carried row,
    // scored against the cache, cache overwritten.  Refresh steps always go V first.
    const bool ksrc = c->source_k && !Rf;
    void* Tc = ksrc ? Kc : Vc;   // cache of the verified tensor
    int S = 1;
    float* sc = scores + static_cast<size_t>(l) * B * L_r;
    // selected-only update: the response rows' new rows wait in the attention output buffer
    // (free until this layer's attention) for the selection
    const bool defer_v = c->v_selected_only && !Rf;
    // The default method in one launch: projection, rounding, the sums of Eq. (cos_sim) per row
    // and column tile, cache overwrite (the selection kernel forms the scores): 64 x 64 tiles over
    // the whole contraction range for up to two tiles per CU, the epilogue of the 128 x 128 /
    // 256 x 256 tile kernels for launches that fill the chip in one slice; else the split
    // contraction and a row kernel.
    const bool want_scores = !Rf && !c->random_sel;
    bool fused_v = false;
    {
      Timed t(c, DLLMC_KC_GEMM_V, gemm_bytes(Mc, d_kv, d), gemm_flops(Mc, d_kv, d));
      if (!ksrc && !defer_v) {
        if (vverify_fused_ok(dt, h, d, Mc, w.wv, d_kv, d, Vc)) {
          gemm_clear_last_stream();
          launch_vverify_fused(h, d, Mc, P ? 0 : L_p, carried_per_seq, n, L_p, w.wv, d_kv, d, Vc,
                               want_scores ? part : nullptr, B * L_r, c->metric, st, rmap);
          fused_v = true;
        } else {
          fused_v = launch_gemm_vverify_tiles(dt, h, d, Mc, P ? 0 : L_p, carried_per_seq, n, L_p, w.wv,
                                              d_kv, d, Vc, want_scores ? part : nullptr, B * L_r,
                                              c->metric, rmap, st);
        }
      }
      if (fused_v) {
        t.bytes = (static_cast<double>(d_kv) * d + static_cast<double>(Mc) * d) * esz +
                  (Rf ? 1.0 : 2.0) * Mc * d_kv * esz;
      } else {
        S = launch_gemm(dt, h, d, carried, Mc, ksrc ? w.wk : w.wv, nullptr, d_kv, d_kv, d, cws, cws_cap,
                        st);
        if (S == 0) return DLLMC_ENOMEM;
      }
    }
    const bool part_scores = fused_v && want_scores;
    if (!fused_v) {
      Timed t(c, DLLMC_KC_ROW, Mc * d_kv * (4.0 + 2.0 * esz), 0);
      float* sc_out = (Rf || c->random_sel) ? nullptr : sc;
      if (ksrc)
        launch_k_finalize(ra, cws, S, carried, Mc, d_kv, d_h, rope_tab, Tc, sc_out, c->metric,
                          defer_v ? abuf : nullptr, st, rmap);
      else
        launch_v_finalize(ra, cws, S, P ? 0 : L_p, carried_per_seq, Mc, d_kv, Tc, sc_out, c->metric,
                          defer_v ? abuf : nullptr, st, rmap);
    }
    if (!Rf) {
      Timed t(c, DLLMC_KC_SELECT, B * (L_r * 4.0 + k_l * 8.0 + L_r * 4.0), 0);
      if (c->random_sel) launch_random_scores(c->seed, step_idx, l, B, L_r, sc, st);
      launch_select(sc, B, L_r, k_l,
                    sel_idx ? sel_idx + static_cast<size_t>(l) * B * L_r : nullptr, L_r, rows_R,
                    per_seq, sel_off, inv, n, L_p, st, part_scores ? part : nullptr,
                    vverify_col_tiles(d_kv), B * L_r, c->metric);
      if (defer_v)
        launch_scatter_v(ra, rows_R, M_R, P ? 0 : L_p, carried_per_seq, d_kv, abuf, Tc, st, rmap);
    }
    S = 1;
    if (M_R > 0) {
      bool qk_direct;
      {
        // Q and the other projection (K; V for K-verify) of the recomputed rows in one launch;
        // with enough rows to fill the chip in one slice, RoPE, the compact Q buffer and the cache
        // scatter happen in the tile kernel's epilogue
        Timed t(c, DLLMC_KC_GEMM_QK, gemm_bytes(M_R, d_q + d_kv, d), gemm_flops(M_R, d_q + d_kv, d));
        qk_direct = launch_gemm_qk_tiles(dt, h, d, rows_R, M_R, w.wq, ksrc ? w.wv : w.wk, d_q, d_kv, d_h,
                                         d, rope_tab, n, qbuf, ksrc ? Vc : Kc, !ksrc, rmap, st);
        if (!qk_direct) {
          S = launch_gemm(dt, h, d, rows_R, M_R, w.wq, ksrc ? w.wv : w.wk, d_q, d_q + d_kv, d, cws,
                          cws_cap, st);
          if (S == 0) return DLLMC_ENOMEM;
        }
      }
      if (!qk_direct) {
        Timed t(c, DLLMC_KC_ROW, M_R * (d_q + d_kv) * (4.0 + esz), 0);
        launch_qk_finalize(ra, cws, S, rows_R, M_R, d_q, d_kv, d_h, rope_tab, qbuf, ksrc ? Vc : Kc,
                           !ksrc, st, rmap);
      }
      {
        // queries in and out once, every sequence's K and V once per group of query heads
        Timed t(c, DLLMC_KC_ATTENTION, (2.0 * M_R * d_q + 2.0 * B * n * d_kv) * esz,
                4.0 * M_R * static_cast<double>(n) * d_q);
        launch_attention(dt, qbuf, B, per_seq, Kc, Vc, n, m.n_q_heads, m.n_kv_heads, d_h, abuf,
                         c->at<float>(c->lay.off_attn), st, rmap);
      }
      {
        Timed t(c, DLLMC_KC_GEMM_O, gemm_bytes(M_R, d, d_q), gemm_flops(M_R, d, d_q));
        S = launch_gemm(dt, abuf, d_q, nullptr, M_R, w.wo, nullptr, d, d, d_q, cws, cws_cap, st);
        if (S == 0) return DLLMC_ENOMEM;
      }
    }
    {
      Timed t(c, DLLMC_KC_ROW, M_R * d * (12.0 + 2.0 * esz), 0);
      launch_o_finalize(ra, cws, S, rows_R, M_R, c->cache(2, l), x, w.ffn_norm_g, gbuf, st, rmap);
    }
    if (M_R > 0) {
      bool fused;
      {
        Timed t(c, DLLMC_KC_GEMM_GATE_UP, gemm_bytes(M_R, 2.0 * mf, d), gemm_flops(M_R, 2.0 * mf, d));
        fused = launch_gemm_swiglu(dt, gbuf, d, nullptr, M_R, w.w_gate, w.w_up, mf, d, ubuf, st);
        if (!fused) S = launch_gemm(dt, gbuf, d, nullptr, M_R, w.w_gate, w.w_up, mf, 2 * mf, d, cws, cws_cap, st);
        if (S == 0) return DLLMC_ENOMEM;
      }
      if (!fused) {
        Timed t(c, DLLMC_KC_ROW, M_R * mf * (8.0 + esz), 0);
        launch_swiglu(dt, cws, S, M_R, mf, ubuf, st);
      }
      {
        Timed t(c, DLLMC_KC_GEMM_DOWN, gemm_bytes(M_R, d, mf), gemm_flops(M_R, d, mf));
        S = launch_gemm(dt, ubuf, mf, nullptr, M_R, w.w_down, nullptr, d, d, mf, cws, cws_cap, st);
        if (S == 0) return DLLMC_ENOMEM;
      }
    }
    const bool last = (l == T - 1);
    {
      Timed t(c, DLLMC_KC_ROW, Mc * d * (8.0 + 2.0 * esz) + M_R * d * 4.0 + (Mc - M_R) * d * esz, 0);
      launch_down_finalize(ra, cws, S, M_R, P ? 0 : L_p, carried_per_seq, Mc, inv, c->cache(2, l), c->cache(3, l), x,
                           last ? nullptr : c->layers[l + 1].attn_norm_g, h, hidden_out,
                           (last && P) ? prompt_out : nullptr, st, rmap);
    }
  }
  if (!P) {
    Timed t(c, DLLMC_KC_LISTS, 2.0 * B * L_p * d * esz, 0);
    launch_copy_prompt(ra, B, prompt_out, hidden_out, st);
  }

  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e);
  if (!Rf) c->have_scores = true;
  c->last_step = step_idx;
  return DLLMC_OK;
}

int dllmc_read_cache(dllmc_ctx* c, int32_t layer, int32_t which, void* dst_device) {
  if (!c || !dst_device || layer < 0 || layer >= c->m.n_layers || which < 0 || which > 3)
    return DLLMC_EINVAL;
  const size_t width = which < 2 ? static_cast<size_t>(c->m.n_kv_heads) * c->m.head_dim
                                 : static_cast<size_t>(c->m.d_model);
  const size_t bytes = static_cast<size_t>(c->m.batch) * c->n * width * c->lay.esz;
  if (c->rmap) {
    // paged layout: the rows gathered into logical order
    (void)hipGetLastError();
    launch_gather_rows(c->m.dtype, c->cache(which, layer), c->rmap, c->m.batch * c->n,
                       static_cast<int>(width), dst_device, c->st);
    HIP_TRY(hipGetLastError());
    return DLLMC_OK;
  }
  HIP_TRY(hipMemcpyAsync(dst_device, c->cache(which, layer), bytes, hipMemcpyDeviceToDevice, c->st));
  return DLLMC_OK;
}

int dllmc_read_scores(dllmc_ctx* c, float* dst_device) {
  if (!c || !dst_device) return DLLMC_EINVAL;
  if (!c->have_scores) return DLLMC_ESTATE;
  const size_t bytes = static_cast<size_t>(c->m.n_layers) * c->m.batch * c->L_r * sizeof(float);
  HIP_TRY(hipMemcpyAsync(dst_device, c->ws + c->lay.off_scores, bytes, hipMemcpyDeviceToDevice,
                         c->st));
  return DLLMC_OK;
}

int dllmc_profile_enable(dllmc_ctx* c, int32_t on) {
  if (!c) return DLLMC_EINVAL;
  c->profiling = on != 0;
  return DLLMC_OK;
}

int dllmc_profile_read(dllmc_ctx* c, dllmc_kernel_stat* out, int32_t reset) {
  if (!c || !out) return DLLMC_EINVAL;
  HIP_TRY(hipStreamSynchronize(c->st));
  for (const dllmc_ctx::Span& sp : c->spans) {
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, sp.a, sp.b));
    dllmc_kernel_stat& t = c->totals[sp.cls];
    t.launches += 1;
    t.ms += ms;
    t.alg_bytes += sp.bytes;
    t.flops += sp.flops;
    if (sp.stream_kernel) {
      dllmc_kernel_stat& k = c->totals[DLLMC_KC_STREAM_KERNEL];
      k.launches += 1;
      k.ms += ms;
      k.alg_bytes += sp.bytes;
      k.flops += sp.flops;
    }
    c->free_events.push_back(sp.b);  // sp.a is the previous span's b or a step's opening event
  }
  c->spans.clear();
  for (hipEvent_t ev : c->step_open_events) c->free_events.push_back(ev);
  c->step_open_events.clear();
  c->last_event = nullptr;
  std::memcpy(out, c->totals, sizeof(c->totals));
  if (reset) std::memset(c->totals, 0, sizeof(c->totals));
  return DLLMC_OK;
}

const char* dllmc_kernel_class_name(int32_t cls) {
  static const char* names[DLLMC_NUM_KERNEL_CLASSES] = {
      "gemm_v", "gemm_qk", "gemm_o", "gemm_gate_up", "gemm_down", "attention", "select",
      "row_kernels", "lists_and_copies", "event_overhead", "k_gemm_stream", "head_gemm",
      "gen_other"};
  return (cls >= 0 && cls < DLLMC_NUM_KERNEL_CLASSES) ? names[cls] : "?";
}

int dllmc_destroy(dllmc_ctx* c) {
  if (!c) return DLLMC_EINVAL;
  hipError_t e = hipStreamSynchronize(c->st);  // the workspace goes back to the caller idle
  for (const dllmc_ctx::Span& sp : c->spans) (void)hipEventDestroy(sp.b);
  for (hipEvent_t ev : c->step_open_events) (void)hipEventDestroy(ev);
  for (hipEvent_t ev : c->free_events) (void)hipEventDestroy(ev);
  delete c;
  if (e != hipSuccess) return hip_fail(e);
  return DLLMC_OK;
}

const char* dllmc_strerror(int code) {
  switch (code) {
    case DLLMC_OK: return "ok";
    case DLLMC_EINVAL: return "invalid argument";
    case DLLMC_ESTATE: return "call out of order (step 0 first, then increasing step_idx)";
    case DLLMC_EHIP: return "HIP runtime error";
    case DLLMC_ENOMEM: return "workspace too small";
    case DLLMC_ETOOBIG: return "problem larger than the library's static scratch buffer";
    default: return "unknown error";
  }
}

int dllmc_last_hip_error(void) { return g_last_hip_error; }

int32_t dllmc_plan_gemm_slices(int32_t dtype, int32_t M, int32_t N, int32_t N0, int32_t K,
                               size_t capacity_floats) {
  return gemm_plan_slices(dtype, M, N, N0, K, capacity_floats);
}

int dllmc_set_gemm_tuning(int32_t nw, int32_t nw_dual, int32_t force_s, int32_t target_wg,
                          int32_t tile_min_m, int32_t fat_min_m, int32_t tall_max_m) {
  gemm_set_tuning(nw, nw_dual, force_s, target_wg);
  gemm_set_tile_min_m(tile_min_m);
  gemm_set_fat_min_m(fat_min_m);
  gemm_set_tall_max_m(tall_max_m);
  return DLLMC_OK;
}

// ---- single operations ------------------------------------------------------------------

int dllmc_op_select(const float* scores, int32_t B, int32_t L, int32_t k, int32_t* idx_out,
                    void* hip_stream) {
  if (!scores || B < 1 || L < 1 || k < 0 || k > L || (k > 0 && !idx_out)) return DLLMC_EINVAL;
  (void)hipGetLastError();
  // without tile sums the scores are only read
  launch_select(const_cast<float*>(scores), B, L, k, idx_out, k, nullptr, 0, 0, nullptr, L, 0,
                static_cast<hipStream_t>(hip_stream));
  HIP_TRY(hipGetLastError());
  return DLLMC_OK;
}

int dllmc_op_vverify(int32_t dtype, const void* h, const void* wv, void* v_cache, float* scores,
                     int32_t rows, int32_t d, int32_t d_kv, float* scratch, void* hip_stream) {
  if ((dtype != DLLMC_F32 && dtype != DLLMC_BF16) || !h || !wv || !v_cache || !scores || !scratch ||
      rows < 1 || d < 1 || d_kv < 1)
    return DLLMC_EINVAL;
  (void)hipGetLastError();
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (vverify_fused_ok(dtype, h, d, rows, wv, d_kv, d, v_cache) &&
      vverify_part_floats(d_kv, rows) <= static_cast<size_t>(rows) * d_kv * 8) {
    launch_vverify_fused(h, d, rows, 0, 0, rows, 0, wv, d_kv, d, v_cache, scratch, rows, 0, st);
    launch_scores_from_part(scratch, vverify_col_tiles(d_kv), rows, 0, scores, st);
    HIP_TRY(hipGetLastError());
    return DLLMC_OK;
  }
  const int S = launch_gemm(dtype, h, d, nullptr, rows, wv, nullptr, d_kv, d_kv, d, scratch,
                            static_cast<size_t>(rows) * d_kv * 8, st);
  if (S == 0) return DLLMC_ENOMEM;
  const RowKernelArgs ra{dtype, rows, 0, d, 0.f};
  launch_v_finalize(ra, scratch, S, 0, 0, rows, d_kv, v_cache, scores, 0, nullptr, st);
  HIP_TRY(hipGetLastError());
  return DLLMC_OK;
}

int dllmc_op_linear(int32_t dtype, const void* a, const int32_t* row_idx, int32_t M, const void* w,
                    int32_t N, int32_t K, float* out, float* scratch, void* hip_stream) {
  if ((dtype != DLLMC_F32 && dtype != DLLMC_BF16) || !a || !w || !out || !scratch || M < 1 ||
      N < 1 || K < 1)
    return DLLMC_EINVAL;
  (void)hipGetLastError();
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int S = launch_gemm(dtype, a, K, row_idx, M, w, nullptr, N, N, K, scratch,
                            static_cast<size_t>(M) * N * 8, st);
  if (S == 0) return DLLMC_ENOMEM;
  launch_reduce_slices(scratch, S, M, N, out, st);
  HIP_TRY(hipGetLastError());
  return DLLMC_OK;
}

// ---- gathered linear map for callers that cannot allocate ---------------------------------
// The float32 slices of the split contraction live in a file-scope device array instead of a
// caller-provided buffer.  In host code the array's name is only a stand-in: its device address
// is looked up once per device (with that device current) and kept.
}  // extern "C"

constexpr size_t kStaticScratchFloats = static_cast<size_t>(8) << 20;  // 32 MiB per GPU
static __device__ __align__(256) float scratch[kStaticScratchFloats];

namespace {
constexpr int kMaxDevices = 64;
float* g_static_scratch_ptr[kMaxDevices] = {};
std::mutex g_static_scratch_mu;

// device address of `scratch` on the current device (nullptr + HIP error on failure)
hipError_t static_scratch_on_current_device(float** out) {
  *out = nullptr;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_static_scratch_mu);
  if (!g_static_scratch_ptr[dev]) {
    float* p = nullptr;
    e = hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_static_scratch_ptr[dev] = p;
  }
  *out = g_static_scratch_ptr[dev];
  return hipSuccess;
}
}  // namespace

extern "C" {

size_t dllmc_op_linear_static_max_elements(void) { return kStaticScratchFloats; }

int dllmc_op_linear_static(int32_t dtype, const void* a, const int32_t* row_idx, int32_t M,
                           const void* w, int32_t N, int32_t K, float* out, void* hip_stream) {
  if ((dtype != DLLMC_F32 && dtype != DLLMC_BF16) || !a || !w || !out || M < 1 || N < 1 || K < 1)
    return DLLMC_EINVAL;
  if (static_cast<size_t>(M) * N > kStaticScratchFloats) return DLLMC_ETOOBIG;
  (void)hipGetLastError();
  float* ptr = nullptr;
  HIP_TRY(static_scratch_on_current_device(&ptr));
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  // every slice the launch produces is written whole before it is read: nothing to clear
  const int S = launch_gemm(dtype, a, K, row_idx, M, w, nullptr, N, N, K, ptr,
                            kStaticScratchFloats, st);
  if (S == 0) return DLLMC_ETOOBIG;
  launch_reduce_slices(ptr, S, M, N, out, st);
  HIP_TRY(hipGetLastError());
  return DLLMC_OK;
}

size_t dllmc_op_attention_scratch_bytes(void) { return attention_scratch_floats() * sizeof(float); }

int dllmc_op_attention(int32_t dtype, const void* q, int32_t B, int32_t Mq, const void* k_cache,
                       const void* v_cache, int32_t n, int32_t H_q, int32_t H_kv, int32_t d_h,
                       void* out, float* scratch, void* hip_stream) {
  if ((dtype != DLLMC_F32 && dtype != DLLMC_BF16) || !q || !k_cache || !v_cache || !out || B < 1 ||
      Mq < 1 || n < 1 || H_q < 1 || H_kv < 1 || H_q % H_kv || d_h < 1 ||
      !attention_supported(dtype, d_h, n))
    return DLLMC_EINVAL;
  (void)hipGetLastError();
  launch_attention(dtype, q, B, Mq, k_cache, v_cache, n, H_q, H_kv, d_h, out, scratch,
                   static_cast<hipStream_t>(hip_stream));
  HIP_TRY(hipGetLastError());
  return DLLMC_OK;
}

}  // extern "C"

// ---- closed denoising loop ----------------------------------------------------------------

namespace {
struct GenLayout {
  size_t off_hin, off_hout, off_z, off_logits, off_elig, off_negconf, off_x0, off_rows, off_chosen,
      total;
  size_t logits_floats;
};

bool gen_cfg_ok(const dllmc_ctx* c, const dllmc_gen_config* g) {
  if (!c || !g || g->vocab < 1 || g->steps < 1 || g->block_len < 0) return false;
  const int bl = g->block_len ? g->block_len : c->L_r;
  if (bl > c->L_r || c->L_r % bl || g->steps % (c->L_r / bl)) return false;
  return true;
}

GenLayout make_gen_layout(const dllmc_ctx* c, const dllmc_gen_config* g) {
  GenLayout L{};
  const size_t esz = c->lay.esz, B = c->m.batch, n = c->n, d = c->m.d_model, L_r = c->L_r;
  const size_t bl = g->block_len ? g->block_len : c->L_r;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o += align_up(bytes, 256); return r; };
  L.off_hin = take(B * n * d * esz);
  L.off_hout = take(B * n * d * esz);
  L.off_z = take(B * bl * d * esz);
  L.logits_floats = B * bl * static_cast<size_t>(g->vocab);  // at most a block is masked per sequence
  L.off_logits = take(L.logits_floats * sizeof(float));
  L.off_elig = take(B * L_r * sizeof(float));
  L.off_negconf = take(B * L_r * sizeof(float));
  L.off_x0 = take(B * L_r * sizeof(int));
  L.off_rows = take(B * L_r * sizeof(int));
  L.off_chosen = take(B * L_r * sizeof(int));
  L.total = o;
  return L;
}

// positions a step reveals: the block's positions spread evenly over its steps, the remainder
// to the first steps
int reveal_count(int block_len, int steps_per_block, int t) {
  return block_len / steps_per_block + (t < block_len % steps_per_block ? 1 : 0);
}
}  // namespace

struct dllmc_gen {
  dllmc_ctx* c;
  dllmc_gen_config g;
  GenLayout lay;
  char* ws;
  int block_len, steps_per_block;
  int last_n_revealed;
};

extern "C" {

size_t dllmc_gen_workspace_bytes(const dllmc_ctx* ctx, const dllmc_gen_config* cfg) {
  if (!gen_cfg_ok(ctx, cfg)) return 0;
  return make_gen_layout(ctx, cfg).total;
}

int dllmc_gen_create(dllmc_gen** out, dllmc_ctx* ctx, const dllmc_gen_config* cfg, void* workspace,
                     size_t workspace_bytes) {
  if (!out) return DLLMC_EINVAL;
  *out = nullptr;
  if (!gen_cfg_ok(ctx, cfg) || !workspace || !cfg->embed || !cfg->final_norm_g || !cfg->lm_head)
    return DLLMC_EINVAL;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) ||
      (reinterpret_cast<uintptr_t>(cfg->embed) & 15u) ||
      (reinterpret_cast<uintptr_t>(cfg->lm_head) & 15u))
    return DLLMC_EINVAL;
  const GenLayout lay = make_gen_layout(ctx, cfg);
  if (workspace_bytes < lay.total) return DLLMC_ENOMEM;
  dllmc_gen* g = new (std::nothrow) dllmc_gen();
  if (!g) return DLLMC_ENOMEM;
  g->c = ctx;
  g->g = *cfg;
  g->lay = lay;
  g->ws = static_cast<char*>(workspace);
  g->block_len = cfg->block_len ? cfg->block_len : ctx->L_r;
  g->steps_per_block = cfg->steps / (ctx->L_r / g->block_len);
  g->last_n_revealed = 0;
  *out = g;
  return DLLMC_OK;
}

int dllmc_gen_step(dllmc_gen* g, int32_t* tokens, int32_t step_idx, int32_t* sel_idx,
                   int32_t* n_sel, int32_t* n_revealed) {
  if (!g || !tokens || step_idx < 0 || step_idx >= g->g.steps) return DLLMC_EINVAL;
  dllmc_ctx* c = g->c;
  const TuningScope tuning(&c->tune);
  const int B = c->m.batch, n = c->n, L_p = c->L_p, L_r = c->L_r, d = c->m.d_model, dt = c->m.dtype;
  hipStream_t st = c->st;
  void* hin = g->ws + g->lay.off_hin;
  void* hout = g->ws + g->lay.off_hout;

  // the step's block and how many of its positions are still masked / get revealed
  const int blk = step_idx / g->steps_per_block, t = step_idx % g->steps_per_block;
  const int lo = blk * g->block_len, hi = lo + g->block_len;
  int masked = g->block_len;
  for (int u = 0; u < t; ++u) masked -= reveal_count(g->block_len, g->steps_per_block, u);
  const int n_rev = reveal_count(g->block_len, g->steps_per_block, t);
  if (n_revealed) *n_revealed = n_rev;
  g->last_n_revealed = n_rev;

  (void)hipGetLastError();
  launch_embed_gather(dt, g->g.embed, g->g.vocab + 1, tokens, B * n, d, hin, st);
  const int rc = dllmc_step(c, hin, step_idx, hout, sel_idx, n_sel);
  if (rc != DLLMC_OK) return rc;

  float* elig = reinterpret_cast<float*>(g->ws + g->lay.off_elig);
  float* negc = reinterpret_cast<float*>(g->ws + g->lay.off_negconf);
  int* x0 = reinterpret_cast<int*>(g->ws + g->lay.off_x0);
  int* rows = reinterpret_cast<int*>(g->ws + g->lay.off_rows);
  int* chosen = reinterpret_cast<int*>(g->ws + g->lay.off_chosen);
  const double esz = static_cast<double>(c->lay.esz);
  {
    Timed tm(c, DLLMC_KC_GEN_OTHER, B * L_r * 16.0, 0);
    launch_elig_scores(tokens, B, n, L_p, lo, hi, g->g.vocab, elig, negc, x0, st);
  }
  if (n_rev > 0) {
    const int M = B * masked;
    const double V = g->g.vocab;
    void* z = g->ws + g->lay.off_z;
    float* logits = reinterpret_cast<float*>(g->ws + g->lay.off_logits);
    {
      // the masked positions of the block, ascending: bottom-`masked` of a 0/1 score
      Timed tm(c, DLLMC_KC_GEN_OTHER, B * L_r * 4.0 + M * (4.0 + 2.0 * d * esz), 0);
      launch_select(elig, B, L_r, masked, nullptr, 0, rows, masked, 0, nullptr, n, L_p, st);
      launch_final_norm(dt, hout, rows, M, d, c->m.rms_eps, g->g.final_norm_g, z, st);
    }
    {
      // capacity of exactly one slice: the whole contraction in one pass, logits complete
      Timed tm(c, DLLMC_KC_HEAD_GEMM, (V * d + static_cast<double>(M) * d) * esz + M * V * 4.0,
               2.0 * M * V * d);
      const int S = launch_gemm(dt, z, d, nullptr, M, g->g.lm_head, nullptr, g->g.vocab, g->g.vocab,
                                d, logits, static_cast<size_t>(M) * g->g.vocab, st);
      if (S != 1) return DLLMC_ENOMEM;
    }
    {
      Timed tm(c, DLLMC_KC_GEN_OTHER, M * V * 4.0 + B * L_r * 8.0, 0);
      launch_head_finalize(logits, M, g->g.vocab, rows, n, L_p, -1.0f, x0, negc, st);
      // the n_rev most confident (lowest negated confidence, ties to the lower position)
      launch_select(negc, B, L_r, n_rev, chosen, L_r, nullptr, 0, 0, nullptr, n, L_p, st);
      launch_apply_tokens(tokens, B, n, L_p, chosen, L_r, n_rev, x0, st);
    }
  }
  HIP_TRY(hipGetLastError());
  return DLLMC_OK;
}

int dllmc_gen_read(dllmc_gen* g, int32_t* x0, float* conf, int32_t* chosen, void* hidden_out) {
  if (!g) return DLLMC_EINVAL;
  dllmc_ctx* c = g->c;
  const size_t BL = static_cast<size_t>(c->m.batch) * c->L_r;
  hipStream_t st = c->st;
  if (x0)
    HIP_TRY(hipMemcpyAsync(x0, g->ws + g->lay.off_x0, BL * sizeof(int), hipMemcpyDeviceToDevice, st));
  if (conf) {
    // stored negated (selection key); the sign flips in place on the copy
    HIP_TRY(hipMemcpyAsync(conf, g->ws + g->lay.off_negconf, BL * sizeof(float),
                           hipMemcpyDeviceToDevice, st));
    launch_negate_f32(conf, BL, st);
  }
  if (chosen)
    HIP_TRY(hipMemcpyAsync(chosen, g->ws + g->lay.off_chosen, BL * sizeof(int),
                           hipMemcpyDeviceToDevice, st));
  if (hidden_out)
    HIP_TRY(hipMemcpyAsync(hidden_out, g->ws + g->lay.off_hout,
                           static_cast<size_t>(c->m.batch) * c->n * c->m.d_model * c->lay.esz,
                           hipMemcpyDeviceToDevice, st));
  HIP_TRY(hipGetLastError());
  return DLLMC_OK;
}

int dllmc_gen_destroy(dllmc_gen* g) {
  if (!g) return DLLMC_EINVAL;
  delete g;
  return DLLMC_OK;
}

size_t dllmc_op_head_scratch_bytes(int32_t dtype, int32_t M, int32_t vocab, int32_t d) {
  if ((dtype != DLLMC_F32 && dtype != DLLMC_BF16) || M < 1 || vocab < 1 || d < 1) return 0;
  const size_t esz = dtype == DLLMC_BF16 ? 2 : 4;
  return align_up(static_cast<size_t>(M) * d * esz, 256) +
         align_up(static_cast<size_t>(M) * vocab * sizeof(float), 256);
}

int dllmc_op_head(int32_t dtype, const void* hidden, const int32_t* rows, int32_t M,
                  const void* final_norm_g, float eps, const void* lm_head, int32_t vocab, int32_t d,
                  void* scratch, int32_t* x0, float* conf, void* hip_stream) {
  if ((dtype != DLLMC_F32 && dtype != DLLMC_BF16) || !hidden || !final_norm_g || !lm_head ||
      !scratch || !x0 || !conf || M < 1 || vocab < 1 || d < 1 ||
      (reinterpret_cast<uintptr_t>(scratch) & 255u))
    return DLLMC_EINVAL;
  (void)hipGetLastError();
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const size_t esz = dtype == DLLMC_BF16 ? 2 : 4;
  void* z = scratch;
  float* logits = reinterpret_cast<float*>(static_cast<char*>(scratch) +
                                           align_up(static_cast<size_t>(M) * d * esz, 256));
  launch_final_norm(dtype, hidden, rows, M, d, eps, final_norm_g, z, st);
  const int S = launch_gemm(dtype, z, d, nullptr, M, lm_head, nullptr, vocab, vocab, d, logits,
                            static_cast<size_t>(M) * vocab, st);
  if (S != 1) return DLLMC_ENOMEM;
  launch_head_finalize(logits, M, vocab, nullptr, 0, 0, 1.0f, x0, conf, st);
  HIP_TRY(hipGetLastError());
  return DLLMC_OK;
}

int dllmc_probe_copy(const void* src, void* dst, size_t bytes, void* hip_stream) {
  if (!src || !dst || bytes < 16 || (bytes & 15u) || (reinterpret_cast<uintptr_t>(src) & 15u) ||
      (reinterpret_cast<uintptr_t>(dst) & 15u))
    return DLLMC_EINVAL;
  (void)hipGetLastError();
  launch_probe_copy(src, dst, bytes, static_cast<hipStream_t>(hip_stream));
  HIP_TRY(hipGetLastError());
  return DLLMC_OK;
}

int dllmc_probe_read(const void* src, size_t bytes, void* sink, void* hip_stream) {
  if (!src || !sink || bytes < 16 || (bytes & 15u) || (reinterpret_cast<uintptr_t>(src) & 15u) ||
      (reinterpret_cast<uintptr_t>(sink) & 3u))
    return DLLMC_EINVAL;
  (void)hipGetLastError();
  launch_probe_read(src, bytes, static_cast<uint32_t*>(sink), static_cast<hipStream_t>(hip_stream));
  HIP_TRY(hipGetLastError());
  return DLLMC_OK;
}

int dllmc_probe_mfma(int32_t iters, int32_t shape, float* sink, double* flops_out, void* hip_stream) {
  if (iters < 1 || iters > (1 << 24) || shape < 0 || shape > 1 || !sink ||
      (reinterpret_cast<uintptr_t>(sink) & 15u))
    return DLLMC_EINVAL;
  (void)hipGetLastError();
  const double f = launch_probe_mfma(iters, shape, sink, static_cast<hipStream_t>(hip_stream));
  if (flops_out) *flops_out = f;
  HIP_TRY(hipGetLastError());
  return DLLMC_OK;
}

}  // extern "C"
