// Host side of the C ABI: argument validation, workspace carving, stage sequencing.
// Nothing here touches device memory; every entry point only enqueues kernels.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>
#include <mutex>
#include <vector>
#include "common.hpp"

namespace obf {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

obf_status_t check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error("%s: %s", what, hipGetErrorString(e));
    return OBF_ERR_HIP;
  }
  return OBF_OK;
}

// ---- the library's own streams -------------------------------------------------------------------
struct StreamPool { hipStream_t s[kAuxStreams]; hipEvent_t ev[EV_COUNT]; int dev; bool ok; };
static thread_local bool g_single_stream = false;
void set_single_stream(bool on) { g_single_stream = on; }

static StreamPool* stream_pool() {
  static thread_local StreamPool pools[16];
  static thread_local int npools = 0;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return nullptr;
  for (int i = 0; i < npools; ++i) if (pools[i].dev == dev) return pools[i].ok ? &pools[i] : nullptr;
  if (npools == 16) return nullptr;
  StreamPool& p = pools[npools++];
  p.dev = dev;
  p.ok = true;
  for (int i = 0; i < kAuxStreams && p.ok; ++i) p.ok = hipStreamCreateWithFlags(&p.s[i], hipStreamNonBlocking) == hipSuccess;
  for (int i = 0; i < EV_COUNT && p.ok; ++i) p.ok = hipEventCreateWithFlags(&p.ev[i], hipEventDisableTiming) == hipSuccess;
  if (!p.ok) (void)hipGetLastError();                             // no second stream on this device: not an error of the call
  return p.ok ? &p : nullptr;
}

hipStream_t aux_stream(int which) {
  if (g_single_stream || which < 0 || which >= kAuxStreams) return nullptr;
  StreamPool* p = stream_pool();
  return p ? p->s[which] : nullptr;
}

obf_status_t stream_after(hipStream_t waiter, hipStream_t signaller, int slot) {
  StreamPool* p = (slot >= 0 && slot < EV_COUNT) ? stream_pool() : nullptr;
  if (!p || hipEventRecord(p->ev[slot], signaller) != hipSuccess || hipStreamWaitEvent(waiter, p->ev[slot], 0) != hipSuccess) {
    set_error("ordering two streams with an event failed");
    return OBF_ERR_HIP;
  }
  return OBF_OK;
}

// ---- stage profiling ---------------------------------------------------------------------------
struct ProfRec { hipEvent_t a, b; };
static thread_local int g_prof_stage = -1;
static thread_local std::vector<ProfRec>* g_prof_used = nullptr;
static thread_local std::vector<ProfRec>* g_prof_free = nullptr;

ProfScope::ProfScope(int stage, hipStream_t s) : rec(nullptr), st(s) {
  if (stage != g_prof_stage || g_prof_stage < 0) return;
  if (!g_prof_used) { g_prof_used = new std::vector<ProfRec>(); g_prof_free = new std::vector<ProfRec>(); }
  ProfRec r;
  if (!g_prof_free->empty()) { r = g_prof_free->back(); g_prof_free->pop_back(); }
  else {
    if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) return;
  }
  g_prof_used->push_back(r);
  rec = &g_prof_used->back();
  (void)hipEventRecord(r.a, st);
}

ProfScope::~ProfScope() {
  if (rec) (void)hipEventRecord(((ProfRec*)rec)->b, st);
}

static const char* kStageNames[ST_COUNT] = {"score_stats", "score_lse", "score_mass", "select", "refine", "gather",
                                            "keep_cert", "keep_basis", "del_stats", "finalize"};

static obf_status_t check_shape(const obf_shape_t* s) {
  if (!s) { set_error("shape is NULL"); return OBF_ERR_INVALID_ARG; }
  if (s->n_layers < 1 || s->n_kv_heads < 1 || s->group < 1 || s->window < 1 || s->n_tokens < 1) {
    set_error("shape: n_layers, n_kv_heads, group, window, n_tokens must all be >= 1");
    return OBF_ERR_INVALID_ARG;
  }
  if (s->dtype != OBF_F32 && s->dtype != OBF_BF16) { set_error("shape: unknown dtype %d", s->dtype); return OBF_ERR_INVALID_ARG; }
  if (s->head_dim != 64 && s->head_dim != 128) { set_error("head_dim %d unsupported (64 or 128)", s->head_dim); return OBF_ERR_UNSUPPORTED; }
  if (s->n_tokens > kMaxTokens) { set_error("n_tokens %d above the supported %d", s->n_tokens, kMaxTokens); return OBF_ERR_UNSUPPORTED; }
  if ((int64_t)s->n_layers * s->n_kv_heads > 65535) { set_error("more than 65535 heads in one call"); return OBF_ERR_UNSUPPORTED; }
  if ((int64_t)s->group * s->window > 4096) { set_error("group*window above 4096"); return OBF_ERR_UNSUPPORTED; }
  return OBF_OK;
}

static obf_status_t check_ws(const Dims& m, const Workspace& w, const void* ws, size_t ws_bytes) {
  (void)m;
  if (!ws) { set_error("workspace is NULL"); return OBF_ERR_INVALID_ARG; }
  if (((uintptr_t)ws & 255) != 0) { set_error("workspace must be 256-byte aligned"); return OBF_ERR_INVALID_ARG; }
  if (ws_bytes < w.total) { set_error("workspace too small: %zu bytes given, %zu needed", ws_bytes, w.total); return OBF_ERR_WORKSPACE_TOO_SMALL; }
  return OBF_OK;
}

static obf_status_t check_budget(const Dims& m, const int32_t* budgets_host, int32_t budget, int32_t max_budget) {
  if (max_budget < 0) { set_error("max_budget < 0"); return OBF_ERR_INVALID_ARG; }
  if (budgets_host) {
    for (int h = 0; h < m.heads; ++h) {
      int32_t b = budgets_host[h];
      if (b < 0) { set_error("budgets_host[%d] = %d < 0", h, b); return OBF_ERR_INVALID_ARG; }
      if ((b < m.N ? b : m.N) > max_budget) { set_error("budgets_host[%d] = %d exceeds max_budget %d", h, b, max_budget); return OBF_ERR_INVALID_ARG; }
    }
  } else {
    if (budget < 0) { set_error("budget < 0"); return OBF_ERR_INVALID_ARG; }
    if ((budget < m.N ? budget : m.N) > max_budget) { set_error("budget %d exceeds max_budget %d", budget, max_budget); return OBF_ERR_INVALID_ARG; }
  }
  return OBF_OK;
}

static obf_status_t run_score(const Dims& m, const Workspace& w, char* ws, const void* K, const void* Q,
                              float* scores, double* row_lse, hipStream_t st) {
  if (mfma_score_supported(m)) return launch_score_mfma(m, w, ws, K, Q, scores, row_lse, st);
  return launch_score_generic(m, w, ws, K, Q, scores, row_lse, st);
}

}  // namespace obf

using namespace obf;

#define OBF_TRY(expr) do { obf_status_t _s = (expr); if (_s != OBF_OK) return _s; } while (0)
#define OBF_NONNULL(p) do { if (!(p)) { set_error(#p " is NULL"); return OBF_ERR_INVALID_ARG; } } while (0)

extern "C" {

const char* obf_last_error(void) { return g_err; }

obf_status_t obf_profile_enable(int32_t stage) {
  if (stage >= ST_COUNT) { set_error("profile stage %d out of range", stage); return OBF_ERR_INVALID_ARG; }
  g_prof_stage = stage < 0 ? -1 : stage;
  return OBF_OK;
}

obf_status_t obf_profile_read(double* total_ms, int32_t* launches) {
  double ms = 0.0;
  int32_t n = 0;
  if (g_prof_used) {
    for (ProfRec& r : *g_prof_used) {
      float t = 0.f;
      if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&t, r.a, r.b) != hipSuccess) {
        set_error("profile: event read failed");
        return OBF_ERR_HIP;
      }
      ms += t; ++n;
      g_prof_free->push_back(r);
    }
    g_prof_used->clear();
  }
  if (total_ms) *total_ms = ms;
  if (launches) *launches = n;
  return OBF_OK;
}

int32_t obf_profile_stage_count(void) { return ST_COUNT; }
const char* obf_profile_stage_name(int32_t stage) { return (stage >= 0 && stage < ST_COUNT) ? kStageNames[stage] : ""; }
const char* obf_version(void) { return "obf_relay 0.1 (gfx950)"; }

size_t obf_workspace_bytes(const obf_shape_t* shape, int32_t max_budget, int32_t rank) {
  if (check_shape(shape) != OBF_OK || max_budget < 0 || rank < 0) return 0;
  Dims m = make_dims(shape);
  return carve(m, max_budget, rank).total;
}

obf_status_t obf_score(const obf_shape_t* shape, const void* K, const void* Qwin, float* scores,
                       double* row_lse, void* ws, size_t ws_bytes, void* stream) {
  OBF_TRY(check_shape(shape));
  OBF_NONNULL(K); OBF_NONNULL(Qwin); OBF_NONNULL(scores);
  Dims m = make_dims(shape);
  Workspace w = carve(m, 0, 0);
  OBF_TRY(check_ws(m, w, ws, ws_bytes));
  if (!row_lse) row_lse = (double*)((char*)ws + w.row_lse);
  return run_score(m, w, (char*)ws, K, Qwin, scores, row_lse, (hipStream_t)stream);
}

obf_status_t obf_select_topk(const obf_shape_t* shape, const float* scores, const int32_t* budgets_host,
                             int32_t budget, int32_t max_budget, int32_t* idx, int32_t* n_keep,
                             void* ws, size_t ws_bytes, void* stream) {
  (void)ws; (void)ws_bytes;
  OBF_TRY(check_shape(shape));
  OBF_NONNULL(scores); OBF_NONNULL(idx); OBF_NONNULL(n_keep);
  Dims m = make_dims(shape);
  OBF_TRY(check_budget(m, budgets_host, budget, max_budget));
  return launch_select(m, scores, budgets_host, budget, max_budget, idx, n_keep, (hipStream_t)stream);
}

obf_status_t obf_refine_boundary(const obf_shape_t* shape, const void* K, const void* Qwin, const float* scores,
                                 const double* row_lse, int32_t max_budget, int32_t* idx, const int32_t* n_keep,
                                 void* ws, size_t ws_bytes, void* stream) {
  OBF_TRY(check_shape(shape));
  OBF_NONNULL(K); OBF_NONNULL(Qwin); OBF_NONNULL(scores); OBF_NONNULL(row_lse); OBF_NONNULL(idx); OBF_NONNULL(n_keep);
  if (max_budget < 0) { set_error("max_budget < 0"); return OBF_ERR_INVALID_ARG; }
  Dims m = make_dims(shape);
  Workspace w = carve(m, max_budget, 0);
  OBF_TRY(check_ws(m, w, ws, ws_bytes));
  return launch_refine(m, w, (char*)ws, K, Qwin, scores, row_lse, max_budget, idx, n_keep, (hipStream_t)stream);
}

obf_status_t obf_gather(const obf_shape_t* shape, const void* K, const void* V, const int32_t* idx,
                        const int32_t* n_keep, int32_t max_budget, void* K_out, void* V_out, void* stream) {
  OBF_TRY(check_shape(shape));
  OBF_NONNULL(idx); OBF_NONNULL(n_keep);
  if (max_budget < 0) { set_error("max_budget < 0"); return OBF_ERR_INVALID_ARG; }
  if (K_out && !K) { set_error("K_out given but K is NULL"); return OBF_ERR_INVALID_ARG; }
  if (V_out && !V) { set_error("V_out given but V is NULL"); return OBF_ERR_INVALID_ARG; }
  Dims m = make_dims(shape);
  return launch_gather(m, K, V, idx, n_keep, max_budget, K_out, V_out, (hipStream_t)stream);
}

obf_status_t obf_backfill(const obf_shape_t* shape, const void* V, const float* scores, const int32_t* idx,
                          const int32_t* n_keep, int32_t max_budget, int32_t rank, void* V_out,
                          float* delta_out, obf_diag_t* diag, void* ws, size_t ws_bytes, void* stream) {
  OBF_TRY(check_shape(shape));
  OBF_NONNULL(V); OBF_NONNULL(scores); OBF_NONNULL(idx); OBF_NONNULL(n_keep); OBF_NONNULL(V_out);
  if (max_budget < 0) { set_error("max_budget < 0"); return OBF_ERR_INVALID_ARG; }
  if (rank < 0) { set_error("rank < 0"); return OBF_ERR_INVALID_ARG; }
  Dims m = make_dims(shape);
  Workspace w = carve(m, max_budget, rank);
  OBF_TRY(check_ws(m, w, ws, ws_bytes));
  return launch_backfill(m, w, (char*)ws, V, scores, idx, n_keep, max_budget, rank, V_out, delta_out, diag,
                         (hipStream_t)stream, aux_stream(0));
}

// obf_variant_t (nullable) checked and packed for the kernels.
static obf_status_t make_variant(const obf_variant_t* v, Variant* out) {
  *out = Variant();
  if (!v) return OBF_OK;
  if (v->subspace != OBF_SUBSPACE_RANK && v->subspace != OBF_SUBSPACE_ALL && v->subspace != OBF_SUBSPACE_EVR) {
    set_error("variant: unknown subspace rule");
    return OBF_ERR_INVALID_ARG;
  }
  if (v->subspace == OBF_SUBSPACE_EVR && !(v->evr_tau > 0.f && v->evr_tau <= 1.f)) {
    set_error("variant: evr_tau must lie in (0, 1]");
    return OBF_ERR_INVALID_ARG;
  }
  if (v->subspace_iters < 0 || v->subspace_iters > 64) {
    set_error("variant: subspace_iters must lie in [0, 64]");
    return OBF_ERR_INVALID_ARG;
  }
  out->subspace_iters = v->subspace_iters;
  if (v->no_projection) out->flags |= VF_NO_PROJECTION;
  if (v->subspace == OBF_SUBSPACE_ALL) out->flags |= VF_SUBSPACE_ALL;
  if (v->subspace == OBF_SUBSPACE_EVR) { out->flags |= VF_SUBSPACE_EVR; out->evr_tau = v->evr_tau; }
  if (v->no_scaling) out->flags |= VF_NO_SCALING;
  if (v->naive_aggregation) out->flags |= VF_NAIVE;
  if (v->attn_inject) out->flags |= VF_ATTN_INJECT;
  if (v->per_token) out->flags |= VF_PER_TOKEN;
  return OBF_OK;
}

// The heads of one call: scores on `score_st`, everything after them on `st` (which waits for the scores when it is
// another stream), side work of that part on `aux` (nullable).
static obf_status_t compress_heads(int layerwise, Variant var, const Dims& mf, int sink,
                                   const void* K, const void* V, const void* Qwin,
                                   const int32_t* budgets_host, int32_t budget, int32_t max_budget, int32_t rank,
                                   void* K_out, void* V_out, int32_t* idx, int32_t* n_keep,
                                   float* scores_out, float* delta_out, obf_diag_t* diag,
                                   char* base, hipStream_t score_st, hipStream_t st, hipStream_t aux) {
  // the eligible tokens (Sec. 4.3.2): a view behind the sink, same strides; selection, gather and back-fill run on it
  Dims m = mf;
  m.N = mf.N - sink;
  m.scs = mf.N;
  Dims mb = m;                                          // the units that own a budget: heads, or layers
  if (layerwise) mb.heads = m.L;
  Workspace w = carve(mf, max_budget, rank);
  float* scores = scores_out ? scores_out : (float*)(base + w.scores);
  double* row_lse = (double*)(base + w.row_lse);
  OBF_TRY(run_score(mf, w, base, K, Qwin, scores, row_lse, score_st));
  if (st != score_st) OBF_TRY(stream_after(st, score_st, EV_SCORED));
  w.nstat = (m.N + kStatChunk - 1) / kStatChunk;        // statistics chunks of the view
  K = (const char*)K + (size_t)sink * m.d * m.esize;
  V = (const char*)V + (size_t)sink * m.d * m.esize;
  scores += sink;
  if (layerwise) {
    OBF_TRY(launch_select_layerwise(m, w, base, scores, budgets_host, budget, max_budget, idx, n_keep, K, Qwin, row_lse, st));
  } else {
    // selection and boundary refinement in one kernel (same decisions as the two stage calls)
    OBF_TRY(launch_select_refine(m, scores, budgets_host, budget, max_budget, idx, n_keep, K, Qwin, row_lse, st,
                                 (int32_t*)(base + w.sel_flags)));
  }
  // the gather also leaves the sums of squares of the retained V rows for the full-rank certificate
  double* fro_part = (m.dtype == OBF_BF16 && m.d == 128) ? (double*)(base + w.fro_part) : nullptr;
  // small budgets: the bases of the retained spans start now on a second stream, beside the gather
  bool basis_started = false;
  if (!var.skips_basis()) {
    const obf_status_t bs = launch_backfill_basis(m, w, base, V, scores, idx, n_keep, max_budget, rank, st, aux, &basis_started);
    if (bs != OBF_OK) {
      if (basis_started) (void)stream_after(st, aux, EV_BASIS_JOIN);      // never leave the second stream un-joined
      return bs;
    }
  }
  // Large budgets: nothing downstream reads K_out, so the retained K rows are copied on the second stream once the
  // V rows (which the certificate waits for) are through, beside the latency-bound per-head kernels.
  bool k_beside = false;
  obf_status_t rs = OBF_OK;
  if (!basis_started && aux && aux != st && (size_t)max_budget * m.heads >= 65536) {
    rs = launch_gather(m, nullptr, V, idx, n_keep, max_budget, nullptr, V_out, st, fro_part);
    if (rs == OBF_OK) rs = stream_after(aux, st, EV_KROWS_FORK);
    if (rs == OBF_OK) { k_beside = true; rs = launch_gather(m, K, nullptr, idx, n_keep, max_budget, K_out, nullptr, aux, nullptr); }
  } else {
    rs = launch_gather(m, K, V, idx, n_keep, max_budget, K_out, V_out, st, fro_part);
  }
  int32_t min_budget = budget;
  if (budgets_host) { min_budget = budgets_host[0]; for (int h = 1; h < mb.heads; ++h) min_budget = budgets_host[h] < min_budget ? budgets_host[h] : min_budget; }
  // (launch_backfill joins the bases' stream itself, on every path; after an earlier error it is only called for that)
  if (rs == OBF_OK || basis_started) {
    const obf_status_t fs = (rs == OBF_OK)
        ? launch_backfill(m, w, base, V, scores, idx, n_keep, max_budget, rank, V_out, delta_out, diag, st, aux, fro_part,
                          basis_started, min_budget, var)
        : stream_after(st, aux, EV_BASIS_JOIN);
    if (rs == OBF_OK) rs = fs;
  }
  if (k_beside) { const obf_status_t js = stream_after(st, aux, EV_KROWS_JOIN); if (rs == OBF_OK) rs = js; }
  OBF_TRY(rs);
  if ((var.flags & VF_PER_TOKEN) && rank > 0)                    // needs the gathered keys: after the join above
    OBF_TRY(launch_per_token_inject(m, w, base, K, V, scores, idx, n_keep, max_budget, K_out, V_out,
                                    (var.flags & VF_NO_SCALING) ? 1 : 0, st));
  if (diag && !layerwise) OBF_TRY(launch_diag_flags(diag, (const int32_t*)(base + w.sel_flags), m.heads, st));
  return launch_idx_offset(idx, (size_t)m.heads * max_budget, sink, st);   // back to the head's own token numbers
}

// Shared body of the fused calls; layerwise != 0 selects the per-layer retention rule.
static obf_status_t compress_relay_impl(int layerwise, Variant var, const obf_window_t* window, const obf_shape_t* shape,
                                        const void* K, const void* V, const void* Qwin,
                                        const int32_t* budgets_host, int32_t budget, int32_t max_budget, int32_t rank,
                                        void* K_out, void* V_out, int32_t* idx, int32_t* n_keep,
                                        float* scores_out, float* delta_out, obf_diag_t* diag,
                                        void* ws, size_t ws_bytes, void* stream,
                                        bool own_side_stream = true /*false: the call forks nothing (its stream is a side stream itself)*/) {
  OBF_TRY(check_shape(shape));
  OBF_NONNULL(K); OBF_NONNULL(V); OBF_NONNULL(Qwin); OBF_NONNULL(K_out); OBF_NONNULL(V_out);
  OBF_NONNULL(idx); OBF_NONNULL(n_keep);
  if (rank < 0) { set_error("rank < 0"); return OBF_ERR_INVALID_ARG; }
  Dims mf = make_dims(shape);                           // all real tokens: the keys of Eq. 1
  int sink = 0;
  if (window) {
    if (window->token_stride != 0 && window->token_stride < mf.N) { set_error("window: token_stride below n_tokens"); return OBF_ERR_INVALID_ARG; }
    if (window->sink < 0 || window->sink >= mf.N) { set_error("window: sink must lie in [0, n_tokens)"); return OBF_ERR_INVALID_ARG; }
    if (window->token_stride) mf.kvs = window->token_stride;
    sink = window->sink;
  }
  Dims mb = mf;
  mb.N = mf.N - sink;
  if (layerwise) mb.heads = mf.L;
  OBF_TRY(check_budget(mb, budgets_host, budget, max_budget));
  Workspace w = carve(mf, max_budget, rank);
  OBF_TRY(check_ws(mf, w, ws, ws_bytes));
  hipStream_t st = (hipStream_t)stream;
  return compress_heads(layerwise, var, mf, sink, K, V, Qwin, budgets_host, budget, max_budget, rank, K_out, V_out, idx, n_keep,
                        scores_out, delta_out, diag, (char*)ws, st, st, own_side_stream ? aux_stream(0) : (hipStream_t)nullptr);
}

obf_status_t obf_compress_relay(const obf_shape_t* shape, const void* K, const void* V, const void* Qwin,
                                const int32_t* budgets_host, int32_t budget, int32_t max_budget, int32_t rank,
                                void* K_out, void* V_out, int32_t* idx, int32_t* n_keep,
                                float* scores_out, float* delta_out, obf_diag_t* diag,
                                void* ws, size_t ws_bytes, void* stream) {
  return compress_relay_impl(0, Variant(), nullptr, shape, K, V, Qwin, budgets_host, budget, max_budget, rank, K_out, V_out, idx, n_keep,
                             scores_out, delta_out, diag, ws, ws_bytes, stream);
}

obf_status_t obf_compress_relay_layerwise(const obf_shape_t* shape, const void* K, const void* V, const void* Qwin,
                                          const int32_t* budgets_host, int32_t budget, int32_t max_budget, int32_t rank,
                                          void* K_out, void* V_out, int32_t* idx, int32_t* n_keep,
                                          float* scores_out, float* delta_out, obf_diag_t* diag,
                                          void* ws, size_t ws_bytes, void* stream) {
  return compress_relay_impl(1, Variant(), nullptr, shape, K, V, Qwin, budgets_host, budget, max_budget, rank, K_out, V_out, idx, n_keep,
                             scores_out, delta_out, diag, ws, ws_bytes, stream);
}

obf_status_t obf_compress_relay_variant(const obf_shape_t* shape, const void* K, const void* V, const void* Qwin,
                                        const int32_t* budgets_host, int32_t budget, int32_t max_budget, int32_t rank,
                                        int32_t layerwise, const obf_variant_t* variant,
                                        void* K_out, void* V_out, int32_t* idx, int32_t* n_keep,
                                        float* scores_out, float* delta_out, obf_diag_t* diag,
                                        void* ws, size_t ws_bytes, void* stream) {
  Variant var;
  OBF_TRY(make_variant(variant, &var));
  return compress_relay_impl(layerwise != 0, var, nullptr, shape, K, V, Qwin, budgets_host, budget, max_budget, rank, K_out, V_out, idx,
                             n_keep, scores_out, delta_out, diag, ws, ws_bytes, stream);
}

obf_status_t obf_backfill_variant(const obf_shape_t* shape, const void* V, const float* scores, const int32_t* idx,
                                  const int32_t* n_keep, int32_t max_budget, int32_t rank,
                                  const obf_variant_t* variant, void* V_out, float* delta_out, obf_diag_t* diag,
                                  void* ws, size_t ws_bytes, void* stream) {
  Variant var;
  OBF_TRY(make_variant(variant, &var));
  if (var.flags & VF_PER_TOKEN) { set_error("the per-token variant routes by the keys: use a fused call"); return OBF_ERR_UNSUPPORTED; }
  OBF_TRY(check_shape(shape));
  OBF_NONNULL(V); OBF_NONNULL(scores); OBF_NONNULL(idx); OBF_NONNULL(n_keep); OBF_NONNULL(V_out);
  if (max_budget < 0) { set_error("max_budget < 0"); return OBF_ERR_INVALID_ARG; }
  if (rank < 0) { set_error("rank < 0"); return OBF_ERR_INVALID_ARG; }
  Dims m = make_dims(shape);
  Workspace w = carve(m, max_budget, rank);
  OBF_TRY(check_ws(m, w, ws, ws_bytes));
  return launch_backfill(m, w, (char*)ws, V, scores, idx, n_keep, max_budget, rank, V_out, delta_out, diag,
                         (hipStream_t)stream, aux_stream(0), nullptr, false, -1, var);
}

obf_status_t obf_compress_relay_window(const obf_shape_t* shape, const obf_window_t* window,
                                       const void* K, const void* V, const void* Qwin,
                                       const int32_t* budgets_host, int32_t budget, int32_t max_budget, int32_t rank,
                                       int32_t layerwise, const obf_variant_t* variant,
                                       void* K_out, void* V_out, int32_t* idx, int32_t* n_keep,
                                       float* scores_out, float* delta_out, obf_diag_t* diag,
                                       void* ws, size_t ws_bytes, void* stream) {
  Variant var;
  OBF_TRY(make_variant(variant, &var));
  return compress_relay_impl(layerwise != 0, var, window, shape, K, V, Qwin, budgets_host, budget, max_budget, rank, K_out, V_out,
                             idx, n_keep, scores_out, delta_out, diag, ws, ws_bytes, stream);
}

// ---- a batch of right-padded samples (App. A.7) ---------------------------------------------------
static size_t batch_align(size_t n) { return (n + 255) & ~(size_t)255; }

static size_t batch_slot_bytes(const obf_shape_t* shape, int32_t token_stride, int32_t max_budget, int32_t rank) {
  // one workspace slot serves every sample that runs on it: the largest any length needs
  obf_shape_t s = *shape;
  size_t need = 0;
  for (int32_t n = 1; n <= token_stride; ++n) {
    s.n_tokens = n;
    const size_t t = carve(make_dims(&s), max_budget, rank).total;
    need = t > need ? t : need;
  }
  return need;
}

size_t obf_workspace_bytes_batch(const obf_shape_t* shape, int32_t n_samples, int32_t token_stride, int32_t max_budget, int32_t rank) {
  if (!shape || n_samples < 1 || token_stride < 1 || token_stride > kMaxTokens || max_budget < 0 || rank < 0) return 0;
  obf_shape_t s = *shape;
  s.n_tokens = token_stride;
  if (check_shape(&s) != OBF_OK) return 0;
  // one slot per sample in flight: the samples take turns on the caller's stream and on the library's own
  const size_t slot = batch_align(batch_slot_bytes(shape, token_stride, max_budget, rank));
  return (size_t)(n_samples < kBatchLanes ? n_samples : kBatchLanes) * slot;
}

obf_status_t obf_compress_relay_batch(const obf_shape_t* shape, int32_t n_samples, const int32_t* n_tokens_host,
                                      int32_t token_stride, int32_t sink,
                                      const void* K, const void* V, const void* Qwin,
                                      const int32_t* budgets_host, int32_t budget, int32_t max_budget, int32_t rank,
                                      void* K_out, void* V_out, int32_t* idx, int32_t* n_keep, obf_diag_t* diag,
                                      void* ws, size_t ws_bytes, void* stream) {
  if (!shape) { set_error("shape is NULL"); return OBF_ERR_INVALID_ARG; }
  OBF_NONNULL(n_tokens_host); OBF_NONNULL(K); OBF_NONNULL(V); OBF_NONNULL(Qwin); OBF_NONNULL(K_out); OBF_NONNULL(V_out);
  OBF_NONNULL(idx); OBF_NONNULL(n_keep);
  if (n_samples < 1) { set_error("n_samples < 1"); return OBF_ERR_INVALID_ARG; }
  if (token_stride < 1 || token_stride > kMaxTokens) { set_error("token_stride outside [1, %d]", kMaxTokens); return OBF_ERR_INVALID_ARG; }
  if (max_budget < 0 || rank < 0 || sink < 0) { set_error("max_budget, rank and sink must not be negative"); return OBF_ERR_INVALID_ARG; }
  // everything the host can check, for every sample, before the first kernel is enqueued
  size_t need = 0;
  for (int32_t i = 0; i < n_samples; ++i) {
    obf_shape_t s = *shape;
    s.n_tokens = n_tokens_host[i];
    if (s.n_tokens < 1 || s.n_tokens > token_stride) { set_error("n_tokens_host[%d] = %d outside [1, token_stride]", i, s.n_tokens); return OBF_ERR_INVALID_ARG; }
    if (sink >= s.n_tokens) { set_error("sink %d leaves sample %d (%d tokens) without eligible tokens", sink, i, s.n_tokens); return OBF_ERR_INVALID_ARG; }
    OBF_TRY(check_shape(&s));
    Dims m = make_dims(&s);
    const int32_t b = budgets_host ? budgets_host[i] : budget;
    if (b < 0) { set_error("budget of sample %d is negative", i); return OBF_ERR_INVALID_ARG; }
    const int32_t eligible = m.N - sink;
    if ((b < eligible ? b : eligible) > max_budget) { set_error("budget of sample %d exceeds max_budget %d", i, max_budget); return OBF_ERR_INVALID_ARG; }
    const size_t t = carve(m, max_budget, rank).total;
    need = t > need ? t : need;
  }
  if (!ws) { set_error("workspace is NULL"); return OBF_ERR_INVALID_ARG; }
  if (ws_bytes < need) { set_error("workspace too small: %zu bytes given, %zu needed", ws_bytes, need); return OBF_ERR_WORKSPACE_TOO_SMALL; }
  Dims m0 = make_dims(shape);
  const size_t heads = (size_t)m0.heads, row = (size_t)m0.d * m0.esize;
  const obf_window_t win = {token_stride, sink};
  // Samples share nothing, and a short sample's per-head kernels leave most of the chip idle: with room for several
  // workspace slots, sample i runs in lane i mod lanes; lane 0 is the caller's stream (with the library's first stream for
  // the forks inside a sample), every further lane one of the library's other streams, forked off the caller's before the
  // first sample and joined back after the last, on every way out.  Not under stream capture (the captured graph stays a
  // chain per sample) and not while stage timing is on.
  hipStream_t st = (hipStream_t)stream, lane_st[kBatchLanes] = {st};
  const size_t slot = batch_align(need);
  int lanes = 1;
  if (n_samples >= 2 && ws_bytes >= 2 * slot && g_prof_stage < 0) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cs) == hipSuccess && cs == hipStreamCaptureStatusNone) {
      const size_t fit = ws_bytes / slot;
      const int want = (int)(fit < (size_t)kBatchLanes ? fit : (size_t)kBatchLanes);
      while (lanes < want && lanes < n_samples) {
        hipStream_t s2 = aux_stream(lanes);
        if (!s2 || stream_after(s2, st, EV_BATCH_FORK) != OBF_OK) break;
        lane_st[lanes++] = s2;
      }
    } else (void)hipGetLastError();
  }
  obf_status_t rs = OBF_OK;
  for (int32_t i = 0; i < n_samples && rs == OBF_OK; ++i) {
    obf_shape_t s = *shape;
    s.n_tokens = n_tokens_host[i];
    const size_t kv_off = (size_t)i * heads * token_stride * row, q_off = (size_t)i * heads * m0.R * row;
    const size_t out_rows = (size_t)i * heads * max_budget;
    const int lane = lanes > 1 ? i % lanes : 0;
    rs = compress_relay_impl(0, Variant(), &win, &s, (const char*)K + kv_off, (const char*)V + kv_off, (const char*)Qwin + q_off,
                             nullptr, budgets_host ? budgets_host[i] : budget, max_budget, rank,
                             (char*)K_out + out_rows * row, (char*)V_out + out_rows * row, idx + out_rows, n_keep + (size_t)i * heads,
                             nullptr, nullptr, diag ? diag + (size_t)i * heads : nullptr,
                             (char*)ws + (size_t)lane * slot, lanes > 1 ? slot : ws_bytes, (void*)lane_st[lane], lane == 0);
  }
  for (int l = 1; l < lanes; ++l) { const obf_status_t js = stream_after(st, lane_st[l], EV_BATCH_JOIN); if (rs == OBF_OK) rs = js; }
  return rs;
}

obf_status_t obf_cache_merge(const obf_shape_t* shape, const void* K, const void* V, const float* scores, const int32_t* idx,
                             const int32_t* n_keep, int32_t max_budget, const void* K_out, void* V_out, int32_t* route_out,
                             void* ws, size_t ws_bytes, void* stream) {
  OBF_TRY(check_shape(shape));
  OBF_NONNULL(K); OBF_NONNULL(V); OBF_NONNULL(scores); OBF_NONNULL(idx); OBF_NONNULL(n_keep); OBF_NONNULL(K_out); OBF_NONNULL(V_out);
  if (max_budget < 0) { set_error("max_budget < 0"); return OBF_ERR_INVALID_ARG; }
  Dims m = make_dims(shape);
  Workspace w = carve(m, max_budget, 0);
  OBF_TRY(check_ws(m, w, ws, ws_bytes));
  return launch_cache_merge(m, w, (char*)ws, K, V, scores, idx, n_keep, max_budget, K_out, V_out, route_out, (hipStream_t)stream);
}

obf_status_t obf_compress_relay_merge(const obf_shape_t* shape, const void* K, const void* V, const void* Qwin,
                                      const int32_t* budgets_host, int32_t budget, int32_t max_budget,
                                      void* K_out, void* V_out, int32_t* idx, int32_t* n_keep,
                                      float* scores_out, int32_t* route_out, void* ws, size_t ws_bytes, void* stream) {
  OBF_TRY(check_shape(shape));
  OBF_NONNULL(K); OBF_NONNULL(V); OBF_NONNULL(Qwin); OBF_NONNULL(K_out); OBF_NONNULL(V_out); OBF_NONNULL(idx); OBF_NONNULL(n_keep);
  Dims m = make_dims(shape);
  OBF_TRY(check_budget(m, budgets_host, budget, max_budget));
  Workspace w = carve(m, max_budget, 0);
  OBF_TRY(check_ws(m, w, ws, ws_bytes));
  char* base = (char*)ws;
  hipStream_t st = (hipStream_t)stream;
  float* scores = scores_out ? scores_out : (float*)(base + w.scores);
  double* row_lse = (double*)(base + w.row_lse);
  OBF_TRY(run_score(m, w, base, K, Qwin, scores, row_lse, st));                                   // (i) the same selector
  OBF_TRY(launch_select_refine(m, scores, budgets_host, budget, max_budget, idx, n_keep, K, Qwin, row_lse, st));
  OBF_TRY(launch_gather(m, K, V, idx, n_keep, max_budget, K_out, V_out, st, nullptr));
  return launch_cache_merge(m, w, base, K, V, scores, idx, n_keep, max_budget, K_out, V_out, route_out, st);   // (ii), (iii)
}

static obf_status_t check_quant(int64_t n_rows, int32_t head_dim, int32_t dtype, int32_t bits) {
  if (n_rows < 0 || n_rows > ((int64_t)1 << 40)) { set_error("n_rows out of range"); return OBF_ERR_INVALID_ARG; }
  if (head_dim != 64 && head_dim != 128) { set_error("head_dim %d unsupported (64 or 128)", head_dim); return OBF_ERR_UNSUPPORTED; }
  if (dtype != OBF_F32 && dtype != OBF_BF16) { set_error("unknown dtype %d", dtype); return OBF_ERR_INVALID_ARG; }
  if (bits != 4 && bits != 8) { set_error("bits must be 4 or 8"); return OBF_ERR_INVALID_ARG; }
  return OBF_OK;
}

obf_status_t obf_quantize_rows(const void* X, int64_t n_rows, int32_t head_dim, int32_t dtype, int32_t bits,
                               uint8_t* codes, uint16_t* scale_f16, uint16_t* zero_f16, void* stream) {
  OBF_TRY(check_quant(n_rows, head_dim, dtype, bits));
  OBF_NONNULL(X); OBF_NONNULL(codes); OBF_NONNULL(scale_f16); OBF_NONNULL(zero_f16);
  return launch_quant_rows(X, (long)n_rows, head_dim, dtype, bits, codes, scale_f16, zero_f16, (hipStream_t)stream);
}

obf_status_t obf_dequantize_rows(const uint8_t* codes, const uint16_t* scale_f16, const uint16_t* zero_f16, int64_t n_rows,
                                 int32_t head_dim, int32_t dtype, int32_t bits, void* X_out, void* stream) {
  OBF_TRY(check_quant(n_rows, head_dim, dtype, bits));
  OBF_NONNULL(X_out); OBF_NONNULL(codes); OBF_NONNULL(scale_f16); OBF_NONNULL(zero_f16);
  return launch_dequant_rows(codes, scale_f16, zero_f16, (long)n_rows, head_dim, dtype, bits, X_out, (hipStream_t)stream);
}

// ---- the entry point that allocates nothing ------------------------------------------------------
// Its workspace is this array in the code object's zero-initialised data: every GPU the library is loaded on holds its
// own copy at its own address for the life of the process.  The name is a host-side handle only; the device address
// comes from hipGetSymbolAddress, once per device.
constexpr size_t kStaticScratchBytes = (size_t)OBF_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static obf_status_t static_scratch_ptr(void** out) {
  static std::mutex mu;
  static void* ptrs[64] = {nullptr};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { set_error("hipGetDevice failed"); return OBF_ERR_HIP; }
  if (dev < 0 || dev >= 64) { set_error("device ordinal %d out of range", dev); return OBF_ERR_UNSUPPORTED; }
  std::lock_guard<std::mutex> lock(mu);
  if (!ptrs[dev]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) { set_error("hipGetSymbolAddress(scratch): %s", hipGetErrorString(e)); return OBF_ERR_HIP; }
    ptrs[dev] = p;
  }
  *out = ptrs[dev];
  return OBF_OK;
}

size_t obf_static_scratch_bytes(void) { return kStaticScratchBytes; }

obf_status_t obf_compress_relay_static(const obf_shape_t* shape, const void* K, const void* V, const void* Qwin,
                                       const int32_t* budgets_host, int32_t budget, int32_t max_budget, int32_t rank,
                                       void* K_out, void* V_out, int32_t* idx, int32_t* n_keep, void* stream) {
  OBF_TRY(check_shape(shape));
  if (max_budget < 0 || rank < 0) { set_error("max_budget and rank must not be negative"); return OBF_ERR_INVALID_ARG; }
  const size_t need = carve(make_dims(shape), max_budget, rank).total;
  if (need > kStaticScratchBytes) {
    set_error("this shape needs %zu bytes of scratch, the built-in array holds %zu: use obf_compress_relay with a workspace",
              need, kStaticScratchBytes);
    return OBF_ERR_UNSUPPORTED;
  }
  if (g_prof_stage >= 0) { set_error("stage profiling creates events: switch it off before this call"); return OBF_ERR_INVALID_ARG; }
  void* ws = nullptr;
  OBF_TRY(static_scratch_ptr(&ws));
  set_single_stream(true);                 // no second stream: creating one allocates
  obf_status_t s = compress_relay_impl(0, Variant(), nullptr, shape, K, V, Qwin, budgets_host, budget, max_budget, rank, K_out,
                                       V_out, idx, n_keep, nullptr, nullptr, nullptr, ws, kStaticScratchBytes, stream);
  set_single_stream(false);
  return s;
}

obf_status_t obf_append_message(int32_t n_heads, int32_t head_dim, int32_t dtype,
                                const void* prev_K, const void* prev_V, const int32_t* prev_len, int32_t prev_len_all,
                                int32_t prev_stride,
                                const void* keep_K, const void* keep_V, const int32_t* n_keep, int32_t keep_stride,
                                const void* gen_K, const void* gen_V, int32_t n_gen, int32_t gen_stride,
                                void* msg_K, void* msg_V, int32_t* msg_len, int32_t msg_stride, void* stream) {
  if (n_heads < 1 || n_heads > 65535) { set_error("n_heads must lie in [1, 65535]"); return OBF_ERR_INVALID_ARG; }
  if (dtype != OBF_F32 && dtype != OBF_BF16) { set_error("unknown dtype %d", dtype); return OBF_ERR_INVALID_ARG; }
  if (head_dim != 64 && head_dim != 128) { set_error("head_dim %d unsupported (64 or 128)", head_dim); return OBF_ERR_UNSUPPORTED; }
  if (prev_stride < 0 || keep_stride < 0 || gen_stride < 0 || msg_stride < 1 || prev_len_all < 0 || n_gen < 0) {
    set_error("strides and lengths must not be negative (msg_stride >= 1)");
    return OBF_ERR_INVALID_ARG;
  }
  OBF_NONNULL(msg_K); OBF_NONNULL(msg_V); OBF_NONNULL(msg_len);
  if ((prev_len || prev_len_all > 0) && (!prev_K || !prev_V)) { set_error("prev rows announced but prev_K / prev_V is NULL"); return OBF_ERR_INVALID_ARG; }
  if (n_keep && (!keep_K || !keep_V)) { set_error("n_keep given but keep_K / keep_V is NULL"); return OBF_ERR_INVALID_ARG; }
  if (n_gen > 0 && (!gen_K || !gen_V)) { set_error("n_gen > 0 but gen_K / gen_V is NULL"); return OBF_ERR_INVALID_ARG; }
  if (n_gen > gen_stride) { set_error("n_gen %d above gen_stride %d", n_gen, gen_stride); return OBF_ERR_INVALID_ARG; }
  if (!prev_len && prev_len_all > prev_stride) { set_error("prev_len_all %d above prev_stride %d", prev_len_all, prev_stride); return OBF_ERR_INVALID_ARG; }
  if (!prev_len && !n_keep && prev_len_all + n_gen > msg_stride) { set_error("message rows exceed msg_stride"); return OBF_ERR_INVALID_ARG; }
  const int esize = (dtype == OBF_BF16) ? 2 : 4;
  return launch_append_message(n_heads, head_dim * esize, prev_K, prev_V, prev_len, prev_len_all, prev_stride, keep_K, keep_V,
                               n_keep, keep_stride, gen_K, gen_V, n_gen, gen_stride, msg_K, msg_V, msg_len, msg_stride,
                               (hipStream_t)stream);
}

}  // extern "C"
