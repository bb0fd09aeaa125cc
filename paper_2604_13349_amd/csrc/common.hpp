// Internal declarations shared by the translation units of libobf_relay.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <mutex>
#include "obf_relay.h"

namespace obf {

constexpr int kMaxTokens = 32768;
constexpr int kNumCU = 256;             // compute units of the target (MI355X)
constexpr int kStatChunk = 1024;        // tokens per deleted-value statistics workgroup
constexpr int kGatherRows = 64;         // rows per gather workgroup when a row is 256 bytes (bf16, head_dim 128)
constexpr int kBandCap = 256;           // most boundary candidates re-scored per head
constexpr double kEps = 1e-12;          // epsilon of Eq. 4 / Eq. 6
constexpr float kBandRel = 1.0e-4f;     // relative half-width of the refinement band

struct Dims {
  int heads;      // n_layers * n_kv_heads
  int L, H, g, d, N, W;
  int kvs;        // tokens between consecutive heads of K and V (>= N; N for a dense cache)
  int scs;        // floats between consecutive heads of the score array handed to selection and back-fill (>= N)
  int R;          // query rows per KV head = g * W
  int dtype;
  int esize;      // bytes per element of K/V/Q
};

inline Dims make_dims(const obf_shape_t* s) {
  Dims m;
  m.L = s->n_layers; m.H = s->n_kv_heads; m.g = s->group; m.d = s->head_dim; m.N = s->n_tokens; m.W = s->window;
  m.kvs = m.N; m.scs = m.N;
  m.heads = m.L * m.H; m.R = m.g * m.W; m.dtype = s->dtype; m.esize = (s->dtype == OBF_BF16) ? 2 : 4;
  return m;
}

// Heads with many retained rows that the full-rank certificate does not settle (rare): the double-precision Gram
// matrix of their rows is summed from kKeepGramChunks partial matrices computed by as many workgroups, for at most
// kKeepGramSlots such heads per call (further ones compute it in their own workgroup); used from kKeepGramMinBudget rows.
constexpr int kJacobiSweeps = 12;       // cap of the cyclic Jacobi iteration of the finalisation
constexpr int kKeepGramChunks = 16;
constexpr int kKeepGramSlots = 8;
constexpr int kKeepGramMinBudget = 2048;

// Query rows per workgroup of the matrix-core score kernels: 128 (four 32-row blocks) or 160 (five), whichever pads the
// g * W rows of a KV head less; ties go to 128, which has one more K buffer in flight.
inline int score_rows_per_group(int R) {
  const int g4 = (R + 127) / 128, g5 = (R + 159) / 160;
  return (g5 * 160 - R < g4 * 128 - R) ? 160 : 128;
}

// Workspace carving.  Every region is 256-byte aligned; offsets are from the workspace base.
struct Workspace {
  size_t stats_part;   // double2 [heads][nchunk][R]      partial (max, sum-exp) per score chunk
  size_t row_lse;      // double  [heads][R]
  size_t scores;       // float   [heads][N]              (fused call without scores_out)
  size_t score_part;   // float   [RG][heads][N]          per-row-group column sums when group*window > 128
  size_t head_state;   // HeadState [heads]
  size_t decided;      // int32   [heads]                 1: the fast full-rank test settled the head
  size_t basis;        // float   [heads][d][d]           orthonormal basis of the retained span (columns)
  size_t gram_part;    // float   [heads][nstat][gram_stride(d)] partial Gram / weighted sum / plain sum / norm of V_del
  size_t mats;         // float   [heads][3][d*d]         scratch matrices of the per-head finalisation
  size_t delta;        // float   [heads][d]
  size_t sel_flags;    // int32   [heads]: OBF_SELECT_* bits of the fused selection (read into obf_diag_t when diagnostics are asked for)
  size_t band;         // 16 bytes [heads][kBandCap]: scratch of the threshold re-decision (layerwise: exact per-head masses of the band)
  size_t layer_scores; // float   [L][N]        attention mass summed over the heads of a layer (layerwise selector)
  size_t layer_idx;    // int32   [L][max_budget], then int32 [L]: the shared index lists and their lengths
  size_t fro_part;     // double  [heads][ceil(max_budget/16)]   per-gather-block sums of squares of the retained V rows
  size_t rot;          // float   [heads][kJacobiSweeps][d-1][d/2]  rotation tangents of the Jacobi iteration (max_budget < d only)
  size_t keep_gram;    // double  [kKeepGramSlots][kKeepGramChunks][d*d]  partial Gram matrices (max_budget >= kKeepGramMinBudget)
  size_t lead_job;     // LeadJob [heads]                 hand-over from the finalisation to the leading-eigenpair kernel
  size_t inv_norm;     // float   [heads][max_budget]     reciprocal norms of the retained keys (cache merging)
  size_t route;        // int32   [heads][N]              retained slot of every deleted token (cache merging, when not an output)
  size_t total;
  int nchunk;          // score chunks per head
  int chunk_tokens;    // tokens per score chunk
  int rgroups, tiles_per_head, tiles_per_range, nranges, nslot;   // matrix-core score partition
  int nstat;           // statistics chunks per head
};

struct HeadState {
  double a_keep, a_del;
  int32_t n_keep, n_del;
  int32_t r_keep;       // dimension of the retained span, -1 = not computed
  int32_t active;       // 1: residual statistics and injection are needed
  int32_t k_used;
  int32_t pad;
  float rcr, ivn;
};

// What the finalisation hands to the leading-eigenpair kernel for a head it does not diagonalise itself.
struct LeadJob {
  int32_t pending;      // 1: the residual Gram matrix T (m x m, complement coordinates) waits in the head's scratch
  int32_t m;
  float res2, vd2, pc, pcr, rcr;
  int32_t pad;
};

// One chunk's statistics of the deleted values: G [d][d] (tiles on and below the diagonal), u = sum_j A_j v_j [d],
// s = sum_j v_j [d], ||V_del||_F^2, padding.
__host__ __device__ inline size_t gram_stride(int d) { return (size_t)d * d + 2 * (size_t)d + 4; }

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

inline Workspace carve(const Dims& m, int max_budget, int rank) {
  Workspace w;
  // reference-precision score path: fixed chunks of 512 tokens
  w.chunk_tokens = 512;
  w.nchunk = (m.N + w.chunk_tokens - 1) / w.chunk_tokens;
  w.nstat = (m.N + kStatChunk - 1) / kStatChunk;
  // matrix-core score path: the flattened (head, 32-token tile) space is cut into one range per
  // persistent workgroup; a head is covered by at most nslot ranges
  w.rgroups = (m.R + score_rows_per_group(m.R) - 1) / score_rows_per_group(m.R);
  w.tiles_per_head = (m.N + 31) / 32;
  {
    const long TT = (long)m.heads * w.tiles_per_head;
    // ranges: a multiple of 8 (one share per XCD) such that an XCD's ranges x row groups fit its 32 compute units
    const int per_xcd = (kNumCU / 8) / w.rgroups > 0 ? (kNumCU / 8) / w.rgroups : 1;
    const int G = 8 * per_xcd;
    long T = (TT + G - 1) / G;
    T = ((T + 3) / 4) * 4;
    if (T < 4) T = 4;
    w.tiles_per_range = (int)T;
    w.nranges = (int)((TT + T - 1) / T);
    w.nslot = (int)((w.tiles_per_head + T - 1) / T) + 1;
  }
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
  w.stats_part = take(sizeof(double) * 2 * (size_t)m.heads * (w.nchunk > w.nslot ? w.nchunk : w.nslot) * m.R);
  w.row_lse = take(sizeof(double) * (size_t)m.heads * m.R);
  w.scores = take(sizeof(float) * (size_t)m.heads * m.N);
  w.score_part = take(w.rgroups > 1 ? sizeof(float) * (size_t)w.rgroups * m.heads * m.N : 0);
  w.head_state = take(sizeof(HeadState) * (size_t)m.heads);
  w.decided = take(sizeof(int32_t) * (size_t)m.heads);
  w.basis = take(sizeof(float) * (size_t)m.heads * m.d * m.d);
  w.gram_part = take(sizeof(float) * (size_t)m.heads * w.nstat * gram_stride(m.d));
  w.mats = take(sizeof(float) * (size_t)m.heads * 3 * m.d * m.d);
  w.delta = take(sizeof(float) * (size_t)m.heads * m.d);
  w.sel_flags = take(sizeof(int32_t) * (size_t)m.heads);
  w.band = take(16 * (size_t)m.heads * kBandCap);
  w.layer_scores = take(sizeof(float) * (size_t)m.L * m.N);
  w.layer_idx = take(sizeof(int32_t) * ((size_t)m.L * (max_budget > 0 ? max_budget : 0) + m.L));
  w.fro_part = take(sizeof(double) * (size_t)m.heads * ((max_budget > 0 ? max_budget : 0) / kGatherRows + 1));
  w.rot = take((max_budget < m.d && rank > 0) ? sizeof(float) * (size_t)m.heads * kJacobiSweeps * (m.d - 1) * (m.d / 2) : 0);
  w.keep_gram = take(max_budget >= kKeepGramMinBudget ? sizeof(double) * kKeepGramSlots * kKeepGramChunks * (size_t)m.d * m.d : 0);
  w.lead_job = take(sizeof(LeadJob) * (size_t)m.heads);
  w.inv_norm = take(sizeof(float) * (size_t)m.heads * (max_budget > 0 ? max_budget : 0));
  w.route = take(sizeof(int32_t) * (size_t)m.heads * m.N);
  w.total = off;
  return w;
}

enum Stage {
  ST_SCORE_STATS = 0, ST_SCORE_LSE, ST_SCORE_MASS, ST_SELECT, ST_REFINE, ST_GATHER, ST_KEEP_CERT, ST_KEEP_BASIS, ST_DEL_STATS,
  ST_FINALIZE, ST_COUNT
};

// Brackets one kernel launch with HIP events when profiling of that stage is enabled.
struct ProfScope {
  ProfScope(int stage, hipStream_t st);
  ~ProfScope();
  void* rec;
  hipStream_t st;
};

void set_error(const char* fmt, ...);
obf_status_t check_launch(const char* what);

// ---- device helpers -------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even float -> bf16 bits; NaN stays NaN
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  uint32_t lsb = (u >> 16) & 1u;
  return (uint16_t)((u + 0x7fffu + lsb) >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<uint16_t> {
  static __device__ __forceinline__ float load(const uint16_t* p) { return bf16_bits_to_float(*p); }
  static __device__ __forceinline__ void store(uint16_t* p, float v) { *p = float_to_bf16_bits(v); }
};

// ---- stage launchers (each enqueues on `st`, returns OBF_OK or OBF_ERR_HIP) --------------
obf_status_t launch_score_generic(const Dims& m, const Workspace& w, char* ws, const void* K, const void* Q,
                                  float* scores, double* row_lse, hipStream_t st);
bool mfma_score_supported(const Dims& m);
obf_status_t launch_score_mfma(const Dims& m, const Workspace& w, char* ws, const void* K, const void* Q,
                               float* scores, double* row_lse, hipStream_t st);
obf_status_t launch_select(const Dims& m, const float* scores, const int32_t* budgets_host, int32_t budget,
                           int32_t max_budget, int32_t* idx, int32_t* n_keep, hipStream_t st);
obf_status_t launch_select_refine(const Dims& m, const float* scores, const int32_t* budgets_host, int32_t budget,
                                  int32_t max_budget, int32_t* idx, int32_t* n_keep, const void* K, const void* Q,
                                  const double* row_lse, hipStream_t st, int32_t* sel_flags = nullptr /*[heads], nullable*/);
// diag[h].select_flags = sel_flags[h] for every head (diagnostics only)
obf_status_t launch_diag_flags(obf_diag_t* diag, const int32_t* sel_flags, int heads, hipStream_t st);
obf_status_t launch_refine(const Dims& m, const Workspace& w, char* ws, const void* K, const void* Q,
                           const float* scores, const double* row_lse, int32_t max_budget, int32_t* idx,
                           const int32_t* n_keep, hipStream_t st);
obf_status_t launch_gather(const Dims& m, const void* K, const void* V, const int32_t* idx, const int32_t* n_keep,
                           int32_t max_budget, void* K_out, void* V_out, hipStream_t st, double* fro_part = nullptr);
// Retained-span basis for the heads with at most head_dim retained rows (the others are left untouched).
obf_status_t launch_keep_basis_small(const Dims& m, const void* V, const float* scores, const int32_t* idx,
                                     const int32_t* n_keep, int32_t max_budget, int32_t rank, HeadState* state,
                                     float* basis, hipStream_t st);
bool del_stats_mfma_supported(const Dims& m);
obf_status_t launch_del_stats_mfma(const Dims& m, const Workspace& w, const void* V, const float* scores,
                                   const int32_t* idx, int32_t max_budget, const HeadState* state,
                                   const int32_t* n_keep /*non-null: do not read the head states*/, float* gram_part,
                                   hipStream_t st, bool few_active = false /*nearly every head is expected to be inactive*/);
bool keep_cert_supported(const Dims& m);
obf_status_t launch_keep_cert(const Dims& m, const void* Vsrc, int via_idx, const float* scores, const int32_t* idx,
                              const int32_t* n_keep, int32_t max_budget, int32_t rank, HeadState* state,
                              int32_t* decided, hipStream_t st, const double* fro_part = nullptr, bool want_sums = true);
obf_status_t launch_refine_layers(const Dims& m, const void* K, const void* Q, const float* layer_scores,
                                  const double* row_lse, int32_t max_budget, int32_t* idx_layer,
                                  const int32_t* n_keep_layer, double* part /*[heads][kBandCap]*/, hipStream_t st);
// Layerwise retention rule: TopK_B of the head-summed scores of each layer (with the exact re-decision at the
// threshold), copied to every head of the layer.  budgets_host: per layer (nullable).
obf_status_t launch_select_layerwise(const Dims& m, const Workspace& w, char* ws, const float* scores,
                                     const int32_t* budgets_host, int32_t budget, int32_t max_budget, int32_t* idx,
                                     int32_t* n_keep, const void* K, const void* Q, const double* row_lse,
                                     hipStream_t st);
// Ablation variants of App. D as the kernels see them (obf_variant_t checked and packed).
enum : int { VF_NO_PROJECTION = 1, VF_SUBSPACE_ALL = 2, VF_SUBSPACE_EVR = 4, VF_NO_SCALING = 8, VF_NAIVE = 16, VF_ATTN_INJECT = 32, VF_PER_TOKEN = 64 };
struct Variant {
  int flags = 0;
  float evr_tau = 0.f;
  int subspace_iters = 0;          // > 0: App. H's Gram subspace iteration with this many steps instead of the eigen-decomposition
  bool skips_basis() const { return (flags & (VF_NO_PROJECTION | VF_NAIVE)) != 0; }
};

obf_status_t launch_append_message(int heads, int row_bytes, const void* prev_K, const void* prev_V, const int32_t* prev_len,
                                   int prev_len_all, int prev_stride, const void* keep_K, const void* keep_V,
                                   const int32_t* n_keep, int keep_stride, const void* gen_K, const void* gen_V, int n_gen,
                                   int gen_stride, void* msg_K, void* msg_V, int32_t* msg_len, int msg_stride, hipStream_t st);
// Cache merging (App. E) on selected and gathered rows: routes (route_out nullable) and merged values in V_out.
obf_status_t launch_cache_merge(const Dims& m, const Workspace& w, char* ws, const void* K, const void* V, const float* scores,
                                const int32_t* idx, const int32_t* n_keep, int32_t max_budget, const void* K_out,
                                void* V_out, int32_t* route_out, hipStream_t st);
// The Per-token alternative of App. D after a back-fill that left its subspace in the workspace (flag VF_PER_TOKEN) and
// did not inject: routes as in the cache merging, then one direction per retained slot added to V_out.
obf_status_t launch_per_token_inject(const Dims& m, const Workspace& w, char* ws, const void* K, const void* V,
                                     const float* scores, const int32_t* idx, const int32_t* n_keep, int32_t max_budget,
                                     const void* K_out, void* V_out, int no_scaling, hipStream_t st);
// Per-row int8 / int4 codes of relay rows and back (App. E's stacked quantisation, the reading stated in quant.hip).
obf_status_t launch_quant_rows(const void* X, long n_rows, int d, int dtype, int bits, uint8_t* codes, uint16_t* scale,
                               uint16_t* zero, hipStream_t st);
obf_status_t launch_dequant_rows(const uint8_t* codes, const uint16_t* scale, const uint16_t* zero, long n_rows, int d, int dtype,
                                 int bits, void* X, hipStream_t st);
// Runs `set` (hipFuncSetAttribute calls) once per device: kernel attributes belong to the device that is current when they
// are set.  `seen` and `mu` are the caller's function-local statics; the device's bit is set only after `set` has returned,
// so a second host thread either waits for the mutex or finds the attributes in place.
template <class F>
inline void once_per_device(std::mutex& mu, uint64_t& seen, F set) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) { set(); return; }
  std::lock_guard<std::mutex> lock(mu);
  if (seen & (1ull << dev)) return;
  set();
  seen |= 1ull << dev;
}

// idx[i] += offset for every valid (non-negative) entry
obf_status_t launch_idx_offset(int32_t* idx, size_t n, int32_t offset, hipStream_t st);

// The library's own streams: kAuxStreams per host thread and device, default priority, created on first use and kept.
// aux_stream returns nullptr when none is available (creation failed, or the thread is in single-stream mode): the
// launchers then keep everything on the caller's stream.
constexpr int kBatchLanes = 3;                                   // samples of a batch in flight at a time: with lane 0's
                                                                  // inner fork that makes four streams, one per hardware queue
constexpr int kAuxStreams = kBatchLanes;                          // the library's own streams per device and thread
hipStream_t aux_stream(int which /*0 .. kAuxStreams-1*/);
// While on (per host thread), no stream or event is created or used by the library.
void set_single_stream(bool on);
// Makes `waiter` wait for everything queued on `signaller` so far, through event `slot` of the calling thread's pool
// (an event may be recorded again as soon as its wait has been enqueued).  Legal under stream capture.
enum EventSlot { EV_SCORED = 0, EV_BASIS_FORK, EV_BASIS_JOIN, EV_KROWS_FORK, EV_KROWS_JOIN, EV_BATCH_FORK, EV_BATCH_JOIN, EV_COUNT };
obf_status_t stream_after(hipStream_t waiter, hipStream_t signaller, int slot);
// Optional early start of the retained-span bases on `aux` (forked from st), for shapes where they do not depend on
// the gather; *started is then passed on to launch_backfill as basis_started, which joins `aux` back.
obf_status_t launch_backfill_basis(const Dims& m, const Workspace& w, char* ws, const void* V, const float* scores,
                                   const int32_t* idx, const int32_t* n_keep, int32_t max_budget, int32_t rank,
                                   hipStream_t st, hipStream_t aux, bool* started);
obf_status_t launch_backfill(const Dims& m, const Workspace& w, char* ws, const void* V, const float* scores,
                             const int32_t* idx, const int32_t* n_keep, int32_t max_budget, int32_t rank,
                             void* V_out, float* delta_out, obf_diag_t* diag, hipStream_t st, hipStream_t aux /*nullable*/,
                             const double* fro_part = nullptr,
                             bool basis_started = false, int32_t min_budget = -1 /*smallest per-head budget if known*/,
                             Variant var = Variant());

}  // namespace obf
