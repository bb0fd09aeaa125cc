/*
 * obf_relay.h -- C ABI of the relay-boundary KV compression library for MI355X (gfx950).
 *
 * One call compresses the prompt block of an agent's KV cache before it is relayed to the
 * next agent: per (layer, KV head) it scores the prompt tokens by the attention mass they
 * receive from a window of observation queries (Eq. 1), keeps the top-B tokens (TopK_B,
 * Sec. 4.3.2 / Alg. 2), gathers their keys and values, and applies Orthogonal BackFill
 * (Sec. 4.4, Eq. 2-7 / Alg. 3): one low-rank correction vector, orthogonal to the span of
 * the retained values, is added to every retained value; keys and the retained index set
 * are left untouched.
 *
 * Conventions common to every entry point
 *   - Every data pointer is a DEVICE pointer unless its name ends in `_host`.
 *   - The caller owns all buffers.  The library never allocates, frees or keeps device
 *     memory; scratch space is the caller's workspace `ws` of at least
 *     obf_workspace_bytes() bytes, 256-byte aligned.  Its contents are undefined after a call.
 *     Host-side resources the library does create, once per host thread and device and kept until the
 *     process ends: two streams and a handful of events (first call that can use a second stream), and
 *     pairs of timing events while stage profiling is on.  obf_compress_relay_static creates none.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*); nothing is
 *     synchronised.  Inputs are never modified.  obf_backfill and the fused calls may run part
 *     of their work on a second stream that the library creates once per host thread and device
 *     (default priority): it is forked from `stream` with an event and joined back into `stream`
 *     before the call returns, so all results are ordered on `stream`; the pattern is legal under
 *     stream capture.
 *   - Argument errors are found on the host before anything is enqueued and reported as
 *     a status code; obf_last_error() gives a thread-local message.  No exceptions, no abort.
 *   - Layouts are contiguous, row-major, head-major:
 *       K, V        [n_layers][n_kv_heads][n_tokens][head_dim]          dtype
 *       Qwin        [n_layers][n_kv_heads*group][window][head_dim]      dtype
 *                   query head i belongs to KV head i / group; Q and K are taken as given
 *                   (position encoding already applied)
 *       scores      [n_layers][n_kv_heads][n_tokens]                    float
 *       row_lse     [n_layers][n_kv_heads][group*window]                double
 *       idx         [n_layers][n_kv_heads][max_budget]                  int32, ascending,
 *                                                                       entries >= n_keep are -1
 *       n_keep      [n_layers][n_kv_heads]                              int32
 *       K_out,V_out [n_layers][n_kv_heads][max_budget][head_dim]        dtype, rows >= n_keep zero
 *       delta_out   [n_layers][n_kv_heads][head_dim]                    float (optional)
 *       diag        [n_layers][n_kv_heads]                              obf_diag_t (optional)
 *   - Limits: head_dim in {64, 128}; 1 <= n_tokens <= 32768; 1 <= group*window <= 4096;
 *     n_layers*n_kv_heads <= 65535; budget >= 0 and min(budget, n_tokens) <= max_budget (a budget above
 *     n_tokens keeps every token).  Anything else is OBF_ERR_UNSUPPORTED / OBF_ERR_INVALID_ARG.
 */
#ifndef OBF_RELAY_H
#define OBF_RELAY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  OBF_OK = 0,
  OBF_ERR_INVALID_ARG = 1,
  OBF_ERR_UNSUPPORTED = 2,
  OBF_ERR_WORKSPACE_TOO_SMALL = 3,
  OBF_ERR_HIP = 4
} obf_status_t;

typedef enum { OBF_F32 = 0, OBF_BF16 = 1 } obf_dtype_t;

typedef struct {
  int32_t n_layers;
  int32_t n_kv_heads;
  int32_t group;      /* query heads per KV head (GQA) */
  int32_t head_dim;   /* d */
  int32_t n_tokens;   /* N prompt tokens per head */
  int32_t window;     /* W observation queries per query head */
  int32_t dtype;      /* obf_dtype_t of K, V, Qwin, K_out, V_out */
} obf_shape_t;

/* Bits of obf_diag_t.select_flags.
 *   OBF_SELECT_BAND_OVERFLOW  more than 256 tokens have single-precision scores within 1e-4 (relative) of the head's threshold
 *                             score and they straddle it: the double-precision re-decision at the threshold was not run
 *                             for this head, its index list follows the single-precision scores (ties to the lowest
 *                             index); exact for all-equal scores, otherwise within the single-precision error of Eq. 1. */
#define OBF_SELECT_BAND_OVERFLOW 1

/* Per-head diagnostics: the quantities of App. K.2 (PCR, RCR, PC, REVR, DR, IVN) and the decisions taken. */
typedef struct {
  int32_t n_keep;   /* retained tokens */
  int32_t r_keep;   /* dimension of the retained value span (Eq. 2); 0 if not computed */
  int32_t k_used;   /* residual principal directions used (Sec. 4.4, k = min(pca_rank, rank R)) */
  int32_t skipped;  /* 1: no injection (empty P_del, rank 0, span = R^d, negligible residual) */
  float a_keep;     /* sum of attention mass over retained tokens (Eq. 6) */
  float a_del;      /* sum over deleted tokens */
  float rcr;        /* residual content ratio ||R||_F^2 / (||V_del||_F^2 + eps) */
  float ivn;        /* injection vector norm ||delta||_2 */
  float pcr;        /* projected content ratio ||V_par||_F^2 / (||V_del||_F^2 + eps); 1 when the retained span is R^d */
  float pc;         /* projection cosine between the column sums of V_del and of V_par; 0 when not computed */
  float revr;       /* residual explained variance ratio of the k_used directions; 0 when none is used */
  float dr;         /* demand ratio a_del / (a_keep + eps) */
  int32_t select_flags; /* OBF_SELECT_* bits of the head's selection; set by the fused headwise calls only (0 elsewhere) */
  float fast_err;   /* with obf_variant_t.subspace_iters > 0: ||Delta_fast - Delta_svd|| / ||Delta_svd|| of the head
                       (App. H), 0 if Delta_svd = 0; -1 when not computed (any other call, and heads without an injection
                       decision by Eq. 5) */
} obf_diag_t;

/* Bytes of workspace any entry point needs for this shape (host function, no device work).
 * Returns 0 if the shape is unsupported. */
size_t obf_workspace_bytes(const obf_shape_t* shape, int32_t max_budget, int32_t rank);

/* Eq. 1 (the scoring step of Alg. 2): scores[l][h][j] = sum over the group*window query rows of
 * softmax_j(q . k_j / sqrt(d)), softmax over the n_tokens keys of the head.
 * row_lse (nullable) receives log(sum_j exp(logit)) of every query row in double; the
 * boundary refinement needs it. */
obf_status_t obf_score(const obf_shape_t* shape, const void* K, const void* Qwin, float* scores,
                       double* row_lse, void* ws, size_t ws_bytes, void* stream);

/* TopK_B (Sec. 4.3.2, the selection step of Alg. 2) on the float scores as given: the B largest, ties to the
 * lowest index, written ascending.  Pure integer/compare work on the fp32 bit patterns.
 * budgets_host (nullable, host memory, [n_layers*n_kv_heads]) gives per-head budgets;
 * otherwise `budget` is used for every head.  Budgets above n_tokens keep everything. */
obf_status_t obf_select_topk(const obf_shape_t* shape, const float* scores, const int32_t* budgets_host,
                             int32_t budget, int32_t max_budget, int32_t* idx, int32_t* n_keep,
                             void* ws, size_t ws_bytes, void* stream);

/* Re-decides, in double precision, the membership of the tokens whose float score lies within
 * a relative band of the selection threshold, so that the retained set is the one exact
 * arithmetic on the given K / Qwin bits would give (ties still to the lowest index).
 * idx / n_keep are updated in place; n_keep does not change. */
obf_status_t obf_refine_boundary(const obf_shape_t* shape, const void* K, const void* Qwin, const float* scores,
                                 const double* row_lse, int32_t max_budget, int32_t* idx, const int32_t* n_keep,
                                 void* ws, size_t ws_bytes, void* stream);

/* The gather step of Alg. 2: K_out = K[idx], V_out = V[idx] as bit copies; rows >= n_keep are zeroed.
 * Either output may be NULL to skip it. */
obf_status_t obf_gather(const obf_shape_t* shape, const void* K, const void* V, const int32_t* idx,
                        const int32_t* n_keep, int32_t max_budget, void* K_out, void* V_out, void* stream);

/* Orthogonal BackFill (Eq. 2-7, Alg. 3) on already gathered values: V_out holds
 * V[idx] on entry and V[idx] + delta on exit (rounded to dtype); untouched where OBF is
 * skipped.  `rank` is pca_rank (0 = plain eviction).  delta_out, diag nullable; the diagnostics take an extra pass over
 * the scores of every head, so a caller on the hot path leaves diag NULL. */
obf_status_t obf_backfill(const obf_shape_t* shape, const void* V, const float* scores, const int32_t* idx,
                          const int32_t* n_keep, int32_t max_budget, int32_t rank, void* V_out,
                          float* delta_out, obf_diag_t* diag, void* ws, size_t ws_bytes, void* stream);

/* The whole relay compression Phi_OBF (Alg. 3) in one enqueue: score, select, refine, gather,
 * back-fill.  Outputs equal those of the five stage calls run in that order.
 * scores_out, delta_out, diag nullable. */
obf_status_t obf_compress_relay(const obf_shape_t* shape, const void* K, const void* V, const void* Qwin,
                                const int32_t* budgets_host, int32_t budget, int32_t max_budget, int32_t rank,
                                void* K_out, void* V_out, int32_t* idx, int32_t* n_keep,
                                float* scores_out, float* delta_out, obf_diag_t* diag,
                                void* ws, size_t ws_bytes, void* stream);

/* The same relay compression with the layerwise granularity of the retention rule (Sec. 4.3.2, the "L" selector
 * and L-OBF of Sec. 5): per layer, TopK_B of the attention mass summed over the layer's KV heads (ties to the
 * lowest index, the threshold re-decided in double precision like the headwise rule); every head of the layer
 * keeps that one index set, and Orthogonal BackFill runs per head with the head's own attention mass in
 * Eq. 4 / Eq. 6.  budgets_host (nullable, host memory) holds one budget per LAYER ([n_layers]); all other
 * arguments, layouts, ownership and error behaviour are those of obf_compress_relay (idx and n_keep are still
 * written per head: the heads of a layer receive identical lists). */
obf_status_t obf_compress_relay_layerwise(const obf_shape_t* shape, const void* K, const void* V, const void* Qwin,
                                          const int32_t* budgets_host, int32_t budget, int32_t max_budget, int32_t rank,
                                          void* K_out, void* V_out, int32_t* idx, int32_t* n_keep,
                                          float* scores_out, float* delta_out, obf_diag_t* diag,
                                          void* ws, size_t ws_bytes, void* stream);

/* Ablation variants of App. D: every field switches one step of Orthogonal BackFill off or replaces it; all zero
 * is the method of Sec. 4.4.  The fields combine freely (naive_aggregation makes the first four irrelevant).
 *   no_projection      "No Projection": Eq. 3 is skipped, R = V_del; the basis of the retained span is not built and
 *                      a head is processed whatever that span is (diag.r_keep = 0, pcr = pc = 0, rcr = 1).
 *   subspace           OBF_SUBSPACE_RANK: the top `rank` right singular directions of R (the method);
 *                      OBF_SUBSPACE_ALL: "Max-P", every direction of R's row space (k = rank R);
 *                      OBF_SUBSPACE_EVR: "EVR-adaptive", the smallest k whose leading squared singular values
 *                      reach the fraction evr_tau of their total (never above rank R); `rank` must still be > 0.
 *   evr_tau            in (0, 1], read only with OBF_SUBSPACE_EVR.
 *   no_scaling         "No Scaling": delta = Delta, without the demand ratio of Eq. 6.
 *   naive_aggregation  "Naive Aggregation": delta = unweighted mean of the deleted value rows (no Eq. 3-6).
 *   attn_inject        "Attn-inject": row t of V_out receives n_keep * A_t / (sum of A over the retained rows + eps)
 *                      times delta instead of delta (Eq. 7 replaced); delta_out is still delta.
 *   subspace_iters     0: the exact top-`rank` directions.  t > 0 (at most 64): the fast path of App. H, t steps of
 *                      C <- orth(C G), G = R^T R, from the first k = min(rank, d - r_keep, |P_del|) rows of the
 *                      orthonormal cosine basis C_0[i][c] = sqrt(2/d) cos(pi (i + 1/2)(c + 1/2) / d) (the paper asks
 *                      only for orthonormal rows and runs t = 3); orth is Gram-Schmidt over the rows in order, a row
 *                      left with at most 1e-5 of the first row's norm is dropped (k_used counts the rows kept, revr is
 *                      their share of the trace).  Needs subspace = OBF_SUBSPACE_RANK, rank <= 16 and head_dim <= 128,
 *                      else OBF_ERR_UNSUPPORTED.  With diag != NULL the exact directions are computed too and
 *                      diag.fast_err reports the distance between the two (this costs the exact route's time).
 *   per_token          "Per-token" (App. D names it without a formula; this is a stated reading): the deleted tokens are
 *                      shared out among the retained slots by key cosine similarity (the routing of obf_cache_merge),
 *                      slot t receives delta_t = n_keep * a_del / (a_keep + eps) * Proj_C(sum over its tokens of
 *                      A_j R_j / (a_del + eps)) instead of delta (C: the subspace of Eq. 5), so that the mean over the
 *                      slots is Eq. 6's delta - which is what delta_out and diag still report.  A slot no token is routed
 *                      to keeps its value.  Fused calls only (the routing reads the keys): obf_backfill_variant returns
 *                      OBF_ERR_UNSUPPORTED for it.  Combines with no_projection, no_scaling and subspace_iters; needs
 *                      subspace = OBF_SUBSPACE_RANK, rank <= 16, head_dim <= 128, no naive_aggregation, no attn_inject.
 * `rank` = 0 is plain eviction under every variant. */
#define OBF_SUBSPACE_RANK 0
#define OBF_SUBSPACE_ALL 1
#define OBF_SUBSPACE_EVR 2
typedef struct obf_variant_t {
  int32_t no_projection;
  int32_t subspace;
  float evr_tau;
  int32_t no_scaling;
  int32_t naive_aggregation;
  int32_t attn_inject;
  int32_t subspace_iters;
  int32_t per_token;
} obf_variant_t;

/* obf_backfill with an ablation variant (App. D); variant == NULL is obf_backfill itself.  Arguments, layouts,
 * ownership and error behaviour as obf_backfill; an unknown subspace value or evr_tau outside (0, 1] is
 * OBF_ERR_INVALID_ARG. */
obf_status_t obf_backfill_variant(const obf_shape_t* shape, const void* V, const float* scores, const int32_t* idx,
                                  const int32_t* n_keep, int32_t max_budget, int32_t rank,
                                  const obf_variant_t* variant, void* V_out, float* delta_out, obf_diag_t* diag,
                                  void* ws, size_t ws_bytes, void* stream);

/* The fused relay compression with an ablation variant (App. D ablates L-OBF: layerwise != 0 selects the per-layer
 * retention rule of obf_compress_relay_layerwise, 0 the headwise one of obf_compress_relay; budgets_host is per
 * layer or per head accordingly).  variant == NULL is the corresponding plain call. */
obf_status_t obf_compress_relay_variant(const obf_shape_t* shape, const void* K, const void* V, const void* Qwin,
                                        const int32_t* budgets_host, int32_t budget, int32_t max_budget, int32_t rank,
                                        int32_t layerwise, const obf_variant_t* variant,
                                        void* K_out, void* V_out, int32_t* idx, int32_t* n_keep,
                                        float* scores_out, float* delta_out, obf_diag_t* diag,
                                        void* ws, size_t ws_bytes, void* stream);

/* Relay assembly around the compression (Sec. 3.2-3.3, Sec. 4.3.2, App. A.7).
 *
 * obf_window_t places the prompt of one sample inside a larger, right-padded cache and names the shared attention sink:
 *   token_stride  tokens between consecutive heads of K and V in memory (>= shape.n_tokens; 0 means n_tokens).
 *                 shape.n_tokens is the number of real prompt tokens; the rows behind them (padding) are never read.
 *   sink          the first `sink` tokens are the attention sink S: they are keys of the softmax of Eq. 1 like every
 *                 real token, but they are not in the eligible set Omega, i.e. neither candidates of TopK_B nor deleted
 *                 values of Eq. 3-6 (the sink travels inside the inherited message, M_0 = S).  0 <= sink < n_tokens.
 * obf_compress_relay_window is obf_compress_relay_variant on that window: budgets count eligible tokens (a budget
 * above n_tokens - sink keeps every eligible token), idx holds token numbers of the head (>= sink), scores_out covers
 * all n_tokens real tokens ([n_layers][n_kv_heads][n_tokens], dense).  window == NULL and variant == NULL are the
 * plain calls.  Errors as obf_compress_relay, plus OBF_ERR_INVALID_ARG for a window outside the limits above. */
typedef struct obf_window_t {
  int32_t token_stride;
  int32_t sink;
} obf_window_t;

obf_status_t obf_compress_relay_window(const obf_shape_t* shape, const obf_window_t* window,
                                       const void* K, const void* V, const void* Qwin,
                                       const int32_t* budgets_host, int32_t budget, int32_t max_budget, int32_t rank,
                                       int32_t layerwise, const obf_variant_t* variant,
                                       void* K_out, void* V_out, int32_t* idx, int32_t* n_keep,
                                       float* scores_out, float* delta_out, obf_diag_t* diag,
                                       void* ws, size_t ws_bytes, void* stream);

/* The message an agent hands on (Sec. 3.3): M_i = [M_{i-1}; Phi(P; G); G], row-wise per (layer, KV head), keys and
 * values alike.  For head h the output rows are prev[h][0 .. prev_len[h]), then keep[h][0 .. n_keep[h]), then
 * gen[h][0 .. n_gen), all bit copies; msg_len[h] receives their number and the rows behind them up to msg_stride are
 * zeroed.  Every part is [n_heads][*_stride][head_dim] of `dtype` (n_heads = layers x KV heads); prev_len
 * (nullable: every head has prev_len_all rows) and n_keep are device arrays [n_heads]; for the first agent prev is the
 * prompt cache itself with prev_len_all = sink.  A part with zero rows may be NULL.  The host checks what it can see
 * (negative sizes, NULL parts, n_gen > gen_stride, prev_len_all > prev_stride: OBF_ERR_INVALID_ARG, nothing enqueued);
 * lengths that live on the device are checked there: a head whose parts exceed prev_stride, keep_stride or msg_stride
 * gets msg_len[h] = -1 and all-zero rows. */
obf_status_t obf_append_message(int32_t n_heads, int32_t head_dim, int32_t dtype,
                                const void* prev_K, const void* prev_V, const int32_t* prev_len, int32_t prev_len_all,
                                int32_t prev_stride,
                                const void* keep_K, const void* keep_V, const int32_t* n_keep, int32_t keep_stride,
                                const void* gen_K, const void* gen_V, int32_t n_gen, int32_t gen_stride,
                                void* msg_K, void* msg_V, int32_t* msg_len, int32_t msg_stride, void* stream);

/* A batch of samples in one call (App. A.7: right padding, per-sample lengths).  Storage is right-padded:
 *   K, V      [n_samples][n_layers][n_kv_heads][token_stride][head_dim], sample s holds n_tokens_host[s] real tokens per head
 *   Qwin      [n_samples][n_layers][n_kv_heads*group][window][head_dim]
 *   K_out, V_out, idx, n_keep, diag: the layouts of obf_compress_relay with a leading [n_samples] dimension
 * shape describes one sample (shape.n_tokens is ignored; every n_tokens_host[s] must lie in [1, token_stride] and obey the
 * library's token limit).  n_tokens_host and budgets_host are HOST arrays of n_samples entries (budgets_host nullable:
 * `budget` for every sample); a sample's budget applies to each of its heads and counts eligible tokens; `sink` as in
 * obf_window_t (0 <= sink < every n_tokens_host[s]).  Each sample is compressed exactly as obf_compress_relay_window would
 * compress it alone.  obf_workspace_bytes_batch() returns room for up to three samples in flight (one slot each; with
 * n_samples = 1 it returns the size of one slot): sample s then runs in lane s mod 3, lane 0 being `stream` and the others
 * streams of the library's own (forked off `stream` and joined back before the call returns, so that all work is ordered
 * on `stream` for the caller); a workspace of one or two slots is accepted too and gives that many lanes, and under stream
 * capture or stage profiling the samples are simply enqueued one after the other on `stream`.  Results do not depend on
 * the number of lanes.  diag nullable.  Errors as
 * obf_compress_relay; nothing is enqueued on a host-side error. */
size_t obf_workspace_bytes_batch(const obf_shape_t* shape, int32_t n_samples, int32_t token_stride, int32_t max_budget, int32_t rank);
obf_status_t obf_compress_relay_batch(const obf_shape_t* shape, int32_t n_samples, const int32_t* n_tokens_host,
                                      int32_t token_stride, int32_t sink,
                                      const void* K, const void* V, const void* Qwin,
                                      const int32_t* budgets_host, int32_t budget, int32_t max_budget, int32_t rank,
                                      void* K_out, void* V_out, int32_t* idx, int32_t* n_keep, obf_diag_t* diag,
                                      void* ws, size_t ws_bytes, void* stream);

/* The cache-merging comparison system of App. E ("Cache-merging implementation", steps ii and iii) on rows that were
 * already selected and gathered: every deleted token j is routed to the retained slot t whose key has the highest
 * cosine similarity with K_j (the first maximum wins; a key of zero norm has cosine 0 with every key), then
 * V_out[t] = V[idx[t]] + sum over the j routed to t of scores[j] / (scores[idx[t]] + 1e-12) * V[j], added in ascending j
 * and rounded once to dtype; slots that receive nothing keep the bit copy.  Keys are unchanged.
 *   K, V      the head's full key / value rows; scores as from obf_score; idx / n_keep as from obf_select_topk
 *   K_out     gathered keys (read only); V_out gathered values on entry, merged values on exit
 *   route_out nullable, int32 [n_layers][n_kv_heads][n_tokens]: the slot of every deleted token, -1 for retained tokens
 * Ownership, stream and error behaviour as obf_backfill. */
obf_status_t obf_cache_merge(const obf_shape_t* shape, const void* K, const void* V, const float* scores, const int32_t* idx,
                             const int32_t* n_keep, int32_t max_budget, const void* K_out, void* V_out, int32_t* route_out,
                             void* ws, size_t ws_bytes, void* stream);

/* The whole comparison system in one enqueue: (i) score, select and refine exactly as obf_compress_relay, gather,
 * then obf_cache_merge.  scores_out, route_out nullable; other arguments as obf_compress_relay. */
obf_status_t obf_compress_relay_merge(const obf_shape_t* shape, const void* K, const void* V, const void* Qwin,
                                      const int32_t* budgets_host, int32_t budget, int32_t max_budget,
                                      void* K_out, void* V_out, int32_t* idx, int32_t* n_keep,
                                      float* scores_out, int32_t* route_out, void* ws, size_t ws_bytes, void* stream);

/* Stacked int8 / int4 relay (the "+ int8" / "+ int4" rows of App. E's comparison table) on rows of the compressed cache
 * (K_out, V_out of the calls above, or any [n_rows][head_dim] array of `dtype`).  The paper names no scheme; this one
 * reproduces its ratios (16 d / (8 d + 32) = 1.94 and 16 d / (4 d + 32) = 3.76 at head_dim 128): per row,
 *   zero = fp16(min x), scale = fp16((max x - min x) / L), L = 2^bits - 1, q_c = clamp(rint((x_c - zero) / scale), 0, L)
 * (all codes 0 when scale is 0), the decision taken in single precision with individually rounded operations.
 *   codes      uint8 [n_rows][head_dim] for bits = 8; [n_rows][head_dim / 2] for bits = 4 (even column in the low half)
 *   scale_f16, zero_f16   half-precision bit patterns, [n_rows] each
 * obf_dequantize_rows writes x_hat = zero + scale * q, rounded once to single precision and then to `dtype`.
 * Values must lie in the half-precision range.  bits other than 4 or 8: OBF_ERR_INVALID_ARG. */
obf_status_t obf_quantize_rows(const void* X, int64_t n_rows, int32_t head_dim, int32_t dtype, int32_t bits,
                               uint8_t* codes, uint16_t* scale_f16, uint16_t* zero_f16, void* stream);
obf_status_t obf_dequantize_rows(const uint8_t* codes, const uint16_t* scale_f16, const uint16_t* zero_f16, int64_t n_rows,
                                 int32_t head_dim, int32_t dtype, int32_t bits, void* X_out, void* stream);

/* For callers that cannot allocate (code under HIP graph capture, serving loops and harnesses that forbid
 * hipMalloc): obf_compress_relay without a workspace argument and without the optional outputs.  Its scratch is
 * an array of OBF_STATIC_SCRATCH_BYTES bytes inside the library's device code (one copy per GPU, held until the
 * process ends), so the call makes no hipMalloc / hipFree, creates no stream or event (all work stays on `stream`;
 * the retained K rows are not copied on a second stream) and calls no allocating routine.  A shape whose
 * obf_workspace_bytes() exceeds the array is OBF_ERR_UNSUPPORTED (nothing enqueued); stage profiling must be off.
 * Outputs equal obf_compress_relay's bit for bit.  Every call on a GPU uses that GPU's one array, which keeps the
 * last call's contents: no kernel relies on its initial contents, but two calls that overlap in time on one GPU
 * (different streams or host threads) race on it - the caller serialises them. */
#define OBF_STATIC_SCRATCH_BYTES (48u << 20)
size_t obf_static_scratch_bytes(void);
obf_status_t obf_compress_relay_static(const obf_shape_t* shape, const void* K, const void* V, const void* Qwin,
                                       const int32_t* budgets_host, int32_t budget, int32_t max_budget, int32_t rank,
                                       void* K_out, void* V_out, int32_t* idx, int32_t* n_keep, void* stream);

/* Profiling aid (tracing of the path's own kernels with HIP events on the caller's stream).
 * obf_profile_enable(stage) makes every later call on this thread bracket the launch of that
 * internal stage's kernel with a pair of events; stage -1 switches it off.  obf_profile_read
 * waits for the recorded events, returns the summed elapsed milliseconds and the number of
 * launches since the last read, and resets both.  Stage ids run 0 .. obf_profile_stage_count()-1;
 * obf_profile_stage_name gives the kernel family each one covers. */
obf_status_t obf_profile_enable(int32_t stage);
obf_status_t obf_profile_read(double* total_ms, int32_t* launches);
int32_t obf_profile_stage_count(void);
const char* obf_profile_stage_name(int32_t stage);

/* Message for the calling thread's last non-OK status (static storage, never NULL). */
const char* obf_last_error(void);

/* Library version string (static storage). */
const char* obf_version(void);

#ifdef __cplusplus
}
#endif
#endif /* OBF_RELAY_H */
