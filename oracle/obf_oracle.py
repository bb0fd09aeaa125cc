"""CPU oracle for relay-boundary KV compression: headwise attention-mass eviction
followed by Orthogonal BackFill (OBF).

THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, fp64 numpy restatement of the
method, one (layer, KV head) at a time, written to be checked against the paper
by eye.  Only tests, the smoke check and the benchmark's cpu_baseline leg may use
it; the product path never does.  It shares no code with the HIP path.

Every input value is taken as the exact real number its bf16 / fp32 bit pattern
denotes; all arithmetic is float64; outputs are rounded once to the I/O dtype.

Steps follow Sec. 4.3.2 (Eq. 1, TopK_B), Sec. 4.4 (Eq. 2-7), Alg. 2 and Alg. 3.
Readings taken where the paper leaves a choice (each is listed in the design notes):
  * Eq. 1's attention rows come from observation-window queries; the softmax is
    over the N prompt keys only, scale 1/sqrt(d) (App. L setup), no mask; the
    rows of all query heads that share a KV head are summed (GQA).
  * TopK_B ties go to the lowest index; index lists are ascending (Sec. 3.1).
  * orth() spans the numerical row space: singular values above
    sigma_max * max(rows, d) * 2^-23 (Eq. 2 only bounds r by min(B, d)).
  * rank(R) in k = min(pca_rank, rank R) uses the same rule.
  * "||R||_F negligible" (footnote of Eq. 7): ||R||_F^2 <= 1e-6 ||V_del||_F^2.
  * epsilon = 1e-12 exactly where Eq. 4 and Eq. 6 place it.
The layerwise granularity of the same retention rule (one index set per layer) is
compress_layer.
The ablations of App. D are the flags of Variant; readings taken there:
  * No Projection: R = V_del, so neither the retained basis nor the "retained
    span is everything" skip takes part; the rest of Eq. 4-7 is unchanged.
  * Max-P: k = rank R (every direction of the residual's row space).
  * No Scaling: delta = Delta (the demand ratio of Eq. 6 is left out).
  * Naive Aggregation: delta = unweighted mean of the deleted value rows, no
    projection, no subspace, no scaling.
  * Attn-inject: V*_t = V_t + B w_t delta, w_t = A_t / (sum_keep A + eps), with
    delta the Eq. 6 vector ("alpha delta" in Alg. 3's naming).
  * EVR-adaptive: k* = smallest k whose leading squared singular values of R
    reach the fraction tau of their total; never above rank R.
  * Fast SVD alternative (Sec. 4.4, App. H): subspace_iters > 0 replaces the SVD by that many steps of
    C <- orth(C G) on G = R^T R from a fixed orthonormal start (start_rows), with
    k = min(pca_rank, d - r, |P_del|) rows of which dependent ones are dropped; fast_err reports
    the distance of the resulting Delta from the SVD's.
  * Per-token (App. D): not stated precisely enough to restate; per_token_offsets is a stated reading, unpinned
    against the paper, pinned by the properties the reading itself fixes.
The cache-merging comparison system of App. E (select, route by key cosine, merge by
attention mass) is merge_head; readings: the first maximum wins the routing, a key of
zero norm has cosine 0 with everything, slots that receive nothing stay bit copies.
Relay assembly (Sec. 3.2-3.3, Sec. 4.3.2): the eligible set Omega leaves out padding
and the shared sink.  Readings: the arrays handed to this module hold real tokens
only (right padding is a storage matter); the first `sink` tokens stay keys of the
softmax of Eq. 1 but are neither candidates of TopK_B nor deleted values of
Eq. 3-6; index lists keep the head's own token numbers.  append_message is the
row-wise concatenation M_i = [M_{i-1}; Phi(P; G); G] of Sec. 3.3.
Pinned by tests/test_oracle_pins.py (closed forms, brute force, invariants).
Parity unpinned: absolute values on realistic caches (the paper prints no worked
numeric example); those rest on invariants only.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

EPS = 1e-12                 # Eq. 4, Eq. 6, footnote of Eq. 7
RANK_EPS = 2.0 ** -23       # single-precision epsilon, used on purpose in the rank rule
RCR_SKIP = 1e-6             # reading of "||R||_F negligible"


# ----------------------------------------------------------------------------- dtype
def decode(x: np.ndarray, dtype: str) -> np.ndarray:
    """Exact float64 value of fp32 values or bf16 bit patterns (uint16)."""
    if dtype == "f32":
        return np.asarray(x, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        bits = np.asarray(x, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
        return bits.view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def round_to_io(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 to the I/O dtype: fp32 (RNE) or bf16 bits (RNE, via one fp32 rounding).

    The device adds delta to V in fp32 and rounds that sum to bf16; the fp64 sum
    rounded to fp32 first and then to bf16 follows the same two roundings.
    """
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    if dtype == "f32":
        return f
    if dtype == "bf16":
        u = f.view(np.uint32)
        lsb = (u >> np.uint32(16)) & np.uint32(1)
        return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------- Eq. 1
def attention_mass(K: np.ndarray, Qrows: np.ndarray) -> np.ndarray:
    """A_j = sum over window-query rows of softmax_j(q . k_j / sqrt(d))   (Eq. 1).

    K [N, d] float64, Qrows [R, d] float64 (all window queries of all query heads
    of the KV group).  Returns A [N] float64; sum(A) == R.
    """
    N, d = K.shape
    if Qrows.shape[0] == 0 or N == 0:
        return np.zeros(N, dtype=np.float64)
    S = (Qrows @ K.T) / np.sqrt(float(d))
    S = S - S.max(axis=1, keepdims=True)
    P = np.exp(S)
    P /= P.sum(axis=1, keepdims=True)
    return P.sum(axis=0)


# ----------------------------------------------------------------------------- TopK_B
def select_topk(A: np.ndarray, budget: int) -> np.ndarray:
    """Indices of the `budget` largest A_j, ties to the lowest index, ascending (Sec. 4.3.2)."""
    N = A.shape[0]
    b = int(min(max(budget, 0), N))
    order = np.argsort(-A, kind="stable")      # stable: equal values keep index order
    return np.sort(order[:b]).astype(np.int64)


def complement(idx: np.ndarray, N: int) -> np.ndarray:
    m = np.ones(N, dtype=bool)
    m[idx] = False
    return np.nonzero(m)[0]


# ----------------------------------------------------------------------------- Eq. 2
def numerical_rank(sigma: np.ndarray, rows: int, cols: int) -> int:
    if sigma.size == 0 or sigma[0] <= 0.0:
        return 0
    return int(np.count_nonzero(sigma > sigma[0] * max(rows, cols) * RANK_EPS))


def orth_rowspace(V_keep: np.ndarray):
    """Q [d, r] with orthonormal columns spanning span(V_keep rows)   (Eq. 2).

    Returns (Q, sigma) where sigma are V_keep's singular values.
    """
    B, d = V_keep.shape
    if B == 0:
        return np.zeros((d, 0)), np.zeros(0)
    _, s, Vt = np.linalg.svd(V_keep, full_matrices=False)
    r = numerical_rank(s, B, d)
    return Vt[:r].T.copy(), s


# ----------------------------------------------------------------------------- Eq. 3-7
@dataclass(frozen=True)
class Variant:
    """One ablation of App. D per flag; the default is the method of Sec. 4.4."""
    no_projection: bool = False      # component ablation "No Projection"
    subspace: str = "rank"           # "rank": top pca_rank directions; "all": Max-P; "evr": EVR-adaptive rank
    evr_tau: float = 0.35
    no_scaling: bool = False         # component ablation "No Scaling"
    naive: bool = False              # component ablation "Naive Aggregation"
    attn_inject: bool = False        # alternative design "Attn-inject"
    per_token: bool = False          # alternative design "Per-token" (App. D), the reading stated at per_token_offsets
    subspace_iters: int = 0          # > 0: the Gram subspace iteration of App. H with this many steps (the paper runs 3) instead of the SVD


@dataclass
class HeadDiag:
    n_keep: int = 0
    r_keep: int = 0              # dim span(V_keep)
    k_used: int = 0              # residual principal directions used
    skipped: int = 1             # 1: V* = V_keep (no injection)
    a_keep: float = 0.0
    a_del: float = 0.0
    rcr: float = 0.0             # ||R||^2 / ||V_del||^2            (App. K.2)
    pcr: float = 0.0
    pc: float = 0.0              # projection cosine                 (App. K.2)
    revr: float = 0.0            # residual explained variance ratio (App. K.2)
    dr: float = 0.0              # demand ratio                      (App. K.2)
    fast_cond: float = 1.0       # subspace iteration only: worst first-norm / remaining-norm ratio met by the orth steps (test tolerances)
    fast_err: float = -1.0       # subspace iteration only: ||delta - delta_svd|| / ||delta_svd|| (App. H quotes ~1e-4)
    ivn: float = 0.0             # ||delta||                         (App. K.2)
    gap: float = np.inf          # sigma_k / sigma_{k+1} of R (subspace conditioning)
    keep_sigma_margin: float = np.inf   # min over sigma of |log10(sigma / rank threshold)|
    res_sigma_margin: float = np.inf
    res_sigma_rel: Optional[np.ndarray] = field(default=None, repr=False)   # sigma_i/sigma_1 of R, i < pca_rank
    res_thr_rel: float = 0.0            # rank threshold of R relative to sigma_1
    evr_margin: float = np.inf          # EVR-adaptive rank: distance of the nearest cumulative ratio from tau
    delta: Optional[np.ndarray] = field(default=None, repr=False)


def _margin(sigma: np.ndarray, rows: int, cols: int, first: Optional[int] = None) -> float:
    """Decades between the rank threshold and the nearest of the (first `first`) singular values."""
    if sigma.size == 0 or sigma[0] <= 0:
        return np.inf
    thr = sigma[0] * max(rows, cols) * RANK_EPS
    sel = sigma if first is None else sigma[:first]
    with np.errstate(divide="ignore"):
        m = np.abs(np.log10(np.maximum(sel, 1e-300) / thr))
    return float(m.min())


def inject(V_keep: np.ndarray, A_keep: np.ndarray, a_keep: float, delta: np.ndarray, variant: Variant) -> np.ndarray:
    """Eq. 7 (the same offset on every retained row), or the attention-weighted shares of App. D."""
    if variant.attn_inject:
        w = A_keep / (a_keep + EPS)
        return V_keep + V_keep.shape[0] * w[:, None] * delta[None, :]
    return V_keep + delta[None, :]


def per_token_offsets(R: np.ndarray, w: np.ndarray, C: np.ndarray, route_del: np.ndarray, B: int, scale: float) -> np.ndarray:
    """The "Per-token" alternative of App. D: one direction delta_t per retained slot t, "analogous to Eq. 6 but with per-t
    residual weighting".  The paper gives no formula; this is a READING (parity against the paper unpinned), built only
    from pieces the paper does define:
      * the deleted tokens are shared out among the retained slots by the routing rule of App. E (key cosine, first
        maximum): route_del[i] is the slot of deleted token i;
      * slot t's residual mean keeps Eq. 4's weights but only over its own tokens:  rbar_t = sum_{pi(j) = t} w_j R_j;
      * Eq. 5's projection onto the same subspace C and Eq. 6's demand ratio;
      * the factor B = |P_keep| that App. D's Attn-inject uses for its per-slot shares, so that the mean over the slots
        of delta_t is exactly the method's single delta (sum_t rbar_t = rbar).
    R [n_del, d] residuals, w [n_del] Eq. 4 weights, C [k, d], scale = a_del / (a_keep + eps) (1 under No Scaling).
    Returns delta [B, d]; a slot nothing was routed to gets zero."""
    d = R.shape[1]
    out = np.zeros((B, d))
    for i in range(R.shape[0]):                            # ascending token order; one term at a time
        out[route_del[i]] += w[i] * R[i]
    return B * scale * ((out @ C.T) @ C)


def backfill(V: np.ndarray, A: np.ndarray, idx: np.ndarray, rank: int, variant: Variant = Variant(), K: np.ndarray = None):
    """OBF for one head (Eq. 2-7, Alg. 3).  V [N, d] float64, A [N], idx ascending.  K [N, d] float64: only the Per-token
    alternative reads the keys (its routing).

    Returns (V_star [B, d] float64 before output rounding, HeadDiag).
    """
    N, d = V.shape
    idx = np.asarray(idx, dtype=np.int64)
    dele = complement(idx, N)
    V_keep = V[idx]
    diag = HeadDiag(n_keep=int(idx.size))
    diag.a_keep = float(A[idx].sum())
    diag.a_del = float(A[dele].sum())
    diag.dr = diag.a_del / (diag.a_keep + EPS)
    diag.delta = np.zeros(d)
    if rank <= 0 or dele.size == 0 or idx.size == 0:
        # rank 0 is the plain selector (App. G); empty P_del is skipped (Alg. 3)
        return V_keep.copy(), diag

    V_del = V[dele]
    if variant.naive:
        delta = V_del.mean(axis=0)
        diag.delta = delta
        diag.ivn = float(np.linalg.norm(delta))
        diag.skipped = 0
        return inject(V_keep, A[idx], diag.a_keep, delta, variant), diag
    if variant.no_projection:
        Q = np.zeros((d, 0))
    else:
        Q, s_keep = orth_rowspace(V_keep)                  # Eq. 2
        diag.keep_sigma_margin = _margin(s_keep, idx.size, d)
    diag.r_keep = Q.shape[1]
    if diag.r_keep == d:
        # retained span is all of R^d: the residual is identically zero
        diag.pcr = 1.0
        return V_keep.copy(), diag
    V_par = (V_del @ Q) @ Q.T
    R = V_del - V_par                                      # Eq. 3
    vd2 = float((V_del * V_del).sum())
    r2 = float((R * R).sum())
    diag.rcr = r2 / (vd2 + EPS)
    diag.pcr = float((V_par * V_par).sum()) / (vd2 + EPS)
    sd, sp = V_del.sum(axis=0), V_par.sum(axis=0)
    den = np.linalg.norm(sd) * np.linalg.norm(sp)
    diag.pc = float(sd @ sp / den) if den > 0 else 0.0
    if r2 <= RCR_SKIP * vd2:
        return V_keep.copy(), diag

    _, sR, VtR = np.linalg.svd(R, full_matrices=False)     # rows of VtR: right singular vectors
    rankR = numerical_rank(sR, R.shape[0], d)
    want = int(rank)
    if variant.subspace == "all":
        want = d
    elif variant.subspace == "evr":
        cum = np.cumsum(sR ** 2) / (sR ** 2).sum()
        want = int(np.argmax(cum >= variant.evr_tau)) + 1 if cum[-1] >= variant.evr_tau else sR.size
        diag.evr_margin = float(np.abs(cum - variant.evr_tau).min())
    elif variant.subspace != "rank":
        raise ValueError(variant.subspace)
    k = min(want, rankR)
    diag.res_sigma_margin = _margin(sR, R.shape[0], d, first=want)        # only these decide k
    diag.res_sigma_rel = sR[:want] / sR[0] if sR[0] > 0 else None
    diag.res_thr_rel = max(R.shape[0], d) * RANK_EPS
    if k == 0:
        return V_keep.copy(), diag
    C = VtR[:k]                                            # [k, d]
    diag.k_used = k
    diag.revr = float((sR[:k] ** 2).sum() / ((sR ** 2).sum() + EPS))
    if k < sR.size and sR[k] > 0:
        diag.gap = float(sR[k - 1] / sR[k])

    w = A[dele] / (diag.a_del + EPS)                       # Eq. 4
    rbar = w @ R
    Delta = (rbar @ C.T) @ C                               # Eq. 5
    if variant.subspace_iters > 0:
        # App. H: the same Delta from C_{t+1} = orth(C_t G), G = R^T R, instead of the SVD; the exact one above is
        # kept for the error report only
        info = {}
        Cf = subspace_iteration(R.T @ R, min(int(rank), d - diag.r_keep, dele.size), variant.subspace_iters, info)
        diag.fast_cond = info.get("cond", 1.0)
        Delta_f = (rbar @ Cf.T) @ Cf
        nd = float(np.linalg.norm(Delta))
        diag.fast_err = float(np.linalg.norm(Delta_f - Delta)) / nd if nd > 0 else 0.0
        Delta = Delta_f
        diag.k_used = Cf.shape[0]
        tr = float(np.trace(R.T @ R))
        diag.revr = float(sum(c @ (R.T @ (R @ c)) for c in Cf) / (tr + EPS))
        if diag.k_used == 0:
            diag.k_used, diag.revr = 0, 0.0
            return V_keep.copy(), diag
    delta = Delta if variant.no_scaling else diag.a_del / (diag.a_keep + EPS) * Delta       # Eq. 6
    diag.delta = delta
    diag.ivn = float(np.linalg.norm(delta))
    diag.skipped = 0
    if variant.per_token:
        if K is None:
            raise ValueError("the Per-token alternative routes by the keys")
        if variant.attn_inject or variant.subspace != "rank":
            raise ValueError("Per-token combines with No Projection, No Scaling and the fast path only")
        Cu = Cf if variant.subspace_iters > 0 else C
        route = merge_routes(K, idx)
        scale = 1.0 if variant.no_scaling else diag.a_del / (diag.a_keep + EPS)
        return V_keep + per_token_offsets(R, w, Cu, route[dele], idx.size, scale), diag    # delta (above) is their mean
    return inject(V_keep, A[idx], diag.a_keep, delta, variant), diag                         # Eq. 7


# ----------------------------------------------------------------------------- App. H: Gram subspace iteration
def start_rows(k: int, d: int) -> np.ndarray:
    """C_0 of App. H, which only asks for orthonormal rows.  Reading: the first k rows of the orthonormal cosine
    basis C_0[i, c] = sqrt(2/d) cos(pi/d (i + 1/2)(c + 1/2)) - fixed, dense, the same on every side."""
    i = np.arange(k, dtype=np.float64)[:, None] + 0.5
    c = np.arange(d, dtype=np.float64)[None, :] + 0.5
    return np.sqrt(2.0 / d) * np.cos(np.pi / d * i * c)


def orth_rows(Y: np.ndarray, info: dict = None) -> np.ndarray:
    """Thin QR of Y^T written as Gram-Schmidt on the rows (two passes); a row that is left with at most 1e-5 of the
    first row's norm depends on the rows before it and is dropped (reading: the QR of App. H is of full rank in the
    paper's setting; this keeps the rule k <= rank R of Sec. 4.4)."""
    rows = []
    first = None
    for y in Y:
        v = y.astype(np.float64).copy()
        for _ in range(2):
            for q in rows:
                v = v - (v @ q) * q
        n = float(np.linalg.norm(v))
        if first is None:
            first = n
        if first <= 0.0 or n <= 1e-5 * first:
            continue
        rows.append(v / n)
        if info is not None:     # how far the kept rows were from dependent: largest ratio first norm / norm left
            info["cond"] = max(info.get("cond", 1.0), first / n)
    return np.array(rows).reshape(len(rows), Y.shape[1])


def subspace_iteration(G: np.ndarray, k: int, iters: int, info: dict = None) -> np.ndarray:
    """C_{t+1} = orth(C_t G), t = 0 .. iters - 1, from C_0 = start_rows (App. H).  Returns C [k' <= k, d]."""
    C = start_rows(k, G.shape[0])
    for _ in range(iters):
        C = orth_rows(C @ G, info)
        if C.shape[0] == 0:
            break
    return C


# ----------------------------------------------------------------------------- one head, whole relay
@dataclass
class HeadResult:
    A: np.ndarray
    idx: np.ndarray
    K_keep: np.ndarray        # I/O dtype (bit copy of the selected rows)
    V_out: np.ndarray         # I/O dtype (rounded V*)
    V_star: np.ndarray        # float64 V* before rounding
    diag: HeadDiag


def compress_head(K_io: np.ndarray, V_io: np.ndarray, Q_io: np.ndarray, budget: int, rank: int,
                  dtype: str, variant: Variant = Variant(), sink: int = 0) -> HeadResult:
    """score -> TopK_B -> gather -> OBF for one (layer, KV head).

    K_io, V_io [N, d]; Q_io [group, window, d] (or [rows, d]); all in the I/O dtype.
    sink: the first `sink` tokens are the shared attention sink (Sec. 4.3.2: not in Omega).
    """
    K = decode(K_io, dtype)
    V = decode(V_io, dtype)
    Qr = decode(Q_io, dtype).reshape(-1, K.shape[1])
    A = attention_mass(K, Qr)                               # the sink tokens are keys like any other
    idx = sink + select_topk(A[sink:], budget)              # TopK_B over Omega
    V_star, diag = backfill(V[sink:], A[sink:], idx - sink, rank, variant, K[sink:] if variant.per_token else None)
    if diag.skipped:
        V_out = np.asarray(V_io)[idx].copy()               # identity: a bit copy, not a re-rounding
    else:
        V_out = round_to_io(V_star, dtype)
    return HeadResult(A=A, idx=idx, K_keep=np.asarray(K_io)[idx].copy(), V_out=V_out, V_star=V_star, diag=diag)


def compress_relay(K_io: np.ndarray, V_io: np.ndarray, Q_io: np.ndarray, budgets: np.ndarray, rank: int,
                   group: int, dtype: str, heads=None, variant: Variant = Variant()):
    """All (layer, KV head) pairs of a cache in the canonical layout.

    K_io, V_io [L, H, N, d]; Q_io [L, H*group, W, d]; budgets int [L, H].
    Returns {(l, h): HeadResult}.
    """
    L, H = K_io.shape[:2]
    out = {}
    todo = heads if heads is not None else [(l, h) for l in range(L) for h in range(H)]
    for (l, h) in todo:
        out[(l, h)] = compress_head(K_io[l, h], V_io[l, h], Q_io[l, h * group:(h + 1) * group],
                                    int(budgets[l, h]), rank, dtype, variant)
    return out


# ----------------------------------------------------------------------------- layerwise selector (Sec. 4.3.2)
def compress_layer(K_io: np.ndarray, V_io: np.ndarray, Q_io: np.ndarray, budget: int, rank: int,
                   group: int, dtype: str, variant: Variant = Variant(), sink: int = 0):
    """Layerwise granularity of the retention rule (Sec. 4.3.2; the "L" and "L-OBF" methods of Sec. 5):
    one index set per layer, TopK_B of the attention mass summed over the layer's heads, shared by
    all of them; Orthogonal BackFill then runs per head exactly as in the headwise case, with that
    head's own attention mass in Eq. 4 and Eq. 6 and the shared index set.

    K_io, V_io [H, N, d]; Q_io [H*group, W, d].  Returns (idx, [HeadResult per head]).
    Reading: Eq. 1 is stated per attention head and the sum of the retention rule runs over all
    heads of the layer; with grouped queries the per-KV-head mass already is the sum over the
    group's query heads, so the layer sum is the sum of the per-KV-head masses.
    """
    H = K_io.shape[0]
    d = K_io.shape[2]
    masses = []
    for h in range(H):
        K = decode(K_io[h], dtype)
        Qr = decode(Q_io[h * group:(h + 1) * group], dtype).reshape(-1, d)
        masses.append(attention_mass(K, Qr))
    layer_mass = np.zeros_like(masses[0])
    for A in masses:                                        # plain left-to-right sum over the heads
        layer_mass = layer_mass + A
    idx = sink + select_topk(layer_mass[sink:], budget)    # Omega leaves out the shared sink (Sec. 4.3.2)
    heads = []
    for h in range(H):
        V = decode(V_io[h], dtype)
        V_star, diag = backfill(V[sink:], masses[h][sink:], idx - sink, rank, variant,
                                decode(K_io[h], dtype)[sink:] if variant.per_token else None)
        if diag.skipped:
            V_out = np.asarray(V_io[h])[idx].copy()
        else:
            V_out = round_to_io(V_star, dtype)
        heads.append(HeadResult(A=masses[h], idx=idx, K_keep=np.asarray(K_io[h])[idx].copy(), V_out=V_out,
                                V_star=V_star, diag=diag))
    return idx, heads


# ----------------------------------------------------------------------------- message of Sec. 3.3
def append_message(prev: np.ndarray, keep: np.ndarray, gen: np.ndarray) -> np.ndarray:
    """M_i = [M_{i-1}; Phi(P; G); G] for one (layer, KV head) and one of K / V: rows of the inherited message,
    then the retained prompt rows, then the rows of the reasoning states, each [rows, d] in the I/O dtype."""
    return np.concatenate([prev, keep, gen], axis=0)


# ----------------------------------------------------------------------------- cache-merging operator (App. E)
def merge_routes(K: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """Step (ii) of App. E: every deleted position j is routed to the retained slot whose key has the highest
    cosine similarity with K_j.  K [N, d] float64, idx ascending.  Returns route [N] int64: the slot number
    (position in idx) for deleted tokens, -1 for retained ones.
    Readings: the first maximum wins (lowest slot); a key of zero norm has cosine 0 with everything."""
    N = K.shape[0]
    idx = np.asarray(idx, dtype=np.int64)
    route = np.full(N, -1, dtype=np.int64)
    dele = complement(idx, N)
    if dele.size == 0 or idx.size == 0:
        return route
    norms = np.sqrt((K * K).sum(axis=1))
    inv = np.where(norms > 0, 1.0 / np.where(norms > 0, norms, 1.0), 0.0)
    cos = (K[dele] @ K[idx].T) * inv[dele][:, None] * inv[idx][None, :]
    route[dele] = np.argmax(cos, axis=1)
    return route


def merge_values(V: np.ndarray, A: np.ndarray, idx: np.ndarray, route: np.ndarray) -> np.ndarray:
    """Step (iii) of App. E: V*_t = V_t + sum over the deleted j routed to t of A_j / (A_t + eps) V_j."""
    idx = np.asarray(idx, dtype=np.int64)
    V_star = V[idx].copy()
    for j in np.nonzero(route >= 0)[0]:                     # ascending j; one term at a time
        t = route[j]
        V_star[t] += A[j] / (A[idx[t]] + EPS) * V[j]
    return V_star


@dataclass
class MergeResult:
    A: np.ndarray
    idx: np.ndarray
    route: np.ndarray         # [N]: retained slot of every deleted token, -1 for retained tokens
    cos_gap: np.ndarray       # [N]: best minus second-best cosine of every deleted token (inf with one slot; checker's tie allowance)
    K_keep: np.ndarray        # I/O dtype
    V_out: np.ndarray         # I/O dtype (rounded V*; a bit copy where nothing was routed to the slot)
    V_star: np.ndarray        # float64


def merge_head(K_io: np.ndarray, V_io: np.ndarray, Q_io: np.ndarray, budget: int, dtype: str) -> MergeResult:
    """The cache-merging comparison system of App. E for one (layer, KV head): (i) the same TopK_B selector,
    (ii) routing by key cosine similarity, (iii) attention-weighted merge of the deleted values; keys unchanged."""
    K = decode(K_io, dtype)
    V = decode(V_io, dtype)
    Qr = decode(Q_io, dtype).reshape(-1, K.shape[1])
    A = attention_mass(K, Qr)
    idx = select_topk(A, budget)
    route = merge_routes(K, idx)
    V_star = merge_values(V, A, idx, route)
    gap = np.full(K.shape[0], np.inf)
    dele = np.nonzero(route >= 0)[0]
    if dele.size and idx.size > 1:
        norms = np.sqrt((K * K).sum(axis=1))
        inv = np.where(norms > 0, 1.0 / np.where(norms > 0, norms, 1.0), 0.0)
        cos = (K[dele] @ K[idx].T) * inv[dele][:, None] * inv[idx][None, :]
        top2 = np.partition(cos, -2, axis=1)[:, -2:]
        gap[dele] = top2[:, 1] - top2[:, 0]
    V_out = np.asarray(V_io)[idx].copy()
    touched = np.zeros(idx.size, dtype=bool)
    touched[route[dele]] = True
    V_out[touched] = round_to_io(V_star[touched], dtype)
    return MergeResult(A=A, idx=idx, route=route, cos_gap=gap, K_keep=np.asarray(K_io)[idx].copy(), V_out=V_out, V_star=V_star)


# ----------------------------------------------------------------------------- stacked int8 / int4 relay (App. E)
def quantize_rows(X_io: np.ndarray, dtype: str, bits: int):
    """Post-hoc quantisation of relay rows (App. E stacks int8 on the compressed relay; the paper fixes no scheme).
    Reading, chosen because it reproduces the table's ratios (16 d / (8 d + 32) = 1.94 and 16 d / (4 d + 32) = 3.76 at
    d = 128): every row gets its own asymmetric code with two half-precision numbers,
        zero = fp16(min x), scale = fp16((max x - min x) / L), L = 2^bits - 1,
        q_c = clamp(rint((x_c - zero) / scale), 0, L)   (0 when scale is 0),
    the arithmetic that decides the integer codes being single precision (subtract, divide, round to nearest even), the
    precision the device takes the same decision in.  X_io [rows, d] in the I/O dtype.
    Returns (codes uint8 [rows, d], scale float16 [rows], zero float16 [rows]); parity of the scheme itself is unpinned
    by the paper."""
    if bits not in (4, 8):
        raise ValueError(bits)
    L = np.float32(2 ** bits - 1)
    X = decode(X_io, dtype).astype(np.float32)              # exact: bf16 and fp32 values are fp32 values
    lo, hi = X.min(axis=1), X.max(axis=1)
    zero = lo.astype(np.float16)
    scale = ((hi - lo) / L).astype(np.float16)
    z32, s32 = zero.astype(np.float32), scale.astype(np.float32)
    with np.errstate(divide="ignore", invalid="ignore"):
        q = np.rint((X - z32[:, None]) / s32[:, None])
    q = np.where(s32[:, None] > 0, np.clip(q, 0, L), 0)
    return q.astype(np.uint8), scale, zero


def dequantize_rows(codes: np.ndarray, scale: np.ndarray, zero: np.ndarray) -> np.ndarray:
    """x_hat = zero + scale * q in float64 (exact for these operand widths up to one rounding)."""
    return zero.astype(np.float64)[:, None] + scale.astype(np.float64)[:, None] * codes.astype(np.float64)


# ----------------------------------------------------------------------------- App. H route (used by pins and as a second CPU timing)
def top_subspace_gram(R: np.ndarray, k: int) -> np.ndarray:
    """Top-k right singular vectors of R from the d x d Gram matrix R^T R (App. H)."""
    G = R.T @ R
    w, U = np.linalg.eigh(G)
    order = np.argsort(-w, kind="stable")[:k]
    return U[:, order].T
