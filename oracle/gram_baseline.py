"""A second CPU baseline for the benchmark: the Gram-matrix route of App. H in single precision.

THIS IS TEST / BENCHMARK INFRASTRUCTURE, like the oracle beside it: only tests and the benchmark's
cpu_baseline leg may import it; the product path never does, and it shares no code with the HIP path.

The oracle (obf_oracle.py) takes the paper's main-text route: exact SVDs in float64.  App. H observes
that the top right singular vectors of the residual R are the top eigenvectors of the d x d matrix
R^T R, so that the O(N d min(N, d)) decomposition can be replaced by one N x d x d product and a small
symmetric eigenproblem.  This module is that route, run to convergence by LAPACK (not the 3-step
iteration), in float32, so that the CPU number printed next to the GPU's is not only the slow exact one:
  * Eq. 1 in float32 (one matmul, max-subtracted softmax);
  * TopK_B exactly as the oracle (stable order, ascending list);
  * Eq. 2 by the reduced QR it names (the rank rule read off the triangular factor's singular values; an
    SVD only when rows turn out dependent);
  * Eq. 3 never forms R: R^T R = P (V_del^T V_del) P with P = I - Q Q^T, and sum_j w_j R_j = P sum_j w_j V_j;
  * Eq. 4-7 as printed.
It is pinned to the oracle in tests/test_oracle_pins.py (same index set, delta within single-precision
Gram accuracy on well-separated spectra); it is NOT a parity reference for the GPU.
"""
from __future__ import annotations

import numpy as np

from . import obf_oracle as O


def compress_head_gram32(K_io, V_io, Q_io, budget: int, rank: int, dtype: str):
    """Returns (idx ascending int64, V_star float32 [B, d], delta float32 [d], skipped int)."""
    f = np.float32
    K = O.decode(K_io, dtype).astype(f)
    V = O.decode(V_io, dtype).astype(f)
    Q = O.decode(Q_io, dtype).astype(f).reshape(-1, K.shape[1])
    N, d = V.shape
    S = (Q @ K.T) * f(1.0 / np.sqrt(d))                     # Eq. 1
    S -= S.max(axis=1, keepdims=True)
    np.exp(S, out=S)
    S /= S.sum(axis=1, keepdims=True)
    A = S.sum(axis=0)
    idx = O.select_topk(A, budget)                          # TopK_B (Sec. 4.3.2)
    dele = O.complement(idx, N)
    Vk, Vd = V[idx], V[dele]
    zero = np.zeros(d, dtype=f)
    if rank <= 0 or dele.size == 0 or idx.size == 0:
        return idx, Vk, zero, 1
    Qb, Rf = np.linalg.qr(Vk.T)                             # Eq. 2 as printed: reduced QR of V_keep^T
    sv = np.linalg.svd(Rf, compute_uv=False)                # the triangular factor has V_keep's singular values
    r = int(np.count_nonzero(sv > sv[0] * max(idx.size, d) * O.RANK_EPS))
    if r < Qb.shape[1]:                                     # dependent rows: take the numerical row space instead
        _, _, Vt = np.linalg.svd(Vk, full_matrices=False)
        Qb = Vt[:r].T
    if r == d:
        return idx, Vk, zero, 1
    P = np.eye(d, dtype=f) - Qb @ Qb.T
    Gd = Vd.T @ Vd
    GR = P @ Gd @ P                                         # R^T R (Eq. 3, App. H)
    if np.trace(GR) <= O.RCR_SKIP * np.trace(Gd):
        return idx, Vk, zero, 1
    mu, W = np.linalg.eigh(GR)
    mu, W = mu[::-1], W[:, ::-1]
    floor = mu[0] * max((max(dele.size, d) * O.RANK_EPS) ** 2, 1e-6)   # single-precision Gram: nothing below 1e-3 sigma_1 is resolved
    k = int(min(rank, np.count_nonzero(mu > floor)))
    if k == 0:
        return idx, Vk, zero, 1
    C = W[:, :k].T
    a_keep, a_del = float(A[idx].sum(dtype=np.float64)), float(A[dele].sum(dtype=np.float64))
    rbar = P @ (Vd.T @ (A[dele] / f(a_del + O.EPS)))        # Eq. 4
    Delta = (rbar @ C.T) @ C                                # Eq. 5
    delta = (f(a_del / (a_keep + O.EPS)) * Delta).astype(f)  # Eq. 6
    return idx, Vk + delta[None, :], delta, 0               # Eq. 7
