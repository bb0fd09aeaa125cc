"""Acceptance rules for GPU-vs-oracle comparison of one head (used by the -m gpu tests).

  * n_keep equals the budget; idx ascending, tail -1.
  * idx bit-exact; a differing pair (i only on the GPU, j only in the oracle) is tolerated only if
    the oracle's exact scores satisfy |A_i - A_j| < 1e-6 * max(A_i, A_j).
  * K_out is a bit copy of K[idx]; padded rows are zero.
  * V_out (heads whose index sets agree): bit copy of V[idx] where the oracle skips OBF; otherwise
    the injected vector must satisfy ||delta_gpu - delta|| <= 2e-3 * g * ||delta|| (g: eigen-gap factor
    max(1, 0.05 / (1 - (sigma_{k+1}/sigma_k)^2)), the rank-k subspace is ill-defined when the gap
    closes), and the stored values, against the oracle's UNROUNDED V*, must satisfy
        |gpu - V*| <= half an ulp of the I/O dtype at V*  +  2e-3 * g * max|delta|      (bf16 I/O)
        |gpu - V*| <= 1e-4 * max(|V*|, rms(V_keep))                                     (fp32 I/O).
    bf16 keeps 8 significant bits, so rounding alone moves a value by up to 2^-8 = 3.9e-3 of itself:
    a flat 2e-3 relative bound on the rounded output cannot be met by any implementation (the
    oracle's own rounded output misses it); the bound therefore applies to what the fp32
    arithmetic controls, and the stored value must be the nearest bf16 to it.  Elements where GPU
    and oracle round to different bf16 neighbours must be rare (< 0.5 %) and one ulp apart.
  * diag.skipped / r_keep / k_used equal the oracle's unless a singular value that decides them sits
    within a decade of the rank threshold, or (rank of R only) between that threshold and the
    1e-3 resolution of the device's fp32 Gram matrix; either answer is then valid.
"""
from __future__ import annotations

import numpy as np

from oracle import obf_oracle as O

SWAP_REL = 1e-6
TOL = {"bf16": 2e-3, "f32": 1e-4}
AMBIG_DECADES_KEEP = 1.0
AMBIG_DECADES_RES = 1.0
GPU_RES_FLOOR = 1e-3      # the device decides rank(R) on an fp32 Gram matrix: sigma resolution ~1e-3 sigma_max


class HeadReport:
    def __init__(self):
        self.swaps = 0
        self.v_checked = False
        self.v_err = 0.0
        self.delta_err = 0.0
        self.ambiguous = False
        self.skipped = None
        self.r_keep = None


def _exact_gap_factor(diag) -> float:
    if not np.isfinite(diag.gap) or diag.gap <= 0:
        return 1.0
    return max(1.0, 0.05 / max(1.0 - 1.0 / (diag.gap * diag.gap), 1e-12))


def gap_factor(diag) -> float:
    if diag.fast_err >= 0.0:
        # the subspace iteration (App. H) does not resolve single directions: what amplifies rounding there is how close
        # to dependent the rows were that its orth steps had to separate
        return max(1.0, diag.fast_cond / 50.0)
    if not np.isfinite(diag.gap) or diag.gap <= 0:
        return 1.0
    ratio2 = 1.0 / (diag.gap * diag.gap)
    den = 1.0 - ratio2
    return max(1.0, 0.05 / max(den, 1e-12))


def check_head(tag, ref: O.HeadResult, K_io, V_io, dtype, budget, gpu_idx, gpu_n_keep, gpu_K, gpu_V,
               gpu_diag=None, gpu_delta=None, gpu_scores=None, variant=None, sink=0) -> HeadReport:
    """variant: the oracle's Variant the reference was computed with (None: the method itself); sink: protected
    leading tokens (the eligible set starts behind them)."""
    rep = HeadReport()
    N, d = K_io.shape
    B = min(int(budget), N - sink)
    maxb = gpu_idx.shape[0]
    assert int(gpu_n_keep) == B, f"{tag}: n_keep {gpu_n_keep} != budget {B}"
    gi = np.asarray(gpu_idx[:B], dtype=np.int64)
    assert np.all(gpu_idx[B:] == -1), f"{tag}: idx tail is not -1"
    if B > 0:
        assert gi.min() >= sink and gi.max() < N, f"{tag}: idx out of range"
        assert np.all(np.diff(gi) > 0), f"{tag}: idx not strictly ascending"
    # gather is a bit copy of whatever the GPU selected
    assert np.array_equal(gpu_K[:B], K_io[gi]), f"{tag}: K_out is not a bit copy of K[idx]"
    assert not gpu_K[B:].any() and not gpu_V[B:].any(), f"{tag}: padded rows not zero"
    if gpu_scores is not None:
        rel = np.abs(gpu_scores.astype(np.float64) - ref.A) / np.maximum(ref.A, 1e-300)
        assert rel.max() < 5e-5, f"{tag}: scores off by {rel.max():.2e}"
    same = np.array_equal(gi, ref.idx)
    if not same:
        only_g = sorted(set(gi.tolist()) - set(ref.idx.tolist()), key=lambda j: -ref.A[j])
        only_r = sorted(set(ref.idx.tolist()) - set(gi.tolist()), key=lambda j: -ref.A[j])
        assert len(only_g) == len(only_r)
        for a, b in zip(only_g, only_r):
            big = max(ref.A[a], ref.A[b])
            assert abs(ref.A[a] - ref.A[b]) < SWAP_REL * big, (
                f"{tag}: index sets differ beyond the tie allowance: gpu-only {a} (A={ref.A[a]:.9e}) vs "
                f"oracle-only {b} (A={ref.A[b]:.9e})")
        rep.swaps = len(only_g)
        assert np.array_equal(gpu_V[:B], V_io[gi]) or gpu_diag is None or not gpu_diag["skipped"], f"{tag}: V_out"
        return rep
    assert np.array_equal(gpu_K[:B], ref.K_keep)
    dg = ref.diag
    rep.ambiguous = (dg.keep_sigma_margin < AMBIG_DECADES_KEEP) or (dg.res_sigma_margin < AMBIG_DECADES_RES)
    if dg.res_sigma_rel is not None and dg.res_thr_rel < GPU_RES_FLOOR:
        # singular values of R between the oracle's threshold and the device's resolution floor
        rel = dg.res_sigma_rel
        rep.ambiguous |= bool(np.any((rel > dg.res_thr_rel / 10) & (rel < GPU_RES_FLOOR * 10)))
    if variant is not None and variant.subspace == "evr":
        rep.ambiguous |= dg.evr_margin < 1e-4               # a cumulative ratio within fp32 Gram noise of tau
    rep.skipped = dg.skipped
    rep.r_keep = dg.r_keep
    # largest multiple of delta any row receives (1 for Eq. 7; the attention-weighted shares of App. D can exceed it)
    inj = 1.0
    if variant is not None and variant.attn_inject and B > 0:
        inj = max(1.0, float(B * ref.A[gi].max() / (dg.a_keep + O.EPS)))
    span_free = variant is not None and (variant.no_projection or variant.naive)
    if gpu_diag is not None and not rep.ambiguous:
        assert int(gpu_diag["skipped"]) == dg.skipped, f"{tag}: skipped {gpu_diag['skipped']} vs oracle {dg.skipped}"
        if dg.r_keep > 0:
            assert int(gpu_diag["r_keep"]) == dg.r_keep, f"{tag}: r_keep {gpu_diag['r_keep']} vs {dg.r_keep}"
        assert int(gpu_diag["k_used"]) == dg.k_used, f"{tag}: k_used {gpu_diag['k_used']} vs {dg.k_used}"
    if gpu_diag is not None:
        assert abs(float(gpu_diag["a_keep"]) - dg.a_keep) <= 1e-4 * max(dg.a_keep, 1e-30) + 1e-30
        assert abs(float(gpu_diag["a_del"]) - dg.a_del) <= 1e-4 * max(dg.a_del, 1e-30) + 1e-7 * dg.a_keep
        if "dr" in gpu_diag.dtype.names:
            # the remaining App. K.2 diagnostics (fp32 Gram arithmetic on the device: 1e-4 absolute on the ratios)
            assert abs(float(gpu_diag["dr"]) - dg.dr) <= 2e-4 * dg.dr + 1e-7, f"{tag}: DR {gpu_diag['dr']} vs {dg.dr}"
            if not rep.ambiguous:
                assert abs(float(gpu_diag["pcr"]) - dg.pcr) <= 2e-4, f"{tag}: PCR {gpu_diag['pcr']} vs {dg.pcr}"
                assert abs(float(gpu_diag["rcr"]) - dg.rcr) <= 2e-4, f"{tag}: RCR {gpu_diag['rcr']} vs {dg.rcr}"
                assert abs(float(gpu_diag["pc"]) - abs(dg.pc)) <= 1e-3, f"{tag}: PC {gpu_diag['pc']} vs {dg.pc}"
                assert abs(float(gpu_diag["revr"]) - dg.revr) <= 1e-3, f"{tag}: REVR {gpu_diag['revr']} vs {dg.revr}"
                if "fast_err" in gpu_diag.dtype.names:
                    fe = float(gpu_diag["fast_err"])
                    if dg.fast_err < 0:
                        assert fe == -1.0, f"{tag}: fast_err {fe} on a head without the fast path"
                    else:
                        # both directions' single-precision errors, relative to the exact Delta
                        tol = 2e-3 * (gap_factor(dg) + _exact_gap_factor(dg)) * (1.0 + dg.fast_err)
                        assert abs(fe - dg.fast_err) <= tol, f"{tag}: fast_err {fe} vs {dg.fast_err}"
                assert abs(float(gpu_diag["ivn"]) - dg.ivn) <= 2e-3 * gap_factor(dg) * dg.ivn + 1e-6 * max(dg.ivn, 1e-3), (
                    f"{tag}: IVN {gpu_diag['ivn']} vs {dg.ivn}")
    if dg.skipped and not rep.ambiguous:
        assert np.array_equal(gpu_V[:B], V_io[gi]), f"{tag}: OBF skipped but V_out is not a bit copy"
        if gpu_delta is not None:
            assert not np.any(gpu_delta), f"{tag}: delta must be zero when skipped"
        rep.v_checked = True
        return rep
    if rep.ambiguous:
        return rep
    Vk = O.decode(V_io[gi], dtype)
    rms = float(np.sqrt((Vk * Vk).mean()))
    got = O.decode(gpu_V[:B], dtype)
    g = gap_factor(dg)
    abs_err = np.abs(got - ref.V_star)
    if dtype == "bf16":
        mag = np.maximum(np.abs(ref.V_star), np.abs(got))
        half_ulp = np.where(mag > 0, 2.0 ** (np.floor(np.log2(np.maximum(mag, 1e-300))) - 8.0), 0.0)
        bound = half_ulp * (1.0 + 1e-6) + 2e-3 * g * inj * np.abs(dg.delta).max()
        rep.v_err = float((abs_err / np.maximum(bound, 1e-300)).max())
        assert rep.v_err <= 1.0, f"{tag}: V_out off by {rep.v_err:.3f} x (half ulp + delta tolerance)"
        diff = gpu_V[:B] != ref.V_out
        frac = float(diff.mean())
        # an element rounds differently when the two sums straddle a bf16 boundary: a share of about (error of delta) /
        # (spacing of the sum) of them, which only matters where delta dominates the sum
        derr = 0.0 if gpu_delta is None else float(np.abs(gpu_delta.astype(np.float64) - dg.delta).max())
        crowd = float(np.mean(derr * inj / np.maximum(2.0 * half_ulp, 1e-300)))
        assert frac < 5e-3 + 4.0 * crowd, f"{tag}: {frac:.2%} of V_out elements round differently from the oracle"
        if diff.any():
            step = np.abs(got - O.decode(ref.V_out, dtype))
            assert np.all(step <= 2.0 * half_ulp * (1.0 + 1e-6) + 2e-3 * g * inj * np.abs(dg.delta).max()), (
                f"{tag}: V_out differs from the oracle's rounded value by more than one bf16 ulp")
    else:
        err = abs_err / np.maximum(np.abs(ref.V_star), rms)
        rep.v_err = float(err.max())
        assert rep.v_err <= TOL[dtype] * g * inj, f"{tag}: V_out max rel err {rep.v_err:.3e} > {TOL[dtype] * g * inj:.3e}"
    if gpu_delta is not None:
        dn = np.linalg.norm(dg.delta)
        rep.delta_err = float(np.linalg.norm(gpu_delta.astype(np.float64) - dg.delta) / max(dn, 1e-300))
        assert rep.delta_err <= 2e-3 * gap_factor(dg) + 1e-6 * rms / max(dn, 1e-300), (
            f"{tag}: delta rel err {rep.delta_err:.3e} (gap factor {gap_factor(dg):.2f})")
        # orthogonality of the injected vector to the retained values (Eq. 3; not for variants that skip Eq. 3)
        orth = 0.0 if span_free else np.abs(Vk @ gpu_delta.astype(np.float64)).max()
        assert orth <= 2e-5 * np.linalg.norm(Vk, axis=1).max() * max(np.linalg.norm(gpu_delta), 1e-300) + 1e-30, (
            f"{tag}: delta not orthogonal to retained values ({orth:.3e})")
    rep.v_checked = True
    return rep
