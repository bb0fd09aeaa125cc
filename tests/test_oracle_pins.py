"""Pins for the CPU oracle: closed forms, brute force, invariants and special
cases fixed by the paper or by the mathematics, none of which re-use the
oracle's own formulas.  A dropped term, wrong sign, wrong axis or transposed
operand in oracle/obf_oracle.py fails at least one of these."""
import itertools
import math

import numpy as np
import pytest
from scipy.special import logsumexp

from oracle import obf_oracle as O


def rng(seed):
    return np.random.default_rng(seed)


# --------------------------------------------------------------------------- S1: Eq. 1
def test_mass_sums_to_number_of_query_rows():
    r = rng(1)
    K = r.standard_normal((300, 64)); Q = r.standard_normal((24, 64))
    A = O.attention_mass(K, Q)
    assert A.shape == (300,)
    assert abs(A.sum() - 24.0) < 1e-11          # each softmax row sums to one over the tokens


def test_zero_queries_give_uniform_mass():
    K = rng(2).standard_normal((50, 64))
    A = O.attention_mass(K, np.zeros((6, 64)))
    assert np.allclose(A, 6.0 / 50.0, rtol=0, atol=1e-15)


def test_rank_one_keys_closed_form_pins_scale_and_axis():
    # k_j = c_j u, q = u  =>  logits c_j |u|^2 / sqrt(d); A_j = exp(.) / sum exp(.)
    r = rng(3)
    d, N = 64, 40
    u = r.standard_normal(d)
    c = r.standard_normal(N)
    K = c[:, None] * u[None, :]
    A = O.attention_mass(K, u[None, :])
    z = c * (u @ u) / math.sqrt(d)
    ref = np.exp(z - z.max()); ref /= ref.sum()
    assert np.allclose(A, ref, rtol=1e-12, atol=0)
    # a wrong scale (1/d, or none) would not match
    bad = np.exp(c * (u @ u) / d); bad /= bad.sum()
    assert not np.allclose(A, bad, rtol=1e-3)


def test_mass_matches_independent_logsumexp_formulation_loopwise():
    r = rng(4)
    N, d, R = 37, 64, 5
    K = r.standard_normal((N, d)) * 3.0; Q = r.standard_normal((R, d)) * 3.0
    A = O.attention_mass(K, Q)
    ref = np.zeros(N)
    for t in range(R):
        s = np.array([sum(Q[t, c] * K[j, c] for c in range(d)) for j in range(N)]) / math.sqrt(d)
        ref += np.exp(s - logsumexp(s))
    assert np.allclose(A, ref, rtol=1e-11, atol=1e-300)


def test_mass_survives_huge_logits():
    K = np.zeros((4, 64)); K[0, 0] = 1e4; K[1, 0] = 1e4 - 8.0 * math.log(3.0)
    q = np.zeros((1, 64)); q[0, 0] = 1.0
    A = O.attention_mass(K, q)           # logits differ by log 3 after the 1/8 scale
    assert np.all(np.isfinite(A)) and abs(A[0] / A[1] - 3.0) < 1e-9


# --------------------------------------------------------------------------- S2: TopK_B
@pytest.mark.parametrize("seed", range(6))
def test_topk_brute_force_tiny(seed):
    r = rng(100 + seed)
    N = int(r.integers(5, 12)); B = int(r.integers(1, N))
    A = r.random(N)
    idx = O.select_topk(A, B)
    assert len(idx) == B and np.all(np.diff(idx) > 0)
    best = max(itertools.combinations(range(N), B), key=lambda s: A[list(s)].sum())
    assert tuple(idx) == best


def test_topk_all_ties_keeps_lowest_indices():
    idx = O.select_topk(np.full(20, 0.25), 7)
    assert idx.tolist() == list(range(7))


def test_topk_partial_ties_lowest_index_wins():
    A = np.array([1.0, 5.0, 2.0, 2.0, 9.0, 2.0, 0.5])
    assert O.select_topk(A, 3).tolist() == [1, 2, 4]      # of the three 2.0s only index 2 fits
    assert O.select_topk(A, 4).tolist() == [1, 2, 3, 4]


def test_topk_budget_edges():
    A = rng(5).random(9)
    assert O.select_topk(A, 0).size == 0
    assert O.select_topk(A, 9).tolist() == list(range(9))
    assert O.select_topk(A, 50).tolist() == list(range(9))


def test_topk_permutation_equivariance():
    r = rng(6)
    A = r.random(64)
    perm = r.permutation(64)
    idx = O.select_topk(A, 10)
    idx_p = O.select_topk(A[perm], 10)
    assert sorted(perm[idx_p].tolist()) == idx.tolist()


# --------------------------------------------------------------------------- S3 + dtype plumbing
def test_bf16_decode_and_round_roundtrip_all_finite_patterns():
    bits = np.arange(0, 1 << 16, dtype=np.uint32).astype(np.uint16)
    exp = (bits >> 7) & 0xFF
    finite = bits[exp != 0xFF]
    x = O.decode(finite, "bf16")
    assert np.array_equal(O.round_to_io(x, "bf16"), finite)
    # 1.0 = 0x3F80, -2.0 = 0xC000, 0.15625 = 0x3E20
    assert O.decode(np.array([0x3F80, 0xC000, 0x3E20], np.uint16), "bf16").tolist() == [1.0, -2.0, 0.15625]


def test_bf16_rounding_is_nearest_even():
    # 1 + 2^-8 is halfway between 1.0 (even mantissa) and 1 + 2^-7: ties to even -> 1.0
    assert O.round_to_io(np.array([1.0 + 2.0 ** -8]), "bf16")[0] == 0x3F80
    assert O.round_to_io(np.array([1.0 + 2.0 ** -8 + 2.0 ** -12]), "bf16")[0] == 0x3F81
    assert O.round_to_io(np.array([1.0 + 3 * 2.0 ** -8]), "bf16")[0] == 0x3F82   # tie -> even (0x82)


def test_gather_is_bit_copy():
    r = rng(7)
    K = r.integers(0, 1 << 16, size=(64, 64)).astype(np.uint16)
    K[(K >> 7) & 0xFF == 0xFF] = 0
    V = K[::-1].copy()
    Q = O.round_to_io(r.standard_normal((2, 4, 64)), "bf16")
    res = O.compress_head(K, V, Q, 9, 0, "bf16")
    assert np.array_equal(res.K_keep, K[res.idx]) and np.array_equal(res.V_out, V[res.idx])


# --------------------------------------------------------------------------- S4-S5: Eq. 2-3
def test_orth_is_orthonormal_basis_of_retained_span():
    V = rng(8).standard_normal((20, 64))
    Q, _ = O.orth_rowspace(V)
    assert Q.shape == (64, 20)
    assert np.allclose(Q.T @ Q, np.eye(20), atol=1e-12)
    assert np.allclose(V - (V @ Q) @ Q.T, 0, atol=1e-11)
    # same projector as the pseudo-inverse route
    assert np.allclose(Q @ Q.T, np.linalg.pinv(V) @ V, atol=1e-10)


def test_orth_drops_dependent_rows():
    r = rng(9)
    base = r.standard_normal((5, 64))
    V = np.vstack([base, base[0] + base[1], 2.0 * base[3]])
    Q, _ = O.orth_rowspace(V)
    assert Q.shape[1] == 5


def test_pcr_plus_rcr_is_one_and_residual_orthogonal():
    r = rng(10)
    V = r.standard_normal((200, 64)); A = r.random(200)
    idx = O.select_topk(A, 24)
    _, dg = O.backfill(V, A, idx, 4)
    assert abs(dg.pcr + dg.rcr - 1.0) < 1e-12
    assert dg.r_keep == 24 and dg.k_used == 4 and dg.skipped == 0


def test_full_rank_retained_span_makes_backfill_identity():
    r = rng(11)
    V = r.standard_normal((300, 64)); A = r.random(300)
    idx = O.select_topk(A, 64)                       # B = d, generic => span = R^d
    Vs, dg = O.backfill(V, A, idx, 4)
    assert dg.skipped == 1 and dg.r_keep == 64 and np.array_equal(Vs, V[idx])
    idx = O.select_topk(A, 100)                      # B > d
    Vs, dg = O.backfill(V, A, idx, 4)
    assert dg.skipped == 1 and np.array_equal(Vs, V[idx])


def test_deleted_rows_inside_retained_span_are_skipped():
    r = rng(12)
    keep_rows = r.standard_normal((10, 64))
    mix = r.standard_normal((50, 10))
    V = np.vstack([keep_rows, mix @ keep_rows])
    A = np.concatenate([np.full(10, 5.0), r.random(50)])
    idx = O.select_topk(A, 10)
    assert idx.tolist() == list(range(10))
    Vs, dg = O.backfill(V, A, idx, 3)
    assert dg.skipped == 1 and dg.rcr < 1e-20 and np.array_equal(Vs, V[idx])


# --------------------------------------------------------------------------- S6: rank-k subspace
def _power_subspace(G, k, iters=4000):
    C = np.linalg.qr(np.random.default_rng(0).standard_normal((G.shape[0], k)))[0]
    for _ in range(iters):
        C = np.linalg.qr(G @ C)[0]
    return C.T


def test_svd_gram_eigh_and_subspace_iteration_agree():
    r = rng(13)
    R = r.standard_normal((400, 32)) * np.linspace(3.0, 0.2, 32)[None, :] @ np.linalg.qr(r.standard_normal((32, 32)))[0]
    k = 4
    C_svd = np.linalg.svd(R, full_matrices=False)[2][:k]
    C_gram = O.top_subspace_gram(R, k)
    C_pow = _power_subspace(R.T @ R, k)
    P = C_svd.T @ C_svd
    assert np.allclose(P, C_gram.T @ C_gram, atol=1e-9)
    assert np.allclose(P, C_pow.T @ C_pow, atol=1e-7)


def test_revr_monotone_in_rank():
    r = rng(14)
    V = r.standard_normal((256, 64)); A = r.random(256)
    idx = O.select_topk(A, 16)
    vals = [O.backfill(V, A, idx, k)[1].revr for k in (1, 2, 4, 8, 16, 32)]
    assert all(b > a for a, b in zip(vals, vals[1:])) and vals[-1] < 1.0


# --------------------------------------------------------------------------- S7-S9: Eq. 4-6 closed forms
def test_closed_form_full_rank_budget_needs_no_svd():
    # pca_rank >= rank(R)  =>  Delta = rbar = P_perp sum_j w_j V_j
    r = rng(15)
    N, d, B = 120, 64, 40
    V = r.standard_normal((N, d)); A = r.random(N) + 0.01
    idx = O.select_topk(A, B)
    dele = np.setdiff1d(np.arange(N), idx)
    Vs, dg = O.backfill(V, A, idx, d)
    Pperp = np.eye(d) - np.linalg.pinv(V[idx]) @ V[idx]
    a_del, a_keep = A[dele].sum(), A[idx].sum()
    rbar = Pperp @ (A[dele] @ V[dele]) / (a_del + 1e-12)
    delta = a_del / (a_keep + 1e-12) * rbar
    assert dg.k_used == d - B
    assert np.allclose(Vs - V[idx], delta[None, :], rtol=1e-9, atol=1e-12)


def test_closed_form_planted_single_direction():
    # retained rows live on coordinates 0..B-1, every deleted row is c_j e_{d-1}
    r = rng(16)
    d, B, nd = 64, 12, 30
    Vk = np.zeros((B, d)); Vk[:, :B] = r.standard_normal((B, B))
    c = r.standard_normal(nd)
    Vd = np.zeros((nd, d)); Vd[:, d - 1] = c
    V = np.vstack([Vk, Vd])
    A = np.concatenate([2.0 + r.random(B), r.random(nd)])
    idx = O.select_topk(A, B)
    assert idx.tolist() == list(range(B))
    Vs, dg = O.backfill(V, A, idx, 3)
    a_keep, a_del = A[:B].sum(), A[B:].sum()
    expect = np.zeros(d)
    expect[d - 1] = (a_del / (a_keep + 1e-12)) * ((A[B:] @ c) / (a_del + 1e-12))
    assert dg.k_used == 1 and dg.r_keep == B and abs(dg.rcr - 1.0) < 1e-12
    assert np.allclose(Vs - Vk, expect[None, :], rtol=1e-10, atol=1e-14)


def test_rank_one_injection_by_hand():
    # hand computation on a 3-d example: keep = e0 ; deleted rows (1,2,0),(1,-2,0.1)
    V = np.array([[1.0, 0, 0], [1.0, 2.0, 0.0], [1.0, -2.0, 0.1]])
    A = np.array([3.0, 1.0, 0.5])
    idx = np.array([0])
    Vs, dg = O.backfill(V, A, idx, 1)
    R = np.array([[0, 2.0, 0.0], [0, -2.0, 0.1]])
    G = R.T @ R
    w, U = np.linalg.eigh(G)
    c = U[:, -1]
    rbar = (1.0 * R[0] + 0.5 * R[1]) / (1.5 + 1e-12)
    delta = 1.5 / (3.0 + 1e-12) * (rbar @ c) * c
    assert np.allclose(Vs[0] - V[0], delta, rtol=1e-12, atol=1e-15)


def test_homogeneity_and_token_permutation():
    r = rng(17)
    N, d, B = 90, 64, 20
    V = r.standard_normal((N, d)); A = r.random(N)
    idx = O.select_topk(A, B)
    d1 = O.backfill(V, A, idx, 3)[1].delta
    d2 = O.backfill(2.5 * V, A, idx, 3)[1].delta
    assert np.allclose(d2, 2.5 * d1, rtol=1e-10)
    d3 = O.backfill(V, 7.0 * A, idx, 3)[1].delta          # mass scale only meets epsilon
    assert np.allclose(d3, d1, rtol=1e-9)
    perm = r.permutation(N)
    inv = np.argsort(perm)
    idx_p = np.sort(inv[idx])
    d4 = O.backfill(V[perm], A[perm], idx_p, 3)[1].delta
    assert np.allclose(d4, d1, rtol=1e-9, atol=1e-13)


# --------------------------------------------------------------------------- S10: Eq. 7 and the whole head
def _head(seed, N=160, d=64, rows=6, scale=1.0):
    r = rng(seed)
    K = r.standard_normal((N, d)).astype(np.float32) * scale
    V = r.standard_normal((N, d)).astype(np.float32)
    Q = r.standard_normal((rows, d)).astype(np.float32)
    return K, V, Q


def test_injection_orthogonal_to_retained_values():
    K, V, Q = _head(18)
    res = O.compress_head(K, V, Q, 24, 4, "f32")
    delta = res.diag.delta
    Vk = V[res.idx].astype(np.float64)
    assert res.diag.skipped == 0 and res.diag.ivn > 0
    assert np.abs(Vk @ delta).max() <= 1e-5 * np.linalg.norm(Vk, axis=1).max() * np.linalg.norm(delta)
    assert np.allclose(res.V_star - Vk, delta[None, :], atol=1e-14)   # same vector on every retained row


def test_indices_and_keys_unchanged_by_backfill_and_rank_zero_is_eviction():
    K, V, Q = _head(19)
    a = O.compress_head(K, V, Q, 24, 0, "f32")
    b = O.compress_head(K, V, Q, 24, 4, "f32")
    assert np.array_equal(a.idx, b.idx) and np.array_equal(a.K_keep, b.K_keep)
    assert a.idx.size == 24
    assert np.array_equal(a.V_out, V[a.idx]) and a.diag.skipped == 1
    assert not np.array_equal(b.V_out, V[b.idx])


def test_budget_at_least_n_keeps_everything_untouched():
    K, V, Q = _head(20, N=40)
    res = O.compress_head(K, V, Q, 40, 4, "f32")
    assert res.idx.tolist() == list(range(40)) and np.array_equal(res.V_out, V) and res.diag.skipped == 1


def test_single_query_attention_output_identities():
    # App. L: with one query, o_evict is the retained conditional mean, and attending the
    # compressed cache gives o_OBF - o_evict = delta exactly.
    K, V, Q = _head(21, rows=1)
    res = O.compress_head(K, V, Q, 20, 3, "f32")
    Kd, Vd, q = K.astype(np.float64), V.astype(np.float64), Q.astype(np.float64)[0]
    s = Kd @ q / math.sqrt(64)
    alpha = np.exp(s - logsumexp(s))
    assert np.allclose(alpha, res.A, rtol=1e-12)
    keep = res.idx
    dele = np.setdiff1d(np.arange(len(s)), keep)
    sk = s[keep]; at = np.exp(sk - logsumexp(sk))
    o_evict = at @ Vd[keep]
    vbar_keep = (alpha[keep] @ Vd[keep]) / alpha[keep].sum()
    assert np.allclose(o_evict, vbar_keep, rtol=1e-12, atol=1e-14)
    o_obf = at @ res.V_star
    assert np.allclose(o_obf - o_evict, res.diag.delta, rtol=1e-10, atol=1e-14)
    # error decomposition with Eq. 6 taken literally (injection = Pi_U tau_perp / A_keep)
    o_full = alpha @ Vd
    A_keep, A_del = alpha[keep].sum(), alpha[dele].sum()
    tau = A_del * ((alpha[dele] @ Vd[dele]) / A_del - vbar_keep)
    assert np.allclose(o_full - o_evict, tau, rtol=1e-10, atol=1e-14)
    Pk = np.linalg.pinv(Vd[keep]) @ Vd[keep]
    tau_perp = tau - Pk @ tau
    R = Vd[dele] - Vd[dele] @ Pk
    C = np.linalg.svd(R, full_matrices=False)[2][:3]
    PU = C.T @ C
    lhs = np.linalg.norm(o_full - o_obf) ** 2
    rhs = (np.linalg.norm(Pk @ tau) ** 2 + np.linalg.norm(tau_perp - PU @ tau_perp) ** 2
           + (1.0 - 1.0 / A_keep) ** 2 * np.linalg.norm(PU @ tau_perp) ** 2)
    assert abs(lhs - rhs) <= 1e-9 * max(lhs, 1e-30)


def test_whole_head_against_loop_implementation_tiny():
    # an independent, loop-level restatement on a tiny head
    r = rng(22)
    N, d, B, p = 10, 4, 2, 1
    K = r.standard_normal((N, d)).astype(np.float32); V = r.standard_normal((N, d)).astype(np.float32)
    Q = r.standard_normal((3, d)).astype(np.float32)
    res = O.compress_head(K, V, Q, B, p, "f32")
    A = [0.0] * N
    for t in range(3):
        s = [sum(float(Q[t, c]) * float(K[j, c]) for c in range(d)) / math.sqrt(d) for j in range(N)]
        m = max(s); e = [math.exp(x - m) for x in s]; z = sum(e)
        for j in range(N):
            A[j] += e[j] / z
    order = sorted(range(N), key=lambda j: (-A[j], j))
    keep = sorted(order[:B]); dele = [j for j in range(N) if j not in keep]
    assert res.idx.tolist() == keep
    Vd = V.astype(np.float64)
    # Gram-Schmidt on the two retained rows
    q1 = Vd[keep[0]] / np.linalg.norm(Vd[keep[0]])
    u2 = Vd[keep[1]] - (Vd[keep[1]] @ q1) * q1; q2 = u2 / np.linalg.norm(u2)
    R = np.array([Vd[j] - (Vd[j] @ q1) * q1 - (Vd[j] @ q2) * q2 for j in dele])
    w, U = np.linalg.eigh(R.T @ R); c = U[:, -1]
    a_del = sum(A[j] for j in dele); a_keep = sum(A[j] for j in keep)
    rbar = sum((A[j] / (a_del + 1e-12)) * R[i] for i, j in enumerate(dele))
    delta = a_del / (a_keep + 1e-12) * (rbar @ c) * c
    assert np.allclose(res.V_star, Vd[keep] + delta[None, :], rtol=1e-10, atol=1e-13)


def test_relay_layout_maps_query_heads_to_kv_heads():
    r = rng(23)
    L, H, g, W, N, d = 2, 2, 3, 2, 30, 64
    K = r.standard_normal((L, H, N, d)).astype(np.float32); V = r.standard_normal((L, H, N, d)).astype(np.float32)
    Q = r.standard_normal((L, H * g, W, d)).astype(np.float32)
    out = O.compress_relay(K, V, Q, np.full((L, H), 5), 2, g, "f32")
    for (l, h), res in out.items():
        ref = O.attention_mass(K[l, h].astype(np.float64), Q[l, h * g:(h + 1) * g].reshape(-1, d).astype(np.float64))
        assert np.allclose(res.A, ref) and abs(res.A.sum() - g * W) < 1e-10


# --------------------------------------------------------------------------- layerwise granularity (Sec. 4.3.2)
def test_layerwise_with_one_head_is_headwise():
    r = rng(31)
    N, d, g, W = 40, 16, 2, 3
    K = r.standard_normal((1, N, d)).astype(np.float32); V = r.standard_normal((1, N, d)).astype(np.float32)
    Q = r.standard_normal((g, W, d)).astype(np.float32)
    idx, heads = O.compress_layer(K, V, Q, 7, 2, g, "f32")
    ref = O.compress_head(K[0], V[0], Q, 7, 2, "f32")
    assert idx.tolist() == ref.idx.tolist()
    assert np.array_equal(heads[0].V_out, ref.V_out) and np.array_equal(heads[0].K_keep, ref.K_keep)


def test_layerwise_index_set_against_loop_sum_tiny():
    # the shared set is TopK_B of the loop-level sum of every head's mass; every head gathers exactly those rows
    r = rng(32)
    H, N, d, g, W, B = 3, 12, 4, 2, 2, 4
    K = r.standard_normal((H, N, d)).astype(np.float32); V = r.standard_normal((H, N, d)).astype(np.float32)
    Q = r.standard_normal((H * g, W, d)).astype(np.float32)
    idx, heads = O.compress_layer(K, V, Q, B, 1, g, "f32")
    tot = [0.0] * N
    for h in range(H):
        for qh in range(g):
            for t in range(W):
                q = Q[h * g + qh, t]
                s = [sum(float(q[c]) * float(K[h, j, c]) for c in range(d)) / math.sqrt(d) for j in range(N)]
                m = max(s); e = [math.exp(x - m) for x in s]; z = sum(e)
                for j in range(N):
                    tot[j] += e[j] / z
    keep = sorted(sorted(range(N), key=lambda j: (-tot[j], j))[:B])
    assert idx.tolist() == keep
    assert abs(sum(tot) - H * g * W) < 1e-9
    for h in range(H):
        assert np.array_equal(heads[h].K_keep, K[h][keep])
        assert heads[h].idx.tolist() == keep


def test_layerwise_is_invariant_to_head_order_and_differs_from_headwise_when_heads_disagree():
    r = rng(33)
    H, N, d, g, W, B = 4, 50, 8, 1, 4, 6
    K = r.standard_normal((H, N, d)).astype(np.float32); V = r.standard_normal((H, N, d)).astype(np.float32)
    Q = (3.0 * r.standard_normal((H * g, W, d))).astype(np.float32)
    idx, heads = O.compress_layer(K, V, Q, B, 2, g, "f32")
    perm = [2, 0, 3, 1]
    idx_p, heads_p = O.compress_layer(K[perm], V[perm], Q[perm], B, 2, g, "f32")
    assert idx_p.tolist() == idx.tolist()
    for a, h in enumerate(perm):
        assert np.array_equal(heads_p[a].V_out, heads[h].V_out)
    # a head whose own mass is concentrated elsewhere keeps the layer's set, not its own
    own = [O.compress_head(K[h], V[h], Q[h * g:(h + 1) * g], B, 2, "f32").idx.tolist() for h in range(H)]
    assert any(o != idx.tolist() for o in own)


def test_layerwise_backfill_uses_each_heads_own_mass():
    # Eq. 4 and Eq. 6 weigh with the head's own attention mass: recompute one head by hand from the shared set
    r = rng(34)
    H, N, d, g, W, B = 2, 14, 5, 1, 3, 3
    K = r.standard_normal((H, N, d)).astype(np.float32); V = r.standard_normal((H, N, d)).astype(np.float32)
    Q = r.standard_normal((H * g, W, d)).astype(np.float32)
    idx, heads = O.compress_layer(K, V, Q, B, 1, g, "f32")
    h = 1
    A = O.attention_mass(K[h].astype(np.float64), Q[h * g:(h + 1) * g].reshape(-1, d).astype(np.float64))
    keep = idx.tolist(); dele = [j for j in range(N) if j not in keep]
    Vd = V[h].astype(np.float64)
    Qb, _ = np.linalg.qr(Vd[keep].T)                      # orthonormal basis of the retained span (columns)
    R = Vd[dele] - (Vd[dele] @ Qb) @ Qb.T
    w, U = np.linalg.eigh(R.T @ R); c = U[:, -1]
    a_del = A[dele].sum(); a_keep = A[keep].sum()
    rbar = (A[dele] / (a_del + 1e-12)) @ R
    delta = a_del / (a_keep + 1e-12) * (rbar @ c) * c
    assert np.allclose(heads[h].V_star, Vd[keep] + delta[None, :], rtol=1e-9, atol=1e-12)


# --------------------------------------------------------------------------- App. D: ablation variants
def _variant_case(seed=41, N=60, d=16, B=6):
    r = rng(seed)
    V = r.standard_normal((N, d))
    A = r.random(N) + 0.05
    idx = np.sort(r.choice(N, B, replace=False))
    return V, A, idx


def test_no_projection_equals_default_when_deleted_rows_are_orthogonal_to_the_retained_span():
    # retained rows live in the first 4 coordinates, deleted rows in the others: Eq. 3 removes nothing
    r = rng(42)
    N, d = 30, 12
    idx = np.array([2, 9, 17, 25])
    V = np.zeros((N, d))
    V[:, 4:] = r.standard_normal((N, 8))
    V[idx] = 0.0
    V[idx, :4] = r.standard_normal((4, 4))
    A = r.random(N) + 0.1
    a, da = O.backfill(V, A, idx, 3)
    b, db = O.backfill(V, A, idx, 3, O.Variant(no_projection=True))
    assert da.skipped == 0 and db.skipped == 0 and db.r_keep == 0
    assert np.allclose(a, b, rtol=0, atol=1e-13)


def test_no_projection_by_hand_where_the_default_has_nothing_to_inject():
    # every deleted row is a multiple of e0 and e0 is a retained row: R = 0 for the method, R = V_del without Eq. 3.
    # Then C = e0, rbar = sum_j w_j c_j e0, Delta = rbar, delta = a_del / a_keep * rbar.
    d = 4
    V = np.zeros((5, d))
    V[0, 0] = 1.0; V[1, 1] = 1.0                                   # retained
    c = np.array([2.0, -1.0, 4.0])
    V[2:, 0] = c                                                  # deleted
    A = np.array([0.3, 0.2, 0.1, 0.15, 0.25])
    idx = np.array([0, 1])
    out, dg = O.backfill(V, A, idx, 1)
    assert dg.skipped == 1 and np.array_equal(out, V[idx])
    out, dg = O.backfill(V, A, idx, 1, O.Variant(no_projection=True))
    a_del, a_keep = 0.5, 0.5
    coef = (0.1 * 2.0 + 0.15 * -1.0 + 0.25 * 4.0) / a_del * (a_del / a_keep)
    assert dg.skipped == 0 and dg.k_used == 1
    assert np.allclose(out - V[idx], np.array([[coef, 0, 0, 0]] * 2), rtol=0, atol=1e-11)


def test_max_p_injects_the_whole_weighted_residual_mean():
    V, A, idx = _variant_case()
    out, dg = O.backfill(V, A, idx, 2, O.Variant(subspace="all"))
    dele = np.setdiff1d(np.arange(V.shape[0]), idx)
    # residual through a least-squares fit instead of an orthonormal basis
    coef, *_ = np.linalg.lstsq(V[idx].T, V[dele].T, rcond=None)
    R = V[dele] - (V[idx].T @ coef).T
    rbar = (A[dele] / A[dele].sum()) @ R
    want = A[dele].sum() / A[idx].sum() * rbar
    assert dg.k_used == V.shape[1] - idx.size
    assert np.allclose(out - V[idx], np.broadcast_to(want, (idx.size, V.shape[1])), rtol=0, atol=1e-11)


def test_no_scaling_differs_from_the_method_by_exactly_the_demand_ratio():
    V, A, idx = _variant_case(43)
    a, da = O.backfill(V, A, idx, 3)
    b, db = O.backfill(V, A, idx, 3, O.Variant(no_scaling=True))
    dele = np.setdiff1d(np.arange(V.shape[0]), idx)
    ratio = A[dele].sum() / A[idx].sum()
    assert abs(ratio - 1.0) > 0.5                                  # the flag matters on this case
    assert np.allclose(a - V[idx], ratio * (b - V[idx]), rtol=0, atol=1e-12)
    assert abs(da.ivn - ratio * db.ivn) < 1e-12


def test_naive_aggregation_by_hand():
    V = np.array([[1.0, 0.0, 0.0], [0.0, 2.0, 0.0], [3.0, 3.0, 3.0], [1.0, -1.0, 5.0], [-4.0, 4.0, 1.0]])
    A = np.array([0.5, 0.1, 0.2, 0.1, 0.1])
    idx = np.array([0, 1])
    out, dg = O.backfill(V, A, idx, 1, O.Variant(naive=True))
    mean = np.array([0.0, 2.0, 3.0])                               # plain average of rows 2, 3, 4; A plays no part
    assert dg.skipped == 0 and dg.k_used == 0
    assert np.allclose(out, V[idx] + mean, rtol=0, atol=1e-15)
    assert abs(dg.ivn - math.sqrt(13.0)) < 1e-14


def test_attn_inject_shares_the_same_total_in_proportion_to_mass():
    V, A, idx = _variant_case(44)
    A[idx[0]] = A[idx[1]]                                          # two retained rows with equal mass
    a, da = O.backfill(V, A, idx, 2)
    b, db = O.backfill(V, A, idx, 2, O.Variant(attn_inject=True))
    assert np.allclose(da.delta, db.delta, rtol=0, atol=0)         # only Eq. 7 differs
    add = b - V[idx]
    assert np.allclose(add.sum(axis=0), idx.size * da.delta, rtol=1e-11, atol=1e-13)   # same total as B equal shares
    assert np.allclose(add[0], add[1], rtol=0, atol=1e-15)
    share = A[idx] / A[idx].sum()
    for t in range(idx.size):
        assert np.allclose(add[t], idx.size * share[t] * da.delta, rtol=1e-11, atol=1e-13)
    # with equal mass on every retained row it is Eq. 7 again
    A2 = A.copy(); A2[idx] = 0.125
    a2, _ = O.backfill(V, A2, idx, 2)
    b2, _ = O.backfill(V, A2, idx, 2, O.Variant(attn_inject=True))
    assert np.allclose(a2, b2, rtol=0, atol=1e-10)              # eps of the share's denominator is all that differs


@pytest.mark.parametrize("tau,k_want", [(0.35, 1), (0.5, 2), (0.7, 3), (0.9, 4), (0.96, 5)])
def test_evr_adaptive_rank_on_known_singular_values(tau, k_want):
    # deleted rows sigma_j e_{2+j}, retained rows e_0, e_1: R = V_del with squared singular values 4, 3, 2, 1, 0.5
    # cumulative fractions of 10.5: 0.381, 0.667, 0.857, 0.952, 1
    d = 8
    V = np.zeros((7, d))
    V[0, 0] = 1.0; V[1, 1] = 1.0
    s2 = [4.0, 3.0, 2.0, 1.0, 0.5]
    for j, v in enumerate(s2):
        V[2 + j, 2 + j] = math.sqrt(v)
    A = np.full(7, 1.0 / 7)
    out, dg = O.backfill(V, A, np.array([0, 1]), 1, O.Variant(subspace="evr", evr_tau=tau))
    assert dg.k_used == k_want
    assert abs(dg.revr - sum(s2[:k_want]) / 10.5) < 1e-12
    # Delta keeps exactly the first k_want coordinates of rbar = (1/5) sum_j sigma_j e_{2+j}; demand ratio 5/2
    want = np.zeros(d)
    for j in range(k_want):
        want[2 + j] = 0.2 * math.sqrt(s2[j]) * 2.5
    assert np.allclose(out[0], V[0] + want, rtol=0, atol=1e-10)   # the eps of Eq. 4 and Eq. 6 is of relative size 4e-12 here


def test_variants_leave_the_default_untouched_and_combine():
    V, A, idx = _variant_case(45)
    a, _ = O.backfill(V, A, idx, 2)
    b, _ = O.backfill(V, A, idx, 2, O.Variant())
    assert np.array_equal(a, b)
    # naive aggregation with attention-weighted shares: both replacements act
    c, dg = O.backfill(V, A, idx, 2, O.Variant(naive=True, attn_inject=True))
    dele = np.setdiff1d(np.arange(V.shape[0]), idx)
    mean = V[dele].sum(axis=0) / dele.size
    share = A[idx] / A[idx].sum()
    assert np.allclose(c - V[idx], idx.size * share[:, None] * mean[None, :], rtol=1e-11, atol=1e-13)


# --------------------------------------------------------------------------- Sec. 4.3.2 eligible set, Sec. 3.3 message
def _sink_case(seed=51, N=40, d=8, rows=6):
    r = rng(seed)
    K = r.standard_normal((N, d)).astype(np.float32)
    V = r.standard_normal((N, d)).astype(np.float32)
    Q = r.standard_normal((rows, d)).astype(np.float32)
    return K, V, Q


def test_sink_tokens_are_never_candidates_but_stay_softmax_keys():
    K, V, Q = _sink_case()
    K[:3] *= 6.0                                                   # the sink keys attract most of the mass
    full = O.compress_head(K, V, Q, 5, 0, "f32")
    assert set(full.idx.tolist()) & {0, 1, 2}                      # without protection some of them are picked
    res = O.compress_head(K, V, Q, 5, 0, "f32", sink=3)
    assert res.idx.min() >= 3 and res.idx.size == 5 and np.all(np.diff(res.idx) > 0)
    assert abs(res.A.sum() - Q.shape[0]) < 1e-12                   # every row still sums to one over all real tokens
    # brute force: the 5 largest masses among tokens 3.., ties to the lowest index
    order = sorted(range(3, K.shape[0]), key=lambda j: (-res.A[j], j))[:5]
    assert sorted(order) == res.idx.tolist()
    # the sink keys shape the masses: without them the candidates' masses are larger
    A_cut = O.attention_mass(O.decode(K[3:], "f32"), O.decode(Q, "f32"))
    assert np.all(A_cut > res.A[3:])


def test_sink_values_take_no_part_in_backfill_and_sink_zero_is_the_plain_call():
    K, V, Q = _sink_case(52, N=30, d=8)
    a = O.compress_head(K, V, Q, 4, 2, "f32", sink=4)
    V2 = V.copy(); V2[:4] = 99.0
    b = O.compress_head(K, V2, Q, 4, 2, "f32", sink=4)
    assert a.diag.skipped == 0
    assert np.array_equal(a.idx, b.idx) and np.array_equal(a.V_out, b.V_out)
    # deleted set = eligible minus kept: the demand masses of Eq. 6 leave the sink out
    elig = np.arange(4, 30)
    dele = np.setdiff1d(elig, a.idx)
    assert abs(a.diag.a_del - a.A[dele].sum()) < 1e-14 and abs(a.diag.a_keep - a.A[a.idx].sum()) < 1e-14
    # the injection is orthogonal to the retained value rows
    Vd = O.decode(V, "f32")
    assert np.abs(Vd[a.idx] @ a.diag.delta).max() < 1e-12 * np.abs(Vd).max() * max(np.abs(a.diag.delta).max(), 1.0) * 100
    p = O.compress_head(K, V, Q, 4, 2, "f32")
    q = O.compress_head(K, V, Q, 4, 2, "f32", sink=0)
    assert np.array_equal(p.idx, q.idx) and np.array_equal(p.V_out, q.V_out)


def test_budget_above_the_eligible_count_keeps_every_eligible_token():
    K, V, Q = _sink_case(53, N=12)
    res = O.compress_head(K, V, Q, 100, 2, "f32", sink=4)
    assert res.idx.tolist() == list(range(4, 12)) and res.diag.skipped == 1


def test_layerwise_sink_shares_one_eligible_index_set():
    r = rng(54)
    H, N, d = 3, 24, 8
    K = r.standard_normal((H, N, d)).astype(np.float32)
    V = r.standard_normal((H, N, d)).astype(np.float32)
    Q = r.standard_normal((H, 4, d)).astype(np.float32)
    K[:, :2] *= 5.0
    idx, heads = O.compress_layer(K, V, Q, 6, 1, 1, "f32", sink=2)
    assert idx.min() >= 2 and idx.size == 6
    tot = sum(h.A for h in heads)
    order = sorted(range(2, N), key=lambda j: (-tot[j], j))[:6]
    assert sorted(order) == idx.tolist()
    assert all(np.array_equal(h.idx, idx) for h in heads)


def test_message_is_the_row_concatenation_in_the_order_of_sec_3_3():
    prev = np.array([[1, 1], [2, 2]], dtype=np.float32)
    keep = np.array([[3, 3]], dtype=np.float32)
    gen = np.array([[4, 4], [5, 5], [6, 6]], dtype=np.float32)
    M = O.append_message(prev, keep, gen)
    assert M.tolist() == [[1, 1], [2, 2], [3, 3], [4, 4], [5, 5], [6, 6]]
    assert O.append_message(prev[:0], keep, gen[:0]).tolist() == [[3, 3]]


# --------------------------------------------------------------------------- App. K.2: PC and DR by hand; threshold constants
def test_projection_cosine_and_demand_ratio_by_hand():
    # d = 4, retained rows e0 and 2 e1 (span = first two coordinates); deleted rows (1,2,3,4) and (2,0,-1,1).
    # Column sums of the deleted rows: s = (3,2,2,5); of their projections onto the retained span: (3,2,0,0).
    # PC = <s, Pi s> / (|s| |Pi s|) = 13 / (sqrt(42) sqrt(13)) = sqrt(13/42)              (App. K.2)
    # DR = (0.25 + 0.5) / (2 + 1) = 0.25 up to the 1e-12 of the denominator               (App. K.2, Eq. 6)
    V = np.array([[1.0, 0, 0, 0], [0, 2.0, 0, 0], [1.0, 2.0, 3.0, 4.0], [2.0, 0.0, -1.0, 1.0]])
    A = np.array([2.0, 1.0, 0.25, 0.5])
    _, dg = O.backfill(V, A, np.array([0, 1]), 1)
    assert abs(dg.pc - math.sqrt(13.0 / 42.0)) < 1e-14
    assert abs(dg.dr - 0.25) < 1e-12 and dg.dr < 0.25          # the epsilon sits in the denominator
    assert abs(dg.a_keep - 3.0) < 1e-15 and abs(dg.a_del - 0.75) < 1e-15
    # squared norms: deleted rows 30 + 6 = 36, their projections 5 + 4 = 9  =>  PCR = 1/4, RCR = 3/4
    assert abs(dg.pcr - 0.25) < 1e-12 and abs(dg.rcr - 0.75) < 1e-12
    # a sign flip of one deleted row's in-span part changes the cosine: rows (1,2,3,4), (-2,0,-1,1):
    # s = (-1,2,2,5), Pi s = (-1,2,0,0): PC = 5 / (sqrt(34) sqrt(5)) = sqrt(5/34)
    V2 = V.copy(); V2[3, 0] = -2.0
    _, dg2 = O.backfill(V2, A, np.array([0, 1]), 1)
    assert abs(dg2.pc - math.sqrt(5.0 / 34.0)) < 1e-14


def test_demand_ratio_on_the_planted_case_is_the_eq6_factor():
    # planted single direction (all deleted rows c_j e_{d-1}, c_j = 1): delta = DR * e_{d-1} exactly, so the
    # diagnostic must equal the injected coordinate
    d, B, nd = 16, 5, 9
    Vk = np.zeros((B, d)); Vk[:, :B] = np.eye(B)
    Vd = np.zeros((nd, d)); Vd[:, d - 1] = 1.0
    A = np.concatenate([np.full(B, 3.0), np.full(nd, 0.5)])
    Vs, dg = O.backfill(np.vstack([Vk, Vd]), A, np.arange(B), 2)
    assert abs(dg.dr - 4.5 / 15.0) < 1e-12
    assert abs((Vs - Vk)[0, d - 1] - dg.dr) < 1e-12 and abs(dg.ivn - dg.dr) < 1e-12


def test_rank_rule_threshold_is_max_of_rows_and_cols_times_single_epsilon():
    # singular values known by construction (scaled unit rows): {1, t}.  Threshold: max(rows, d) * 2^-23.
    d = 4
    def keep_rows(rows, t):
        V = np.zeros((rows, d)); V[0, 0] = 1.0; V[1, 1] = t
        return V
    # 2 rows, d = 4: threshold 4 * 2^-23 = 2^-21
    assert O.orth_rowspace(keep_rows(2, 1.01 * 2.0 ** -21))[0].shape[1] == 2
    assert O.orth_rowspace(keep_rows(2, 0.99 * 2.0 ** -21))[0].shape[1] == 1
    # 8 rows (six of them zero), d = 4: threshold 8 * 2^-23 = 2^-20 (with min(rows, d) it would still be 2^-21)
    assert O.orth_rowspace(keep_rows(8, 1.5 * 2.0 ** -21))[0].shape[1] == 1
    assert O.orth_rowspace(keep_rows(8, 1.01 * 2.0 ** -20))[0].shape[1] == 2
    # the same rule decides rank(R) in k = min(pca_rank, rank R): residual rows (0,0,1,0) and (0,0,0,t), 2 deleted rows
    for t, k_want in ((1.01 * 2.0 ** -21, 2), (0.99 * 2.0 ** -21, 1)):
        V = np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0], [0, 0, 1.0, 0], [0, 0, 0, t]])
        _, dg = O.backfill(V, np.array([2.0, 2.0, 0.5, 0.5]), np.array([0, 1]), 3)
        assert dg.k_used == k_want


def test_negligible_residual_threshold_is_one_millionth_of_the_deleted_energy():
    # retained e0; one deleted row (1, t): ||R||^2 / ||V_del||^2 = t^2 / (1 + t^2)
    for t, skipped in ((1.1e-3, 0), (0.9e-3, 1)):
        V = np.array([[1.0, 0.0], [1.0, t]])
        Vs, dg = O.backfill(V, np.array([2.0, 1.0]), np.array([0]), 1)
        assert dg.skipped == skipped and abs(dg.rcr - t * t / (1 + t * t)) < 1e-17
        assert (Vs[0, 1] != 0.0) == (skipped == 0)


# --------------------------------------------------------------------------- the benchmark's second CPU baseline (App. H route)
def test_single_precision_gram_baseline_agrees_with_the_oracle():
    import synth_inputs as si
    from oracle import gram_baseline as G
    cfg = si.shrink(si.CONFIGS["2s"], n_layers=1, n_kv_heads=2)
    K, V, Q = si.make_cache(cfg, 4, threads=2)
    for h in range(2):
        Qh = Q[0, h * cfg.group:(h + 1) * cfg.group]
        ref = O.compress_head(K[0, h], V[0, h], Qh, 40, 2, cfg.dtype)
        idx, Vs, delta, skipped = G.compress_head_gram32(K[0, h], V[0, h], Qh, 40, 2, cfg.dtype)
        assert skipped == 0 and ref.diag.skipped == 0
        # float32 scores can swap tokens whose masses agree to ~1e-6; allow a couple
        assert len(set(idx.tolist()) ^ set(ref.idx.tolist())) <= 2
        if np.array_equal(idx, ref.idx):
            err = np.linalg.norm(delta - ref.diag.delta) / np.linalg.norm(ref.diag.delta)
            assert err < 2e-3 * max(1.0, 0.05 / max(1.0 - 1.0 / ref.diag.gap ** 2, 1e-12)), err
    # full-rank retained span: identity, like the oracle
    cfg3 = si.shrink(si.CONFIGS["2"], n_layers=1, n_kv_heads=1)
    K, V, Q = si.make_cache(cfg3, 0, threads=2)
    idx, Vs, delta, skipped = G.compress_head_gram32(K[0, 0], V[0, 0], Q[0, :cfg3.group], cfg3.budget, cfg3.rank, cfg3.dtype)
    assert skipped == 1 and not delta.any() and idx.size == cfg3.budget


# --------------------------------------------------------------------------- App. E: cache merging
def test_merge_routing_brute_force_and_by_hand():
    # by hand, d = 2: retained keys (1,0) [slot 0] and (0,2) [slot 1]; deleted keys (3,1): cos (0.949, 0.316) -> slot 0;
    # (1,5): cos (0.196, 0.981) -> slot 1; (-1,-1): cos (-0.707, -0.707): a tie, the lowest slot wins; (0,0): all cosines
    # are taken as 0, lowest slot
    K = np.array([[1.0, 0], [3.0, 1.0], [0, 2.0], [1.0, 5.0], [-1.0, -1.0], [0.0, 0.0]])
    route = O.merge_routes(K, np.array([0, 2]))
    assert route.tolist() == [-1, 0, -1, 1, 0, 0]
    # scale invariance of the cosine: rescaling any key changes no route (powers of two, so that the exact tie stays exact)
    K2 = K * np.array([4.0, 0.125, 8.0, 2.0, 0.5, 1.0])[:, None]
    assert O.merge_routes(K2, np.array([0, 2])).tolist() == route.tolist()
    # brute force with an independent formulation (angles through arccos of normalised rows, python loops)
    r = rng(40)
    K = r.standard_normal((30, 8)); idx = np.sort(r.choice(30, 7, replace=False))
    route = O.merge_routes(K, idx)
    for j in range(30):
        if j in idx:
            assert route[j] == -1
            continue
        best, arg = None, None
        for s, t in enumerate(idx):
            ang = math.acos(max(-1.0, min(1.0, float(K[j] @ K[t]) / math.sqrt(float(K[j] @ K[j]) * float(K[t] @ K[t])))))
            if best is None or ang < best - 1e-12:
                best, arg = ang, s
        assert route[j] == arg


def test_merge_values_by_hand_and_mass_conservation():
    # two retained slots (tokens 0 and 2), three deleted tokens: 1 -> slot 0, 3 -> slot 1, 4 -> slot 0
    V = np.array([[1.0, 1.0], [2.0, 0.0], [0.0, 3.0], [4.0, 4.0], [0.0, -2.0]])
    A = np.array([4.0, 1.0, 2.0, 0.5, 2.0])
    idx = np.array([0, 2]); route = np.array([-1, 0, -1, 1, 0])
    Vs = O.merge_values(V, A, idx, route)
    # slot 0: (1,1) + 1/4 (2,0) + 2/4 (0,-2) = (1.5, 0);  slot 1: (0,3) + 0.5/2 (4,4) = (1, 4)
    assert np.allclose(Vs, [[1.5, 0.0], [1.0, 4.0]], rtol=0, atol=1e-11)
    # the epsilon sits in the denominator next to A_t: a retained mass of zero gives a finite (huge) weight, not inf
    A0 = A.copy(); A0[2] = 0.0
    assert np.isfinite(O.merge_values(V, A0, idx, route)).all()
    # attention-mass weighted first moment is conserved: sum_t A_t V*_t = sum over all tokens A_j V_j (up to eps)
    r = rng(41)
    K = r.standard_normal((60, 16)); V = r.standard_normal((60, 16)); A = r.random(60) + 0.1
    idx = O.select_topk(A, 9)
    route = O.merge_routes(K, idx)
    Vs = O.merge_values(V, A, idx, route)
    assert np.allclose((A[idx][:, None] * Vs).sum(axis=0), (A[:, None] * V).sum(axis=0), rtol=1e-10)


def test_merge_head_keeps_keys_and_index_set_and_leaves_untouched_slots_as_bit_copies():
    import synth_inputs as si
    cfg = si.RelayConfig("merge-pin", 50, 1, 1, 2, 64, 200, 4, 150, 0, "bf16", "structured")
    K, V, Q = si.make_cache(cfg, 0)
    ev = O.compress_head(K[0, 0], V[0, 0], Q[0, :2], 150, 0, "bf16")          # plain eviction: the same selector
    mg = O.merge_head(K[0, 0], V[0, 0], Q[0, :2], 150, "bf16")
    assert np.array_equal(mg.idx, ev.idx) and np.array_equal(mg.K_keep, ev.K_keep)
    routed_to = set(mg.route[mg.route >= 0].tolist())
    assert 0 < len(routed_to) < 150                                            # 50 deleted tokens cannot reach all 150 slots
    for s in range(150):
        same = np.array_equal(mg.V_out[s], V[0, 0][mg.idx[s]])
        assert same == (s not in routed_to) or (s in routed_to and same)       # untouched slots are bit copies
        if s not in routed_to:
            assert same
    # budget >= N: nothing deleted, nothing merged
    full = O.merge_head(K[0, 0], V[0, 0], Q[0, :2], 500, "bf16")
    assert np.array_equal(full.V_out, V[0, 0]) and (full.route == -1).all()


# --------------------------------------------------------------------------- App. E: stacked int8 / int4 relay (a reading; unpinned by the paper)
def test_row_quantisation_by_hand_roundtrip_bound_and_ratio():
    # by hand: x = 0, 0.5, ..., 127.5: zero = 0, scale = 127.5 / 255 = 0.5 exactly, code of entry i is i
    x = (np.arange(256, dtype=np.float32) * 0.5)[None, :]
    q, s, z = O.quantize_rows(x, "f32", 8)
    assert float(z[0]) == 0.0 and float(s[0]) == 0.5 and q[0].tolist() == list(range(256))
    # int4: x = -3 + 0.4 i, i = 0..15: zero = fp16(-3), scale = fp16(0.4), codes 0..15
    x4 = (-3.0 + 0.4 * np.arange(16, dtype=np.float32))[None, :].astype(np.float32)
    q4, s4, z4 = O.quantize_rows(x4, "f32", 4)
    assert q4[0].tolist() == list(range(16)) and float(z4[0]) == -3.0 and abs(float(s4[0]) - 0.4) < 2e-4
    # a constant row: scale 0, codes 0, the value comes back as fp16(x)
    qc, sc, zc = O.quantize_rows(np.full((1, 64), 1.5, dtype=np.float32), "f32", 8)
    assert not qc.any() and float(sc[0]) == 0.0 and np.all(O.dequantize_rows(qc, sc, zc) == 1.5)
    # round trip on random bf16 rows: |x - x_hat| <= scale / 2 + the rounding of zero and scale to half precision
    r = rng(60)
    X = O.round_to_io(r.standard_normal((50, 128)) * np.exp(r.standard_normal((50, 1))), "bf16")
    for bits in (8, 4):
        q, s, z = O.quantize_rows(X, "bf16", bits)
        assert q.max() <= 2 ** bits - 1
        x = O.decode(X, "bf16")
        err = np.abs(O.dequantize_rows(q, s, z) - x)
        span = x.max(axis=1) - x.min(axis=1)
        bound = 0.5 * s.astype(np.float64) + 2.0 ** -10 * (np.abs(x).max(axis=1) + span)      # fp16 keeps 11 significant bits
        assert np.all(err <= bound[:, None] * 1.01 + 1e-12)
        # every row uses its range: the smallest entry gets code 0 or 1, the largest the top code or one below
        assert np.all(q[np.arange(50), x.argmin(axis=1)] <= 1) and np.all(q[np.arange(50), x.argmax(axis=1)] >= 2 ** bits - 2)
    # the sizes behind the paper's ratios at head_dim 128: 16-bit rows against codes plus two half-precision numbers
    assert abs(16 * 128 / (8 * 128 + 32) - 1.94) < 0.01 and abs(16 * 128 / (4 * 128 + 32) - 3.76) < 0.01


# --------------------------------------------------------------------------- App. H: the literal Gram subspace iteration
def test_subspace_iteration_start_is_orthonormal_and_converges_to_the_svd_subspace():
    C0 = O.start_rows(8, 64)
    assert np.allclose(C0 @ C0.T, np.eye(8), atol=1e-13)
    # a residual with a clear gap after the third singular value: three steps already agree with the SVD to ~1e-4
    # (the accuracy App. H quotes), many steps to rounding
    r = rng(80)
    U = np.linalg.qr(r.standard_normal((400, 64)))[0]; Vt = np.linalg.qr(r.standard_normal((64, 64)))[0]
    sv = np.concatenate([[10.0, 9.0, 8.0], 0.4 * r.random(61)])
    R = (U * sv) @ Vt
    exact = Vt[:3]
    P = exact.T @ exact
    C3 = O.subspace_iteration(R.T @ R, 3, 3)
    C60 = O.subspace_iteration(R.T @ R, 3, 60)
    assert C3.shape == (3, 64) and np.allclose(C3 @ C3.T, np.eye(3), atol=1e-12)
    assert np.linalg.norm(C3.T @ C3 - P) < 5e-4 and np.linalg.norm(C60.T @ C60 - P) < 1e-10
    # one step from C_0 is literally orth(C_0 G): its rows span the rows of C_0 G
    C1 = O.subspace_iteration(R.T @ R, 3, 1)
    Y = O.start_rows(3, 64) @ (R.T @ R)
    assert np.linalg.matrix_rank(np.vstack([C1, Y]), tol=1e-8 * np.linalg.norm(Y)) == 3
    # dependent rows are dropped: a residual of rank 2 leaves two rows whatever k asks for
    R2 = (U[:, :2] * np.array([3.0, 1.0])) @ Vt[:2]
    assert O.subspace_iteration(R2.T @ R2, 5, 3).shape[0] == 2


def test_fast_path_variant_reports_its_distance_from_the_svd_and_injects_its_own_direction():
    r = rng(81)
    V = r.standard_normal((300, 64)) * np.exp(-0.05 * np.arange(64)); A = r.random(300)
    idx = O.select_topk(A, 20)
    Vs, dg = O.backfill(V, A, idx, 2)
    Vf, df = O.backfill(V, A, idx, 2, O.Variant(subspace_iters=3))
    V50, d50 = O.backfill(V, A, idx, 2, O.Variant(subspace_iters=200))
    assert df.k_used == 2 and df.skipped == 0 and dg.fast_err == -1.0
    # the reported error is the relative distance of the two injected vectors (same scaling on both)
    assert abs(df.fast_err - np.linalg.norm(df.delta - dg.delta) / np.linalg.norm(dg.delta)) < 1e-12
    assert df.fast_err > 1e-8                      # three steps are an approximation on a flat spectrum ...
    assert d50.fast_err < 1e-6 * max(1.0, 0.05 / max(1 - 1 / dg.gap ** 2, 1e-12)) + 1e-9   # ... many steps are not
    assert np.allclose(Vf - V[idx], df.delta[None, :], atol=1e-13)
    # still orthogonal to the retained values: every iterate stays in the row space of R
    assert np.abs(V[idx] @ df.delta).max() < 1e-10 * np.linalg.norm(V[idx], axis=1).max() * np.linalg.norm(df.delta)


# --------------------------------------------------------------------------- App. D: the Per-token alternative (a stated reading)
def test_per_token_offsets_average_to_the_methods_delta_and_stay_orthogonal():
    r = rng(90)
    N, d, B, k = 260, 32, 12, 3
    K = r.standard_normal((N, d)); V = r.standard_normal((N, d)) * np.exp(-0.08 * np.arange(d)); A = r.random(N)
    idx = O.select_topk(A, B)
    Vm, dm = O.backfill(V, A, idx, k)                                        # the method itself
    Vp, dp = O.backfill(V, A, idx, k, O.Variant(per_token=True), K)
    off = Vp - V[idx]
    # the reading's defining property: the slots' directions average to Eq. 6's single delta, which is also what is reported
    assert np.allclose(off.mean(axis=0), dm.delta, rtol=0, atol=1e-12 * np.abs(dm.delta).max())
    assert np.allclose(dp.delta, dm.delta, rtol=0, atol=1e-15) and dp.k_used == dm.k_used and dp.skipped == 0
    # every slot's direction lies in the residual subspace: orthogonal to every retained value (Eq. 3)
    assert np.abs(V[idx] @ off.T).max() < 1e-10 * np.linalg.norm(V[idx], axis=1).max() * np.linalg.norm(off, axis=1).max()
    # a slot that no deleted token is routed to keeps its value exactly
    route = O.merge_routes(K, idx)
    empty = sorted(set(range(B)) - set(route[route >= 0].tolist()))
    for t in empty:
        assert np.array_equal(Vp[t], V[idx][t])
    # No Scaling leaves Eq. 6's ratio out of every slot alike
    Vn, dn = O.backfill(V, A, idx, k, O.Variant(per_token=True, no_scaling=True), K)
    ratio = dm.a_del / (dm.a_keep + O.EPS)
    assert np.allclose((Vn - V[idx]) * ratio, off, rtol=1e-12, atol=1e-15)


def test_per_token_with_every_deleted_token_on_one_slot_gives_that_slot_everything():
    r = rng(91)
    N, d, B, k = 120, 16, 5, 2
    K = 0.01 * r.standard_normal((N, d)); V = r.standard_normal((N, d)); A = r.random(N) + 0.1
    idx = np.array([3, 40, 41, 77, 100])
    # keys: every deleted token points along e_0 like slot 2 (token 41); the other slots point elsewhere
    K[:, 0] += 1.0
    for s, t in enumerate(idx):
        if s != 2:
            K[t] = 0.0; K[t, 1 + s] = 1.0
    route = O.merge_routes(K, idx)
    assert set(route[route >= 0].tolist()) == {2}
    Vm, dm = O.backfill(V, A, idx, k)
    Vp, dp = O.backfill(V, A, idx, k, O.Variant(per_token=True), K)
    off = Vp - V[idx]
    assert np.allclose(off[2], B * dm.delta, rtol=1e-12, atol=1e-15)         # B times the method's share, so that the mean is delta
    assert not off[[0, 1, 3, 4]].any()
    # with a single retained slot the alternative IS the method
    i1 = np.array([41])
    V1, d1 = O.backfill(V, A, i1, k)
    P1, _ = O.backfill(V, A, i1, k, O.Variant(per_token=True), K)
    assert np.allclose(P1, V1, rtol=1e-13, atol=1e-15)


def test_per_token_needs_keys_and_refuses_the_combinations_it_has_no_reading_for():
    r = rng(92)
    V = r.standard_normal((50, 8)); A = r.random(50); K = r.standard_normal((50, 8))
    idx = O.select_topk(A, 4)
    with pytest.raises(ValueError):
        O.backfill(V, A, idx, 2, O.Variant(per_token=True))
    for bad in (O.Variant(per_token=True, attn_inject=True), O.Variant(per_token=True, subspace="all")):
        with pytest.raises(ValueError):
            O.backfill(V, A, idx, 2, bad, K)
    # the fast path's subspace is used when both are asked for
    Vf, df = O.backfill(V, A, idx, 2, O.Variant(per_token=True, subspace_iters=3), K)
    Vg, dg = O.backfill(V, A, idx, 2, O.Variant(subspace_iters=3))
    assert np.allclose((Vf - V[idx]).mean(axis=0), dg.delta, rtol=0, atol=1e-12 * np.abs(dg.delta).max())
