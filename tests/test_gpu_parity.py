"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import obf_oracle as O
from tests import parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from tests import gpu_util
    from paper_2604_13349_amd import binding
    binding.load_library()          # no fallback: a missing library is an error, not a skip
    return gpu_util


def _gpu_variant(v):
    """The binding's obf_variant_t for an oracle Variant (field by field, no arithmetic)."""
    from paper_2604_13349_amd import binding as B
    return B.make_variant(no_projection=v.no_projection, subspace=v.subspace, evr_tau=v.evr_tau, no_scaling=v.no_scaling,
                          naive_aggregation=v.naive, attn_inject=v.attn_inject, subspace_iters=v.subspace_iters,
                          per_token=v.per_token)


def _check_cfg(gpu, cfg, seed=0, budgets=None, rank=None, expect_active=None, max_budget=None, edit=None, variant=None):
    K, V, Q = si.make_cache(cfg, seed, threads=8)
    if edit is not None:
        edit(K, V, Q)                     # in-place change of the synthetic cache (still seeded, still no oracle data)
    bud = si.budgets(cfg, seed) if budgets is None else np.asarray(budgets, dtype=np.int32).reshape(cfg.n_layers, cfg.n_kv_heads)
    rank = cfg.rank if rank is None else rank
    out = gpu.run_fused(cfg, K, V, Q, budgets=bud, rank=rank, max_budget=max_budget,
                        variant=None if variant is None else _gpu_variant(variant))
    reps = []
    for l in range(cfg.n_layers):
        for h in range(cfg.n_kv_heads):
            ref = O.compress_head(K[l, h], V[l, h], Q[l, h * cfg.group:(h + 1) * cfg.group], int(bud[l, h]), rank, cfg.dtype,
                                  *(() if variant is None else (variant,)))
            rep = parity.check_head(f"{cfg.name}[{l},{h}]", ref, K[l, h], V[l, h], cfg.dtype, int(bud[l, h]),
                                    out["idx"][l, h], out["n_keep"][l, h], out["K_out"][l, h], out["V_out"][l, h],
                                    gpu_diag=out["diag"][l, h], gpu_delta=out["delta"][l, h], gpu_scores=out["scores"][l, h],
                                    variant=variant)
            reps.append(rep)
    checked = [r for r in reps if r.v_checked]
    swapped = sum(r.swaps > 0 for r in reps)
    ambiguous = sum(r.ambiguous for r in reps)
    print(f"[{cfg.name} seed {seed}] heads {len(reps)}: value-checked {len(checked)}, index swaps inside the 1e-6 allowance "
          f"{swapped}, rank-ambiguous {ambiguous}")
    # every head must reach the value check unless it is excused by name: a tolerated index swap or a singular value
    # within a decade of a rank threshold
    assert len(checked) == len(reps) - sum((r.swaps > 0) or r.ambiguous for r in reps), "a head skipped the value check unexcused"
    assert len(checked) >= max(1, len(reps) // 2), "too few heads reached the value check"
    if expect_active is True:
        assert any(r.skipped == 0 for r in checked), "no head exercised the back-fill"
    if expect_active is False:
        assert all(r.skipped == 1 for r in checked)
    return reps


def test_config1_tiny_fp32(gpu):
    _check_cfg(gpu, si.CONFIGS["1"], expect_active=False)       # B = d: retained span is R^d


def test_config1_shadow_fp32(gpu):
    _check_cfg(gpu, si.CONFIGS["1s"], expect_active=True)


def test_config2_shape_one_layer(gpu):
    _check_cfg(gpu, si.shrink(si.CONFIGS["2"], n_layers=1), expect_active=False)


def test_config2_shadow_one_layer(gpu):
    _check_cfg(gpu, si.shrink(si.CONFIGS["2s"], n_layers=1), expect_active=True)


def test_config3_shape_four_heads(gpu):
    _check_cfg(gpu, si.shrink(si.CONFIGS["3"], n_layers=1, n_kv_heads=4), expect_active=False)


def test_config3_shadow_four_heads(gpu):
    _check_cfg(gpu, si.shrink(si.CONFIGS["3s"], n_layers=1, n_kv_heads=4), expect_active=True)


def test_config4_shape_two_heads(gpu):
    _check_cfg(gpu, si.shrink(si.CONFIGS["4"], n_layers=1, n_kv_heads=2), expect_active=False)


def test_config4_shadow_two_heads(gpu):
    _check_cfg(gpu, si.shrink(si.CONFIGS["4s"], n_layers=1, n_kv_heads=2), expect_active=True)


def test_config5_shape_ragged_budgets(gpu):
    cfg = si.shrink(si.CONFIGS["5"], n_layers=1, n_kv_heads=3)
    _check_cfg(gpu, cfg, seed=1, expect_active=False)


def test_config5_shadow_ragged_budgets(gpu):
    cfg = si.shrink(si.CONFIGS["5s"], n_layers=1, n_kv_heads=3)
    _check_cfg(gpu, cfg, seed=2, expect_active=True)


def test_paper_shape(gpu):
    _check_cfg(gpu, si.shrink(si.CONFIGS["paper"], n_layers=2), expect_active=True)


@pytest.mark.parametrize("seed,rank,budget", [(1, 2, 32), (3, 8, 32), (4, 4, 16), (5, 1, 24), (6, 12, 20)])
def test_wide_complement_few_leading_directions(gpu, seed, rank, budget):
    """Complements 96 to 112 wide with 1 to 12 back-fill directions: the regime in which the eigen-iteration may stop as
    soon as the leading eigenpairs have separated from the rest (and the one in which it keeps no eigenvector matrix)."""
    cfg = si.shrink(si.CONFIGS["paper"], n_layers=3, budget=budget, name=f"paper-r{rank}-b{budget}")
    _check_cfg(gpu, cfg, seed=seed, rank=rank, expect_active=True)


@pytest.mark.parametrize("N,d,dtype,g,W,B,rank", [
    (1000, 64, "bf16", 3, 8, 40, 3),        # ragged tail, odd group, d = 64
    (777, 128, "f32", 1, 5, 100, 2),        # fp32 at d = 128, rows not a multiple of anything
    (1, 64, "f32", 1, 1, 1, 2),             # a single token
    (513, 128, "bf16", 2, 16, 20, 40),      # rank above the complement's dimension is capped
    (4099, 128, "bf16", 4, 32, 130, 4),     # budget just above head_dim
    (31, 128, "bf16", 4, 32, 8, 2),         # less than one 32-token tile: three of the four score waves have nothing to do
    (97, 128, "bf16", 4, 32, 20, 2),        # one-launch score kernel, ragged fourth tile
    (768, 128, "bf16", 4, 32, 50, 2),       # the longest prompt of the one-launch score kernel
    (769, 128, "bf16", 4, 32, 50, 2),       # the shortest of the two-launch one
])
def test_ragged_shapes(gpu, N, d, dtype, g, W, B, rank):
    cfg = si.RelayConfig("ragged", 7, 1, 2, g, d, N, W, B, rank, dtype, "structured", outlier_frac=0.01)
    _check_cfg(gpu, cfg)


@pytest.mark.parametrize("d,dtype,budgets", [
    (128, "bf16", [16, 33, 64, 96, 97, 112, 127, 128]),     # every tile width of the small-budget basis kernel, n == d,
                                                            # complements wider than 90 (second finalisation launch)
    (64, "f32", [8, 31, 33, 64]),                           # head_dim 64, fp32 I/O
    (128, "f32", [20, 100, 120, 129]),                      # fp32 at head_dim 128, one head just above d
])
def test_small_budget_basis_variants(gpu, d, dtype, budgets):
    cfg = si.RelayConfig("smallb", 11, 1, len(budgets), 2, d, 1500, 8, 0, 4, dtype, "structured", outlier_frac=0.01)
    reps = _check_cfg(gpu, cfg, budgets=budgets, max_budget=max(budgets))
    assert sum(r.skipped == 0 for r in reps) >= len(budgets) // 2


@pytest.mark.parametrize("budget", [48, 300])
def test_rank_deficient_retained_rows(gpu, budget):
    """Values that repeat 24 distinct rows (plus a few free tokens): the retained span has rank far below both the
    budget and head_dim, on the small-budget kernel (48 rows) and on the general one (300 rows)."""
    cfg = si.RelayConfig("rankdef", 12, 1, 4, 2, 128, 1200, 8, budget, 4, "bf16", "structured")

    def edit(K, V, Q):
        N = V.shape[2]
        free = np.arange(N) % 97 == 5                      # every 97th token keeps its own value row
        for h in range(V.shape[1]):
            rep = V[0, h, :24].copy()
            tiled = rep[np.arange(N) % 24]
            V[0, h] = np.where(free[:, None], V[0, h], tiled)

    reps = _check_cfg(gpu, cfg, edit=edit)
    assert all(r.r_keep < 128 for r in reps)


def test_rank_deficient_large_budget_uses_partial_gram_sums(gpu):
    """More than 2048 retained rows of rank-deficient values on ten heads (two plain ones among them): the certificate
    cannot settle the eight-plus deficient heads, the first eight of them get their double-precision Gram matrix as
    sixteen partial sums from as many workgroups, the others compute it alone; all must agree with the oracle."""
    cfg = si.RelayConfig("rankdef-big", 13, 1, 10, 2, 128, 6000, 8, 2200, 4, "bf16", "structured")

    def edit(K, V, Q):
        N = V.shape[2]
        free = np.arange(N) % 211 == 7
        for h in range(V.shape[1]):
            if h in (3, 6):
                continue                                   # ordinary heads: full rank, certified
            rep = V[0, h, :24 + h].copy()                  # rank 24 + h (+ the free rows' directions)
            tiled = rep[np.arange(N) % (24 + h)]
            V[0, h] = np.where(free[:, None], V[0, h], tiled)

    reps = _check_cfg(gpu, cfg, edit=edit)
    assert sum(r.r_keep < 128 for r in reps) == 8 and sum(r.r_keep == 128 for r in reps) == 2


def test_few_active_heads_among_many_certified_ones(gpu):
    """256 heads of 16K tokens with budgets above head_dim, twelve of them rank-deficient: the certificate settles the
    other 244, and the statistics launch (whose full grid would be 4096 workgroups) finds the twelve on the device, in
    eight rows of workgroups that take more than one head each."""
    cfg = si.RelayConfig("few-active", 14, 32, 8, 1, 128, 16384, 8, 2100, 4, "bf16", "structured")
    special = {5, 77, 130, 131, 200, 255, 16, 17, 18, 100, 180, 254}

    def edit(K, V, Q):
        N = V.shape[2]
        free = np.arange(N) % 509 == 3
        for hh in special:
            l, h = divmod(hh, V.shape[1])
            rep = V[l, h, :40].copy()
            V[l, h] = np.where(free[:, None], V[l, h], rep[np.arange(N) % 40])

    reps = _check_cfg(gpu, cfg, edit=edit)
    low = [i for i, r in enumerate(reps) if r.r_keep is not None and r.r_keep < 128]
    assert set(low) == special


def test_budget_edges_and_rank_zero(gpu):
    cfg = si.RelayConfig("edge", 8, 1, 4, 2, 64, 300, 8, 0, 2, "bf16", "structured")
    _check_cfg(gpu, cfg, budgets=[0, 300, 1000, 17], max_budget=300)
    reps = _check_cfg(gpu, cfg, budgets=[5, 30, 63, 17], rank=0)
    assert all(r.skipped == 1 for r in reps)


def test_all_ties_keep_lowest_indices(gpu):
    cfg = si.RelayConfig("ties", 9, 1, 2, 2, 64, 640, 4, 50, 2, "bf16", "structured")
    K, V, Q = si.make_cache(cfg, 0)
    Q[:] = 0                                   # every logit is zero: all scores equal
    out = gpu.run_fused(cfg, K, V, Q, budget=50)
    for h in range(2):
        assert out["idx"][0, h].tolist() == list(range(50))
    # 640 equal scores straddle the threshold: more than the re-decision takes, and the call says so per head
    from paper_2604_13349_amd import binding as Bd
    assert np.all(out["diag"]["select_flags"] == Bd.OBF_SELECT_BAND_OVERFLOW)
    cfg2 = si.shrink(si.CONFIGS["2s"], n_layers=1)
    K2, V2, Q2 = si.make_cache(cfg2, 0, threads=8)
    assert np.all(gpu.run_fused(cfg2, K2, V2, Q2, budget=cfg2.budget)["diag"]["select_flags"] == 0)


def test_fused_equals_staged_and_is_deterministic(gpu):
    import torch
    from paper_2604_13349_amd import binding as Bd
    cfg = si.shrink(si.CONFIGS["2s"], n_layers=1, n_kv_heads=4)
    K, V, Q = si.make_cache(cfg, 3)
    Kd, Vd, Qd = (gpu.to_dev(x, cfg.dtype) for x in (K, V, Q))
    a = Bd.compress_relay(Kd, Vd, Qd, budget=cfg.budget, rank=cfg.rank, want_scores=True, want_delta=True)
    b = Bd.compress_relay(Kd, Vd, Qd, budget=cfg.budget, rank=cfg.rank, want_scores=True, want_delta=True)
    for k in ("K_out", "V_out", "idx", "n_keep", "scores", "delta"):
        assert torch.equal(a[k].view(torch.uint8), b[k].view(torch.uint8)), f"run-to-run difference in {k}"
    sh = Bd.shape_of(Kd, Qd)
    scores, lse = Bd.score(Kd, Qd)
    idx, n_keep = Bd.select_topk(sh, scores, budget=cfg.budget)
    Bd.refine_boundary(Kd, Qd, scores, lse, idx, n_keep)
    K_out, V_out = Bd.gather(sh, Kd, Vd, idx, n_keep)
    delta = torch.empty((1, 4, cfg.head_dim), dtype=torch.float32, device="cuda")
    Bd.backfill(sh, Vd, scores, idx, n_keep, cfg.rank, V_out, delta_out=delta)
    torch.cuda.synchronize()
    assert torch.equal(scores, a["scores"]) and torch.equal(idx, a["idx"]) and torch.equal(n_keep, a["n_keep"])
    assert torch.equal(K_out.view(torch.int16), a["K_out"].view(torch.int16))
    assert torch.equal(V_out.view(torch.int16), a["V_out"].view(torch.int16))
    assert torch.equal(delta, a["delta"])
    # the same for the variant entry points: obf_backfill_variant on staged inputs == obf_compress_relay_variant
    var = Bd.make_variant(no_scaling=True, attn_inject=True, subspace="evr", evr_tau=0.5)
    c = Bd.compress_relay(Kd, Vd, Qd, budget=cfg.budget, rank=cfg.rank, want_delta=True, variant=var)
    K_out, V_out = Bd.gather(sh, Kd, Vd, idx, n_keep)
    Bd.backfill(sh, Vd, scores, idx, n_keep, cfg.rank, V_out, delta_out=delta, variant=var)
    torch.cuda.synchronize()
    assert torch.equal(V_out.view(torch.int16), c["V_out"].view(torch.int16)) and torch.equal(delta, c["delta"])
    assert not torch.equal(c["V_out"].view(torch.int16), a["V_out"].view(torch.int16))


def test_large_fused_call_equals_the_stage_calls(gpu):
    """72 heads of 16K tokens (288 MiB of keys) with a budget below head_dim: the fused call is bit-identical to the stage
    calls in sequence, and a head from each end of the cache matches the oracle."""
    import torch
    from paper_2604_13349_amd import binding as Bd
    cfg = si.RelayConfig("large", 71, 9, 8, 4, 128, 16384, 8, 96, 4, "bf16", "structured", outlier_frac=0.01)   # 72 heads, 288 MiB of K
    K, V, Q = si.make_cache(cfg, 1, threads=8)
    Kd, Vd, Qd = (gpu.to_dev(x, cfg.dtype) for x in (K, V, Q))
    a = Bd.compress_relay(Kd, Vd, Qd, budget=cfg.budget, rank=cfg.rank, want_scores=True, want_delta=True)
    sh = Bd.shape_of(Kd, Qd)
    scores, lse = Bd.score(Kd, Qd)
    idx, n_keep = Bd.select_topk(sh, scores, budget=cfg.budget)
    Bd.refine_boundary(Kd, Qd, scores, lse, idx, n_keep)
    K_out, V_out = Bd.gather(sh, Kd, Vd, idx, n_keep)
    delta = torch.empty((cfg.n_layers, cfg.n_kv_heads, cfg.head_dim), dtype=torch.float32, device="cuda")
    Bd.backfill(sh, Vd, scores, idx, n_keep, cfg.rank, V_out, delta_out=delta)
    torch.cuda.synchronize()
    assert torch.equal(scores, a["scores"]) and torch.equal(idx, a["idx"]) and torch.equal(n_keep, a["n_keep"])
    assert torch.equal(K_out.view(torch.int16), a["K_out"].view(torch.int16))
    assert torch.equal(V_out.view(torch.int16), a["V_out"].view(torch.int16)) and torch.equal(delta, a["delta"])
    assert bool(delta.abs().sum() > 0)
    # and against the oracle on a head of each chunk
    out = {k: (gpu.to_host(a[k], cfg.dtype) if k in ("K_out", "V_out") else a[k].cpu().numpy()) for k in ("K_out", "V_out", "idx", "n_keep", "scores", "delta")}
    for (l, h) in ((0, 3), (8, 7)):
        ref = O.compress_head(K[l, h], V[l, h], Q[l, h * cfg.group:(h + 1) * cfg.group], cfg.budget, cfg.rank, cfg.dtype)
        rep = parity.check_head(f"large[{l},{h}]", ref, K[l, h], V[l, h], cfg.dtype, cfg.budget, out["idx"][l, h], out["n_keep"][l, h],
                                out["K_out"][l, h], out["V_out"][l, h], gpu_delta=out["delta"][l, h], gpu_scores=out["scores"][l, h])
        assert rep.v_checked or rep.swaps or rep.ambiguous


def test_select_stage_is_exact_on_given_scores(gpu):
    import torch
    from paper_2604_13349_amd import binding as Bd
    rng = np.random.default_rng(5)
    N = 5000
    s = np.empty((1, 4, N), dtype=np.float32)
    s[0, 0] = rng.random(N).astype(np.float32)
    s[0, 1] = np.round(rng.random(N) * 8).astype(np.float32) / 8           # many exact ties
    s[0, 2] = rng.standard_normal(N).astype(np.float32)                    # negatives
    s[0, 2, ::7] = 0.0
    s[0, 2, 3::7] = -0.0
    s[0, 3] = 1.0
    sh = Bd.make_shape(1, 4, 1, 64, N, 1, "bf16")
    for budgets in ([1, 77, 2500, 4999], [5000, 0, 13, 700]):
        idx, n_keep = Bd.select_topk(sh, torch.from_numpy(s).cuda(), budgets=budgets, max_budget=5000)
        torch.cuda.synchronize()
        idx, n_keep = idx.cpu().numpy(), n_keep.cpu().numpy()
        for h in range(4):
            b = budgets[h]
            # the decision is taken on the fp32 values by both sides; -0 orders below +0 as bit patterns
            key = s[0, h].astype(np.float64)
            key = np.where((s[0, h] == 0) & np.signbit(s[0, h]), -1e-300, key)
            ref = O.select_topk(key, b)
            assert n_keep[0, h] == b and np.array_equal(idx[0, h, :b], ref), f"head {h} budget {b}"
            assert np.all(idx[0, h, b:] == -1)


# --------------------------------------------------------------------------- full sizes, sampled heads
def _full_size(gpu, name, seed, sample, expect_active):
    """The whole named config through the fused call (the launch configuration bench.py times);
    the oracle checks a sample of heads one by one, every head is checked for structure."""
    cfg = si.CONFIGS[name]
    K, V, Q = si.make_cache(cfg, seed, threads=16)
    bud = si.budgets(cfg, seed)
    out = gpu.run_fused(cfg, K, V, Q, budgets=bud, rank=cfg.rank)
    L, H, N = cfg.n_layers, cfg.n_kv_heads, cfg.n_tokens
    nk = np.minimum(bud, N)
    assert np.array_equal(out["n_keep"], nk)
    for l in range(L):
        for h in range(H):
            b = int(nk[l, h])
            ix = out["idx"][l, h]
            assert np.all(np.diff(ix[:b]) > 0) and ix[0] >= 0 and ix[b - 1] < N and np.all(ix[b:] == -1)
            assert abs(float(out["scores"][l, h].sum(dtype=np.float64)) - cfg.rows) < 1e-3 * cfg.rows   # Eq. 1: rows sum to one
    rng = np.random.default_rng(1234 + seed)
    heads = [(int(l), int(h)) for l, h in zip(rng.integers(0, L, sample), rng.integers(0, H, sample))]
    heads += [(0, 0), (L - 1, H - 1)]
    active = 0
    reps = []
    for (l, h) in heads:
        ref = O.compress_head(K[l, h], V[l, h], Q[l, h * cfg.group:(h + 1) * cfg.group], int(bud[l, h]), cfg.rank, cfg.dtype)
        rep = parity.check_head(f"{name}[{l},{h}]", ref, K[l, h], V[l, h], cfg.dtype, int(bud[l, h]),
                                out["idx"][l, h], out["n_keep"][l, h], out["K_out"][l, h], out["V_out"][l, h],
                                gpu_diag=out["diag"][l, h], gpu_delta=out["delta"][l, h], gpu_scores=out["scores"][l, h])
        active += int(rep.skipped == 0)
        reps.append(rep)
    print(f"[{name} seed {seed}] oracle heads {len(reps)}: value-checked {sum(r.v_checked for r in reps)}, index swaps inside "
          f"the 1e-6 allowance {sum(r.swaps > 0 for r in reps)}, rank-ambiguous {sum(r.ambiguous for r in reps)}")
    assert sum(r.v_checked for r in reps) >= 2, "fewer than two heads reached the value check"
    if expect_active:
        assert active > 0
    else:
        assert active == 0 and int((out["diag"]["skipped"] == 0).sum()) == 0


def test_full_config2(gpu):
    _full_size(gpu, "2", 0, 10, False)


def test_full_config3(gpu):
    _full_size(gpu, "3", 0, 8, False)


def test_full_config3_shadow(gpu):
    _full_size(gpu, "3s", 0, 6, True)


def test_full_config4(gpu):
    _full_size(gpu, "4", 0, 4, False)


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_full_config5_every_handoff(gpu, seed):
    """Config 5 is four hand-offs with per-agent seeds 0-3: each one at full size, with its own ragged budgets."""
    _full_size(gpu, "5", seed, 2 if seed != 1 else 3, False)


def test_full_paper_shape(gpu):
    _full_size(gpu, "paper", 0, 16, True)


# --------------------------------------------------------------------------- boundary refinement really decides
def _bf16_next_toward_zero(bits):
    """The neighbouring bf16 value with smaller magnitude (bit pattern arithmetic on the magnitude)."""
    return np.uint16(bits - 1) if (bits & 0x7FFF) != 0 else bits


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64)])
def test_near_tie_at_threshold_is_decided_exactly(gpu, dtype, d):
    """Two tokens whose exact masses differ by less than fp32 can resolve straddle the budget boundary; the
    lower index is the (slightly) lighter one, so an fp32 tie-break would keep the wrong token."""
    cfg = si.RelayConfig("neartie", 11, 1, 1, 2, d, 1536, 16, 150, 0, dtype, "structured")
    K, V, Q = si.make_cache(cfg, 0)
    Kh = K[0, 0]
    ref0 = O.compress_head(Kh, V[0, 0], Q[0, 0:cfg.group], cfg.budget, 0, dtype)
    order = np.argsort(-ref0.A, kind="stable")
    a = int(order[cfg.budget - 1])                     # the last retained token
    dropped = [int(j) for j in order[cfg.budget + 20:] if j < a]
    assert dropped, "need a dropped token at a lower index"
    p = dropped[0]
    found = False
    for c in np.argsort(np.abs(O.decode(Kh[a], dtype))):       # smallest components first: smallest nudges
        row = Kh[a].copy()
        if dtype == "bf16":
            row[c] = _bf16_next_toward_zero(row[c])
        else:
            row[c] = np.nextafter(row[c], np.float32(0.0))
        Kt = Kh.copy(); Kt[p] = row
        A = O.attention_mass(O.decode(Kt, dtype), O.decode(Q[0, 0:cfg.group], dtype).reshape(-1, d))
        rel = (A[a] - A[p]) / A[a]
        if 1e-9 < rel < 2e-7:                          # lighter by less than an fp32 ulp of the score
            srt = np.sort(A)[::-1]
            if srt[cfg.budget - 2] > A[a] * (1 + 1e-5) and srt[cfg.budget + 1] < A[p] * (1 - 1e-5):
                found = True
                break
    assert found, "could not build a near tie"
    K2 = K.copy(); K2[0, 0] = Kt
    ref = O.compress_head(Kt, V[0, 0], Q[0, 0:cfg.group], cfg.budget, 0, dtype)
    assert a in ref.idx and p not in ref.idx
    out = gpu.run_fused(cfg, K2, V, Q, budget=cfg.budget, rank=0)
    assert np.array_equal(out["idx"][0, 0], ref.idx), "fused call: near tie decided differently from exact arithmetic"
    # the staged calls give the same list
    import torch
    from paper_2604_13349_amd import binding as Bd
    Kd, Qd = gpu.to_dev(K2, dtype), gpu.to_dev(Q, dtype)
    sh = Bd.shape_of(Kd, Qd)
    scores, lse = Bd.score(Kd, Qd)
    idx, n_keep = Bd.select_topk(sh, scores, budget=cfg.budget)
    plain = idx.cpu().numpy()[0, 0].copy()
    Bd.refine_boundary(Kd, Qd, scores, lse, idx, n_keep)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy()[0, 0], ref.idx)
    print("fp32 selection alone agreed with exact arithmetic:", bool(np.array_equal(plain, ref.idx)))


# --------------------------------------------------------------------------- layerwise granularity (Sec. 4.3.2)
def _check_layerwise(gpu, cfg, seed=0, budgets=None, rank=None, variant=None):
    """obf_compress_relay_layerwise against oracle.compress_layer: the shared index set must be the oracle's (the exact
    re-decision at the threshold is part of the call), every head then goes through the per-head checks."""
    K, V, Q = si.make_cache(cfg, seed, threads=8)
    L, H = cfg.n_layers, cfg.n_kv_heads
    bud = np.full(L, cfg.budget, dtype=np.int32) if budgets is None else np.asarray(budgets, dtype=np.int32)
    rank = cfg.rank if rank is None else rank
    out = gpu.run_fused(cfg, K, V, Q, budgets=bud, rank=rank, max_budget=int(min(bud.max(), cfg.n_tokens)), layerwise=True,
                        variant=None if variant is None else _gpu_variant(variant))
    active = 0
    for l in range(L):
        idx, heads = O.compress_layer(K[l], V[l], Q[l], int(bud[l]), rank, cfg.group, cfg.dtype,
                                      *(() if variant is None else (variant,)))
        n = len(idx)
        for h in range(H):
            assert int(out["n_keep"][l, h]) == n
            assert out["idx"][l, h, :n].tolist() == idx.tolist(), f"layer {l} head {h}: shared index set differs"
            rep = parity.check_head(f"{cfg.name}-L[{l},{h}]", heads[h], K[l, h], V[l, h], cfg.dtype, int(bud[l]),
                                    out["idx"][l, h], out["n_keep"][l, h], out["K_out"][l, h], out["V_out"][l, h],
                                    gpu_diag=out["diag"][l, h], gpu_delta=out["delta"][l, h], gpu_scores=out["scores"][l, h],
                                    variant=variant)
            active += int(rep.skipped == 0)
    return active


def test_layerwise_config2_shape(gpu):
    cfg = si.shrink(si.CONFIGS["2"], n_layers=2)
    assert _check_layerwise(gpu, cfg) == 0                  # budget above head_dim: plain layerwise eviction


def test_layerwise_shadow_budget_runs_backfill(gpu):
    cfg = si.shrink(si.CONFIGS["2s"], n_layers=2)
    assert _check_layerwise(gpu, cfg, rank=4) > 0           # L-OBF: pca_rank 4 (Sec. 5)


def test_layerwise_paper_shape_and_ragged_layer_budgets(gpu):
    cfg = si.shrink(si.CONFIGS["paper"], n_layers=3)
    assert _check_layerwise(gpu, cfg, budgets=[32, 7, 200], rank=4) > 0


def test_layerwise_fp32_head_dim_64(gpu):
    cfg = si.RelayConfig("lw64", 13, 2, 3, 2, 64, 700, 8, 40, 4, "f32", "structured", outlier_frac=0.01)
    assert _check_layerwise(gpu, cfg) > 0


def test_layerwise_with_one_head_equals_headwise(gpu):
    cfg = si.RelayConfig("lw1", 14, 3, 1, 4, 128, 900, 16, 60, 2, "bf16", "structured")
    K, V, Q = si.make_cache(cfg, 0, threads=8)
    a = gpu.run_fused(cfg, K, V, Q, budget=60)
    b = gpu.run_fused(cfg, K, V, Q, budget=60, layerwise=True)
    for k in ("idx", "n_keep", "K_out", "V_out", "delta"):
        assert np.array_equal(a[k], b[k]), k


def test_layerwise_near_tie_at_threshold_is_decided_exactly(gpu):
    """A near tie of the LAYER mass (sum over three heads) at the budget boundary, built by nudging one key row of one
    head: the lower index is the lighter token by less than fp32 resolves, so only the exact multi-head
    re-decision keeps the right one."""
    dtype, d, H = "bf16", 128, 3
    cfg = si.RelayConfig("lwtie", 15, 1, H, 2, d, 1536, 16, 150, 0, dtype, "structured")
    K, V, Q = si.make_cache(cfg, 0)

    def layer_mass(Kl):
        tot = np.zeros(cfg.n_tokens)
        for h in range(H):
            tot = tot + O.attention_mass(O.decode(Kl[h], dtype), O.decode(Q[0, h * cfg.group:(h + 1) * cfg.group], dtype).reshape(-1, d))
        return tot

    A0 = layer_mass(K[0])
    order = np.argsort(-A0, kind="stable")
    a = int(order[150])                                # a token of middling mass; the budget is set below
    found = False
    budget = 0
    for p in [int(j) for j in order[170:600] if j < a][:6]:
        # make token p a copy of token a in every head, then nudge one component of one head's copy
        Kt = K[0].copy()
        Kt[:, p] = Kt[:, a]
        for c in np.argsort(np.abs(O.decode(Kt[0, a], dtype)))[:60]:
            Kn = Kt.copy()
            Kn[0, p, c] = _bf16_next_toward_zero(Kn[0, p, c])
            A = layer_mass(Kn)
            rel = (A[a] - A[p]) / A[a]
            if 1e-9 < rel < 2e-7:
                srt = np.argsort(-A, kind="stable")
                ra = int(np.nonzero(srt == a)[0][0])
                if int(srt[ra + 1]) == p and A[srt[ra - 1]] > A[a] * (1 + 1e-5) and A[srt[ra + 2]] < A[p] * (1 - 1e-5):
                    budget = ra + 1                    # a is the last retained token, p the first dropped one
                    found = True
                    break
        if found:
            break
    assert found, "could not build a near tie of the layer mass"
    K2 = K.copy(); K2[0] = Kn
    idx, _ = O.compress_layer(K2[0], V[0], Q[0], budget, 0, cfg.group, dtype)
    assert a in idx and p not in idx
    out = gpu.run_fused(cfg, K2, V, Q, budget=budget, rank=0, layerwise=True)
    for h in range(H):
        assert np.array_equal(out["idx"][0, h], idx), "layerwise call: near tie decided differently from exact arithmetic"


# --------------------------------------------------------------------------- ablation variants (App. D)
VARIANTS = {
    "no_projection": O.Variant(no_projection=True),
    "max_p": O.Variant(subspace="all"),
    "no_scaling": O.Variant(no_scaling=True),
    "naive": O.Variant(naive=True),
    "attn_inject": O.Variant(attn_inject=True),
    "evr_0.35": O.Variant(subspace="evr", evr_tau=0.35),
    "evr_0.8": O.Variant(subspace="evr", evr_tau=0.8),
    "no_projection+no_scaling+attn_inject": O.Variant(no_projection=True, no_scaling=True, attn_inject=True),
    "fast_path_3": O.Variant(subspace_iters=3),
    "fast_path_1+no_projection": O.Variant(subspace_iters=1, no_projection=True),
    "fast_path_6+attn_inject": O.Variant(subspace_iters=6, attn_inject=True),
}


@pytest.mark.parametrize("name", list(VARIANTS))
def test_variants_headwise_small_budget(gpu, name):
    """Each ablation of App. D through obf_compress_relay_variant on the paper-shaped shadow cache (budget below head_dim:
    every head runs the back-fill) against the oracle with the same flag."""
    reps = _check_cfg(gpu, si.shrink(si.CONFIGS["paper"], n_layers=1), variant=VARIANTS[name])
    assert sum(r.skipped == 0 for r in reps if r.v_checked) >= len(reps) // 2


@pytest.mark.parametrize("name", ["no_projection", "naive", "attn_inject"])
def test_variants_headwise_budget_above_head_dim(gpu, name):
    """Budget above head_dim on 8K-token bf16 heads: the method itself skips every head here (the retained span is everything);
    the two variants without Eq. 3 still inject, the third stays skipped."""
    cfg = si.shrink(si.CONFIGS["3"], n_layers=1, n_kv_heads=2)
    reps = _check_cfg(gpu, cfg, variant=VARIANTS[name])
    want_active = name != "attn_inject"
    assert all((r.skipped == 0) == want_active for r in reps if r.v_checked)


@pytest.mark.parametrize("name", ["max_p", "evr_0.35", "no_scaling"])
def test_variants_layerwise(gpu, name):
    """App. D ablates L-OBF: the same flags under the layerwise retention rule."""
    cfg = si.shrink(si.CONFIGS["2s"], n_layers=2)
    assert _check_layerwise(gpu, cfg, rank=4, variant=VARIANTS[name]) > 0


def test_variant_null_and_default_equal_the_plain_call(gpu):
    cfg = si.shrink(si.CONFIGS["2s"], n_layers=1)
    K, V, Q = si.make_cache(cfg, 0, threads=8)
    from paper_2604_13349_amd import binding as B
    a = gpu.run_fused(cfg, K, V, Q, budget=cfg.budget)
    b = gpu.run_fused(cfg, K, V, Q, budget=cfg.budget, variant=B.make_variant())
    for k in ("K_out", "V_out", "idx", "n_keep", "delta"):
        assert np.array_equal(a[k], b[k]), k


def test_variant_argument_errors(gpu):
    cfg = si.shrink(si.CONFIGS["1s"], n_layers=1)
    K, V, Q = si.make_cache(cfg, 0, threads=8)
    from paper_2604_13349_amd import binding as B
    for bad in (B.make_variant(subspace=7), B.make_variant(subspace="evr", evr_tau=0.0), B.make_variant(subspace="evr", evr_tau=1.5)):
        with pytest.raises(B.ObfError):
            gpu.run_fused(cfg, K, V, Q, budget=cfg.budget, variant=bad)


# --------------------------------------------------------------------------- relay assembly (Sec. 3.3, Sec. 4.3.2)
def _check_window(gpu, cfg, sink, pad, seed=0, budget=None, rank=None, layerwise=False, variant=None):
    """obf_compress_relay_window on right-padded storage (pad rows of junk behind every head) with a protected sink,
    against the oracle on the real tokens."""
    K, V, Q = si.make_cache(cfg, seed, threads=8)
    L, H, N, d = K.shape
    junk = np.random.default_rng(99)

    def padded(a):
        out = np.empty((L, H, N + pad, d), dtype=a.dtype)
        out[:, :, :N] = a
        if pad:
            fill = junk.integers(0, 0x7F00, size=(L, H, pad, d)).astype(np.uint16)      # finite bf16 bit patterns
            out[:, :, N:] = fill if a.dtype == np.uint16 else fill.astype(np.float32)
        return out

    budget = cfg.budget if budget is None else budget
    rank = cfg.rank if rank is None else rank
    out = gpu.run_fused(cfg, padded(K), padded(V), Q, budget=budget, rank=rank, max_budget=min(budget, N - sink),
                        layerwise=layerwise, variant=None if variant is None else _gpu_variant(variant), n_tokens=N, sink=sink)
    var = () if variant is None else (variant,)
    active = 0
    for l in range(L):
        if layerwise:
            idx, heads = O.compress_layer(K[l], V[l], Q[l], budget, rank, cfg.group, cfg.dtype, *(var or (O.Variant(),)), sink)
        for h in range(H):
            if layerwise:
                ref = heads[h]
                assert out["idx"][l, h, :len(idx)].tolist() == idx.tolist()
            else:
                ref = O.compress_head(K[l, h], V[l, h], Q[l, h * cfg.group:(h + 1) * cfg.group], budget, rank, cfg.dtype,
                                      *(var or (O.Variant(),)), sink)
            rep = parity.check_head(f"{cfg.name}-win[{l},{h}]", ref, K[l, h], V[l, h], cfg.dtype, budget,
                                    out["idx"][l, h], out["n_keep"][l, h], out["K_out"][l, h], out["V_out"][l, h],
                                    gpu_diag=out["diag"][l, h], gpu_delta=out["delta"][l, h], gpu_scores=out["scores"][l, h],
                                    variant=variant, sink=sink)
            active += int(rep.skipped == 0 and rep.v_checked)
    return active


@pytest.mark.parametrize("sink,pad", [(4, 0), (4, 37), (0, 64), (3, 5)])
def test_window_paper_shape(gpu, sink, pad):
    # sink_size = 4 is the paper's setting (App. A.1); 3 makes the score view misaligned for 16-byte loads
    assert _check_window(gpu, si.shrink(si.CONFIGS["paper"], n_layers=2), sink, pad) > 0


def test_window_mfma_score_path_ragged_length(gpu):
    cfg = si.RelayConfig("win", 21, 1, 3, 4, 128, 2000 + 13, 32, 96, 4, "bf16", "structured", outlier_frac=0.01)
    assert _check_window(gpu, cfg, sink=4, pad=51) > 0


def test_window_budget_above_head_dim_and_fp32(gpu):
    cfg = si.RelayConfig("win", 22, 1, 2, 4, 128, 1500, 32, 300, 4, "bf16", "structured")
    _check_window(gpu, cfg, sink=4, pad=20)
    cfg = si.RelayConfig("win", 23, 1, 2, 2, 64, 700, 8, 40, 2, "f32", "structured")
    assert _check_window(gpu, cfg, sink=2, pad=9) > 0


def test_window_layerwise_and_variant(gpu):
    cfg = si.shrink(si.CONFIGS["2s"], n_layers=2)
    assert _check_window(gpu, cfg, sink=4, pad=12, rank=4, layerwise=True) > 0
    assert _check_window(gpu, si.shrink(si.CONFIGS["paper"], n_layers=1), sink=4, pad=3, variant=VARIANTS["no_projection"]) > 0


def test_window_budget_above_eligible_count_and_errors(gpu):
    cfg = si.RelayConfig("win", 24, 1, 2, 2, 64, 50, 8, 100, 2, "f32", "structured")
    _check_window(gpu, cfg, sink=4, pad=6)                  # keeps tokens 4 .. 49
    from paper_2604_13349_amd import binding as B
    K, V, Q = si.make_cache(cfg, 0, threads=8)
    for bad in (dict(n_tokens=51), dict(sink=50), dict(sink=-1)):
        with pytest.raises(B.ObfError):
            gpu.run_fused(cfg, K, V, Q, budget=10, **bad)


def test_append_message_matches_concatenation(gpu):
    """obf_append_message against the oracle's row concatenation: ragged inherited lengths and retained counts per head,
    one head that does not fit."""
    import torch
    from paper_2604_13349_amd import binding as B
    r = np.random.default_rng(5)
    heads, d = 6, 128
    prev_stride, keep_stride, n_gen, msg_stride = 40, 32, 7, 70
    prev_len = np.array([0, 40, 13, 25, 31, 40], dtype=np.int32)
    n_keep = np.array([32, 20, 0, 32, 32, 32], dtype=np.int32)        # head 5: 40 + 32 + 7 > 70
    mk = lambda rows: r.integers(0, 0x7F00, size=(heads, rows, d)).astype(np.uint16)
    parts = {k: mk(rows) for k, rows in (("pK", prev_stride), ("pV", prev_stride), ("kK", keep_stride), ("kV", keep_stride),
                                         ("gK", n_gen), ("gV", n_gen))}
    dev = {k: gpu.to_dev(v, "bf16") for k, v in parts.items()}
    mK, mV, mlen = B.append_message(dev["pK"], dev["pV"], torch.from_numpy(prev_len).cuda(), dev["kK"], dev["kV"],
                                    torch.from_numpy(n_keep).cuda(), dev["gK"], dev["gV"], msg_stride)
    torch.cuda.synchronize()
    mK, mV, mlen = gpu.to_host(mK, "bf16"), gpu.to_host(mV, "bf16"), mlen.cpu().numpy()
    for h in range(heads):
        wantK = O.append_message(parts["pK"][h, :prev_len[h]], parts["kK"][h, :n_keep[h]], parts["gK"][h])
        wantV = O.append_message(parts["pV"][h, :prev_len[h]], parts["kV"][h, :n_keep[h]], parts["gV"][h])
        if wantK.shape[0] > msg_stride:
            assert mlen[h] == -1 and not mK[h].any() and not mV[h].any()
            continue
        n = wantK.shape[0]
        assert mlen[h] == n
        assert np.array_equal(mK[h, :n], wantK) and np.array_equal(mV[h, :n], wantV)
        assert not mK[h, n:].any() and not mV[h, n:].any()
    # first agent: the inherited message is the sink, i.e. the first rows of the prompt cache itself (uniform length)
    mK, mV, mlen = B.append_message(dev["pK"], dev["pV"], None, dev["kK"], dev["kV"], torch.from_numpy(n_keep).cuda(),
                                    None, None, msg_stride, prev_len_all=4)
    torch.cuda.synchronize()
    mK, mlen = gpu.to_host(mK, "bf16"), mlen.cpu().numpy()
    for h in range(heads):
        want = O.append_message(parts["pK"][h, :4], parts["kK"][h, :n_keep[h]], parts["gK"][h, :0])
        assert mlen[h] == want.shape[0] and np.array_equal(mK[h, :want.shape[0]], want)
    with pytest.raises(B.ObfError):
        B.append_message(dev["pK"], dev["pV"], None, dev["kK"], dev["kV"], None, None, None, msg_stride, prev_len_all=41)


# --------------------------------------------------------------------------- HIP graph capture of the fused call
@pytest.mark.parametrize("name,layerwise,layers", [("2", False, 3), ("2s", False, 3), ("2s", True, 3), ("3", False, 8), ("3", False, 18),
                                                   ("3s", False, 18)])
def test_graph_capture_replays_match_eager(gpu, name, layerwise, layers):
    """The fused call is captured into a HIP graph (the small-budget shape forks the library's second stream for the
    bases, the config-3 shapes for the copy of the retained K rows, and both join inside the capture; the 18-layer shapes
    hold 300 MB of keys) and replayed
    several times with eager calls and synchronisations in between; every replay must reproduce the eager outputs bit
    for bit."""
    import torch
    from paper_2604_13349_amd import binding as Bd
    cfg = si.shrink(si.CONFIGS[name], n_layers=layers)
    K, V, Q = si.make_cache(cfg, 0, threads=8)
    Kd, Vd, Qd = gpu.to_dev(K, cfg.dtype), gpu.to_dev(V, cfg.dtype), gpu.to_dev(Q, cfg.dtype)
    out = None
    for _ in range(2):
        out = Bd.compress_relay(Kd, Vd, Qd, budget=cfg.budget, rank=cfg.rank, out=out, ws=(out or {}).get("ws"),
                                want_diag=True, want_delta=True, layerwise=layerwise)
    torch.cuda.synchronize()
    keys = ("idx", "n_keep", "K_out", "V_out", "delta", "diag")
    ref = {k: out[k].clone() for k in keys}

    def call():
        Bd.compress_relay(Kd, Vd, Qd, budget=cfg.budget, rank=cfg.rank, out=out, ws=out["ws"], want_diag=True,
                          want_delta=True, layerwise=layerwise)

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call()
    torch.cuda.synchronize()
    for rep in range(3):
        for k in keys:
            out[k].zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in keys:
            assert torch.equal(out[k], ref[k]), f"replay {rep}: {k} differs from the eager call"
        call()
        torch.cuda.synchronize()
        for k in keys:
            assert torch.equal(out[k], ref[k]), f"eager call after replay {rep}: {k} differs"


# --------------------------------------------------------------------------- the call a hot path makes: no optional output
@pytest.mark.parametrize("name,heads,expect_active", [("3", 6, False), ("3s", 6, True)])
def test_bare_call_without_optional_outputs(gpu, name, heads, expect_active):
    """The fused call with scores_out, delta_out and diag all NULL (the configuration the benchmark times): the scores
    stay in the workspace and the certificate skips its diagnostic sums; idx, K_out and V_out against the oracle."""
    from paper_2604_13349_amd import binding as Bd
    cfg = si.shrink(si.CONFIGS[name], n_layers=1, n_kv_heads=heads)
    K, V, Q = si.make_cache(cfg, 2, threads=8)
    o = Bd.compress_relay(gpu.to_dev(K, cfg.dtype), gpu.to_dev(V, cfg.dtype), gpu.to_dev(Q, cfg.dtype), budget=cfg.budget,
                          rank=cfg.rank)
    import torch
    torch.cuda.synchronize()
    assert "scores" not in o and "delta" not in o and "diag" not in o
    idx, nk = o["idx"].cpu().numpy(), o["n_keep"].cpu().numpy()
    Ko, Vo = gpu.to_host(o["K_out"], cfg.dtype), gpu.to_host(o["V_out"], cfg.dtype)
    reps = []
    for h in range(heads):
        ref = O.compress_head(K[0, h], V[0, h], Q[0, h * cfg.group:(h + 1) * cfg.group], cfg.budget, cfg.rank, cfg.dtype)
        reps.append(parity.check_head(f"bare {name}[{h}]", ref, K[0, h], V[0, h], cfg.dtype, cfg.budget, idx[0, h], nk[0, h],
                                      Ko[0, h], Vo[0, h], gpu_diag=None, gpu_delta=None))
    assert sum(r.v_checked for r in reps) >= heads - 1
    assert any(r.skipped == 0 for r in reps) == expect_active


@pytest.mark.parametrize("support,rank,k_want", [(44, 16, 4), (41, 8, 1), (40, 8, 0)])
def test_residual_rank_below_requested_rank(gpu, support, rank, k_want):
    """k = min(pca_rank, rank R) with rank R the smaller one (Sec. 4.4): the value rows live on the first `support`
    coordinates, the 40 retained rows span 40 of those dimensions, so the residual has rank support - 40 exactly
    (its further singular values are zero on both sides, far from either side's rank threshold); with support = 40
    nothing is left to inject."""
    cfg = si.RelayConfig("res-rank", 21, 1, 4, 2, 128, 900, 8, 40, rank, "bf16", "structured")

    def edit(K, V, Q):
        V[..., support:] = 0

    reps = _check_cfg(gpu, cfg, edit=edit)
    assert all(r.v_checked and not r.ambiguous for r in reps)
    if k_want == 0:
        assert all(r.skipped == 1 for r in reps)


def test_complement_projector_with_coinciding_columns(gpu):
    """Every seventh token carries a multiple of e_0 - e_1 as its value row and no other row touches those two
    coordinates: e_0 - e_1 lies in the retained span, e_0 + e_1 in its complement, so columns 0 and 1 of the projector
    onto the complement coincide and carry its largest diagonal entries (1/2 against about (d - r)/d).  A factorisation
    that takes the two leading columns in one step meets them as a pair, and the first leaves nothing of the second."""
    cfg = si.RelayConfig("twin-cols", 23, 1, 4, 2, 64, 600, 8, 58, 2, "f32", "structured")

    def edit(K, V, Q):
        twin = np.arange(V.shape[2]) % 7 == 3
        amp = V[..., twin, 0].copy()
        V[..., twin, :] = 0
        V[..., twin, 0] = amp
        V[..., twin, 1] = -amp
        V[..., ~twin, 0:2] = 0

    reps = _check_cfg(gpu, cfg, edit=edit, expect_active=True)
    assert all(r.v_checked for r in reps)


@pytest.mark.parametrize("dtype,d,rank", [("bf16", 128, 4), ("f32", 64, 2), ("bf16", 128, 8), ("bf16", 128, 12)])
def test_fast_path_is_close_to_the_svd_on_a_steep_residual_spectrum(gpu, dtype, d, rank):
    """App. H quotes a relative error near 1e-4 for three steps: that needs a gap behind the k-th singular value of R.
    Values = `rank` strong directions + weak noise give one; the device's fast path then matches the oracle's fast path to
    the usual tolerance, both report the same small distance from the SVD route, and the plain call (the SVD route on
    the device) lands that close to it too."""
    cfg = si.RelayConfig("steep", 31, 1, 4, 2, d, 1500, 8, 24, rank, dtype, "structured")

    def edit(K, V, Q):
        r = np.random.default_rng(5)
        L, H, N, _ = V.shape
        dirs = np.linalg.qr(r.standard_normal((d, rank)))[0].T * np.linspace(6.0, 4.0, rank)[:, None]
        X = r.standard_normal((L, H, N, rank)) @ dirs + 0.05 * r.standard_normal((L, H, N, d))
        for h in range(H):
            # the retained rows (decided by K and Q alone) carry only the noise, so the strong directions stay in R
            keep = O.compress_head(K[0, h], V[0, h], Q[0, h * cfg.group:(h + 1) * cfg.group], cfg.budget, 0, dtype).idx
            X[0, h, keep] = 0.05 * r.standard_normal((keep.size, d))
        V[...] = O.round_to_io(X, dtype)

    var = O.Variant(subspace_iters=3)
    reps = _check_cfg(gpu, cfg, edit=edit, variant=var, expect_active=True)
    assert all(r.v_checked for r in reps)
    K, V, Q = si.make_cache(cfg, 0, threads=8)
    edit(K, V, Q)
    fast = gpu.run_fused(cfg, K, V, Q, budgets=si.budgets(cfg, 0), rank=rank, variant=_gpu_variant(var))
    plain = gpu.run_fused(cfg, K, V, Q, budgets=si.budgets(cfg, 0), rank=rank)
    fe = fast["diag"]["fast_err"]
    assert np.all((fe >= 0) & (fe < 5e-3)), fe
    assert np.all(plain["diag"]["fast_err"] == -1.0)
    for h in range(cfg.n_kv_heads):
        a, b = fast["delta"][0, h].astype(np.float64), plain["delta"][0, h].astype(np.float64)
        assert abs(np.linalg.norm(a - b) / np.linalg.norm(b) - fe[0, h]) < 1e-3


@pytest.mark.parametrize("support,k_want", [(43, 3), (41, 1), (40, 0)])
def test_fast_path_drops_dependent_rows_when_the_residual_rank_is_smaller(gpu, support, k_want):
    """The iteration starts from min(pca_rank, d - r, |P_del|) rows; a residual of lower rank leaves fewer independent ones."""
    cfg = si.RelayConfig("fast-rank", 22, 1, 4, 2, 128, 900, 8, 40, 8, "bf16", "structured")

    def edit(K, V, Q):
        V[..., support:] = 0

    reps = _check_cfg(gpu, cfg, edit=edit, variant=O.Variant(subspace_iters=3))
    assert all(r.v_checked and not r.ambiguous for r in reps)
    assert all(r.skipped == (1 if k_want == 0 else 0) for r in reps)


def test_fast_path_argument_errors(gpu):
    cfg = si.shrink(si.CONFIGS["1s"], n_layers=1)
    K, V, Q = si.make_cache(cfg, 0, threads=8)
    from paper_2604_13349_amd import binding as B
    for bad, rank in ((B.make_variant(subspace_iters=-1), 2), (B.make_variant(subspace_iters=65), 2),
                      (B.make_variant(subspace_iters=3), 17), (B.make_variant(subspace_iters=3, subspace="all"), 2)):
        with pytest.raises(B.ObfError):
            gpu.run_fused(cfg, K, V, Q, budget=cfg.budget, rank=rank, variant=bad)
    # the aggregate of the deleted rows has no subspace: the field is ignored there
    gpu.run_fused(cfg, K, V, Q, budget=cfg.budget, rank=2, variant=B.make_variant(subspace_iters=3, naive_aggregation=True))


# --------------------------------------------------------------------------- cache-merging comparison system (App. E)
COS_TIE = 2e-5       # a route may differ from the oracle's only where the oracle's two best cosines are this close


def _check_merge(gpu, cfg, seed, budgets):
    import torch
    from paper_2604_13349_amd import binding as Bd
    K, V, Q = si.make_cache(cfg, seed, threads=8)
    bud = np.asarray(budgets, dtype=np.int32).reshape(cfg.n_layers, cfg.n_kv_heads)
    o = Bd.compress_relay_merge(gpu.to_dev(K, cfg.dtype), gpu.to_dev(V, cfg.dtype), gpu.to_dev(Q, cfg.dtype),
                                budgets=bud.reshape(-1), want_scores=True, want_route=True)
    torch.cuda.synchronize()
    idx, nk, route = o["idx"].cpu().numpy(), o["n_keep"].cpu().numpy(), o["route"].cpu().numpy()
    Ko, Vo = gpu.to_host(o["K_out"], cfg.dtype), gpu.to_host(o["V_out"], cfg.dtype)
    N = cfg.n_tokens
    checked_slots = moved = deleted = 0
    for l in range(cfg.n_layers):
        for h in range(cfg.n_kv_heads):
            B = int(min(bud[l, h], N))
            ref = O.merge_head(K[l, h], V[l, h], Q[l, h * cfg.group:(h + 1) * cfg.group], B, cfg.dtype)
            tag = f"merge {cfg.name}[{l},{h}]"
            assert nk[l, h] == B and np.all(idx[l, h, B:] == -1)
            assert np.array_equal(Ko[l, h, :B], K[l, h][idx[l, h, :B]]), f"{tag}: keys must stay bit copies"
            assert not Vo[l, h, B:].any()
            if not np.array_equal(idx[l, h, :B], ref.idx):
                only_g = set(idx[l, h, :B].tolist()) - set(ref.idx.tolist())
                only_r = set(ref.idx.tolist()) - set(idx[l, h, :B].tolist())
                for a, b in zip(sorted(only_g, key=lambda j: -ref.A[j]), sorted(only_r, key=lambda j: -ref.A[j])):
                    assert abs(ref.A[a] - ref.A[b]) < parity.SWAP_REL * max(ref.A[a], ref.A[b]), f"{tag}: index sets differ"
                continue                                     # a tolerated swap at the threshold: routes are not comparable
            g = route[l, h]
            assert np.array_equal(g < 0, ref.route < 0), f"{tag}: retained tokens must carry no route"
            diff = np.nonzero(g != ref.route)[0]
            assert np.all(ref.cos_gap[diff] < COS_TIE), f"{tag}: {len(diff)} routes differ beyond the cosine tie allowance"
            deleted += int((ref.route >= 0).sum()); moved += len(diff)
            tainted = set(g[diff].tolist()) | set(ref.route[diff].tolist())
            touched = set(ref.route[ref.route >= 0].tolist())
            got = O.decode(Vo[l, h, :B], cfg.dtype)
            for s in range(B):
                if s in tainted:
                    continue
                if s not in touched:
                    assert np.array_equal(Vo[l, h, s], V[l, h][ref.idx[s]]), f"{tag}: slot {s} received nothing and must stay a bit copy"
                    continue
                want = ref.V_star[s]
                mag = np.maximum(np.abs(want), np.abs(got[s]))
                if cfg.dtype == "bf16":
                    half_ulp = np.where(mag > 0, 2.0 ** (np.floor(np.log2(np.maximum(mag, 1e-300))) - 8.0), 0.0)
                    bound = half_ulp * (1 + 1e-6) + 1e-5 * np.abs(want).max()
                else:
                    bound = 1e-5 * np.maximum(np.abs(want), np.abs(want).max() * 1e-2)
                assert np.all(np.abs(got[s] - want) <= bound), f"{tag}: slot {s} off by {np.abs(got[s] - want).max():.3e}"
                checked_slots += 1
    print(f"[merge {cfg.name}] slots value-checked {checked_slots}; routes differing inside the cosine tie allowance {moved} of {deleted}")
    assert moved <= max(2, deleted // 200)
    return checked_slots


def test_cache_merging_matrix_core_route(gpu):
    cfg = si.shrink(si.CONFIGS["2"], n_layers=1, n_kv_heads=4, name="merge-2")
    assert _check_merge(gpu, cfg, 1, [205, 205, 64, 700]) > 500


def test_cache_merging_fp32_and_head_dim_64(gpu):
    assert _check_merge(gpu, si.CONFIGS["1"], 0, [64, 100]) > 100
    cfg = si.RelayConfig("merge-ragged", 23, 1, 4, 3, 64, 1000, 8, 0, 0, "bf16", "structured", outlier_frac=0.01)
    assert _check_merge(gpu, cfg, 2, [40, 0, 1000, 333]) > 250


def test_cache_merging_ragged_token_count_on_the_matrix_cores(gpu):
    cfg = si.RelayConfig("merge-tail", 24, 1, 3, 2, 128, 4099, 16, 0, 0, "bf16", "structured", outlier_frac=0.01)
    assert _check_merge(gpu, cfg, 3, [130, 1, 615]) > 600


# --------------------------------------------------------------------------- batch of right-padded samples (App. A.7)
# --------------------------------------------------------------------------- the Per-token alternative (App. D; a stated reading)
PER_TOKEN = {
    "plain": O.Variant(per_token=True),
    "no_scaling": O.Variant(per_token=True, no_scaling=True),
    "fast_path_3": O.Variant(per_token=True, subspace_iters=3),
    "no_projection": O.Variant(per_token=True, no_projection=True),
}


@pytest.mark.parametrize("name,cfgname", [("plain", "paper"), ("no_scaling", "paper"), ("fast_path_3", "paper"),
                                          ("no_projection", "paper"), ("plain", "1s"), ("plain", "2s")])
def test_per_token_alternative(gpu, name, cfgname):
    """One direction per retained slot (the reading stated at the oracle's per_token_offsets): the fused variant call against
    the oracle, slot by slot.  The routing is the cache-merging one; a route may differ from the oracle's only where the
    oracle's two best cosines agree to COS_TIE, and the slots such a token touches are left out of the value check."""
    import torch
    from paper_2604_13349_amd import binding as Bd
    var = PER_TOKEN[name]
    cfg = si.shrink(si.CONFIGS[cfgname], n_layers=1)
    K, V, Q = si.make_cache(cfg, 3, threads=8)
    out = gpu.run_fused(cfg, K, V, Q, budget=cfg.budget, variant=_gpu_variant(var))
    mo = Bd.compress_relay_merge(gpu.to_dev(K, cfg.dtype), gpu.to_dev(V, cfg.dtype), gpu.to_dev(Q, cfg.dtype),
                                 budget=cfg.budget, want_route=True)
    torch.cuda.synchronize()
    route = mo["route"].cpu().numpy()
    checked = untouched = 0
    for h in range(cfg.n_kv_heads):
        tag = f"per-token {cfgname}/{name}[{h}]"
        Qh = Q[0, h * cfg.group:(h + 1) * cfg.group]
        ref = O.compress_head(K[0, h], V[0, h], Qh, cfg.budget, cfg.rank, cfg.dtype, var)
        mref = O.merge_head(K[0, h], V[0, h], Qh, cfg.budget, cfg.dtype)
        B = ref.idx.size
        if not np.array_equal(out["idx"][0, h][:B], ref.idx):
            continue                                         # a tolerated swap at the threshold (checked elsewhere)
        assert np.array_equal(out["K_out"][0, h][:B], K[0, h][ref.idx])
        dg = ref.diag
        assert int(out["diag"][0, h]["skipped"]) == dg.skipped == 0 and int(out["diag"][0, h]["k_used"]) == dg.k_used
        # delta_out is the slots' mean, i.e. Eq. 6's vector
        g = parity.gap_factor(dg)
        dn = np.linalg.norm(dg.delta)
        assert np.linalg.norm(out["delta"][0, h].astype(np.float64) - dg.delta) <= 2e-3 * g * dn, f"{tag}: delta"
        diff = np.nonzero(route[0, h] != mref.route)[0]
        assert np.all(mref.cos_gap[diff] < COS_TIE), f"{tag}: routes differ beyond the cosine tie allowance"
        tainted = set(route[0, h][diff].tolist()) | set(mref.route[diff].tolist())
        touched = set(mref.route[mref.route >= 0].tolist())
        Vk = O.decode(V[0, h][ref.idx], cfg.dtype)
        got = O.decode(out["V_out"][0, h][:B], cfg.dtype)
        for s_ in range(B):
            if s_ in tainted:
                continue
            if s_ not in touched:
                assert np.array_equal(out["V_out"][0, h][s_], V[0, h][ref.idx[s_]]), f"{tag}: slot {s_} must stay a bit copy"
                untouched += 1
                continue
            want = ref.V_star[s_]
            off = np.abs(want - Vk[s_]).max()
            mag = np.maximum(np.abs(want), np.abs(got[s_]))
            half_ulp = np.where(mag > 0, 2.0 ** (np.floor(np.log2(np.maximum(mag, 1e-300))) - 8.0), 0.0) if cfg.dtype == "bf16" else 0.0
            bound = half_ulp * (1 + 1e-6) + 2e-3 * g * off + 1e-6 * np.abs(want).max()
            assert np.all(np.abs(got[s_] - want) <= bound), f"{tag}: slot {s_} off by {np.abs(got[s_] - want).max():.3e} (offset {off:.3e})"
            checked += 1
    print(f"[per-token {cfgname}/{name}] slots value-checked {checked}, untouched bit copies {untouched}")
    assert checked >= 4 * cfg.n_kv_heads


def test_per_token_argument_errors(gpu):
    cfg = si.shrink(si.CONFIGS["1s"], n_layers=1)
    K, V, Q = si.make_cache(cfg, 0, threads=8)
    from paper_2604_13349_amd import binding as B
    for bad, rank in ((B.make_variant(per_token=True, attn_inject=True), 2), (B.make_variant(per_token=True, subspace="all"), 2),
                      (B.make_variant(per_token=True, naive_aggregation=True), 2), (B.make_variant(per_token=True), 17)):
        with pytest.raises(B.ObfError):
            gpu.run_fused(cfg, K, V, Q, budget=cfg.budget, rank=rank, variant=bad)


@pytest.mark.parametrize("sink", [0, 4])
def test_batch_of_right_padded_samples_with_mixed_lengths(gpu, sink):
    """Four samples of different lengths in one right-padded buffer, one budget per sample (below and above head_dim),
    one call: every (sample, layer, head) must equal what the oracle computes for that sample alone."""
    import torch
    from paper_2604_13349_amd import binding as Bd
    lens, buds, stride = [340, 165, 512, 97], [32, 32, 200, 500], 512
    cfg = si.RelayConfig("batch", 61, 2, 2, 2, 128, stride, 8, 0, 2, "bf16", "structured", outlier_frac=0.01)
    Ks, Vs, Qs = [], [], []
    for s in range(len(lens)):
        K, V, Q = si.make_cache(cfg, 100 + s, threads=4)
        K[:, :, lens[s]:] = 0x7FC0                        # padding rows hold NaNs: they must never be read
        V[:, :, lens[s]:] = 0x7FC0
        Ks.append(K); Vs.append(V); Qs.append(Q)
    Kb, Vb, Qb = (np.stack(x) for x in (Ks, Vs, Qs))
    o = Bd.compress_relay_batch(gpu.to_dev(Kb, "bf16"), gpu.to_dev(Vb, "bf16"), gpu.to_dev(Qb, "bf16"), lens, budgets=buds,
                                rank=cfg.rank, sink=sink, want_diag=True)
    torch.cuda.synchronize()
    idx, nk = o["idx"].cpu().numpy(), o["n_keep"].cpu().numpy()
    Ko, Vo = gpu.to_host(o["K_out"], "bf16"), gpu.to_host(o["V_out"], "bf16")
    diag = o["diag"].cpu().numpy().view(Bd.DIAG_DTYPE).reshape(len(lens), cfg.n_layers, cfg.n_kv_heads)
    checked = active = 0
    for s, n in enumerate(lens):
        for l in range(cfg.n_layers):
            for h in range(cfg.n_kv_heads):
                ref = O.compress_head(Kb[s, l, h, :n], Vb[s, l, h, :n], Qb[s, l, h * cfg.group:(h + 1) * cfg.group], buds[s],
                                      cfg.rank, "bf16", O.Variant(), sink)
                rep = parity.check_head(f"batch[{s},{l},{h}]", ref, Kb[s, l, h, :n], Vb[s, l, h, :n], "bf16", buds[s], idx[s, l, h],
                                        nk[s, l, h], Ko[s, l, h], Vo[s, l, h], gpu_diag=diag[s, l, h], sink=sink)
                checked += int(rep.v_checked); active += int(rep.skipped == 0)
    assert checked >= 14 and active >= 6


# --------------------------------------------------------------------------- stacked int8 / int4 relay codes (App. E, a reading)
def test_batch_with_two_samples_in_flight_equals_one_at_a_time(gpu):
    """With room for several workspace slots the samples take turns on the caller's stream and the library's own; the
    outputs are those of the same batch run one sample after the other (one slot), bit for bit, also when the call is
    repeated on the same buffers."""
    import torch
    from paper_2604_13349_amd import binding as Bd
    cfg = si.shrink(si.CONFIGS["paper"], n_layers=2)
    lens = [256, 201, 256, 77, 130]
    stride = 256
    S = len(lens)
    r = np.random.default_rng(11)
    Ks, Vs, Qs = [], [], []
    for s_ in range(S):
        K, V, Q = si.make_cache(cfg, 20 + s_, threads=8)
        Ks.append(K); Vs.append(V); Qs.append(Q)
    Kb, Vb, Qb = (gpu.to_dev(np.stack(x), cfg.dtype) for x in (Ks, Vs, Qs))
    buds = [32, 20, 48, 16, 32]
    two = Bd.compress_relay_batch(Kb, Vb, Qb, lens, budgets=buds, rank=2, want_diag=True)
    one = Bd.compress_relay_batch(Kb, Vb, Qb, lens, budgets=buds, rank=2, want_diag=True, lanes=1)
    pair = Bd.compress_relay_batch(Kb, Vb, Qb, lens, budgets=buds, rank=2, want_diag=True, lanes=2)
    torch.cuda.synchronize()
    keep = {k: two[k].clone() for k in ("K_out", "V_out", "idx", "n_keep", "diag")}
    for k in keep:
        assert torch.equal(two[k], one[k]), k
        assert torch.equal(pair[k], one[k]), f"{k} with a workspace of two slots"
    for _ in range(3):
        Bd.compress_relay_batch(Kb, Vb, Qb, lens, budgets=buds, rank=2, want_diag=True, out=two)
    torch.cuda.synchronize()
    for k in keep:
        assert torch.equal(two[k], keep[k]), f"{k} changed on a repeated call"
    # under stream capture the samples are enqueued one after the other on the capturing stream: same bits on every replay
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        Bd.compress_relay_batch(Kb, Vb, Qb, lens, budgets=buds, rank=2, want_diag=True, out=two)
    torch.cuda.synchronize()
    for rep in range(2):
        for k in keep:
            two[k].zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in keep:
            assert torch.equal(two[k], keep[k]), f"graph replay {rep}: {k} differs from the eager call"


@pytest.mark.parametrize("dtype,d,bits", [("bf16", 128, 8), ("bf16", 128, 4), ("f32", 64, 8), ("bf16", 64, 4)])
def test_relay_row_codes_are_bit_exact(gpu, dtype, d, bits):
    import torch
    from paper_2604_13349_amd import binding as Bd
    r = np.random.default_rng(70 + bits + d)
    X = (r.standard_normal((1500, d)) * np.exp(r.standard_normal((1500, 1)))).astype(np.float32)
    X[7] = 0.0; X[8] = 2.5; X[9, 1:] = X[9, 0]                  # all-zero, constant and almost constant rows
    X_io = O.round_to_io(X, dtype)
    q_ref, s_ref, z_ref = O.quantize_rows(X_io, dtype, bits)
    Xd = gpu.to_dev(X_io, dtype)
    codes, scale, zero = Bd.quantize_rows(Xd, bits)
    back = Bd.dequantize_rows(codes, scale, zero, d, Xd.dtype, bits)
    torch.cuda.synchronize()
    assert np.array_equal(scale.cpu().numpy().view(np.uint16), s_ref.view(np.uint16))
    assert np.array_equal(zero.cpu().numpy().view(np.uint16), z_ref.view(np.uint16))
    got = codes.cpu().numpy()
    want = q_ref if bits == 8 else (q_ref[:, 0::2] | (q_ref[:, 1::2] << 4)).astype(np.uint8)
    assert np.array_equal(got, want), f"{int((got != want).sum())} codes differ"
    ref_back = O.round_to_io(O.dequantize_rows(q_ref, s_ref, z_ref), dtype)
    assert np.array_equal(gpu.to_host(back, dtype), ref_back)
