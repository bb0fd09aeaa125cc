#!/usr/bin/env python3
"""Benchmark of the fused relay compression (score -> TopK_B -> refine -> gather -> OBF) on one MI355X.

A step is one obf_compress_relay call over a whole synthetic cache that is already resident in
HBM.  Prints ONE JSON line: head-tokens/s, the HBM roofline of the dominant kernel (timed with
HIP events inside the library, on the launch stream), and the CPU oracle timed on a bounded
sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
METRIC = "compressed KV-head-tokens/s + achieved HBM GB/s, Qwen3-8B-shape 8K cache"


def stage_bytes(stage: str, cfg, budgets, active_heads: int) -> float:
    """Algorithmic HBM bytes one launch of a stage must move (inputs read once, outputs written once)."""
    es = 2 if cfg.dtype == "bf16" else 4
    heads, N, d, R = cfg.n_heads, cfg.n_tokens, cfg.head_dim, cfg.rows
    kept = float(sum(min(int(b), N) for b in budgets.reshape(-1)))
    k_bytes = heads * N * d * es
    q_bytes = heads * R * d * es
    if stage == "score_stats":
        return k_bytes + q_bytes
    if stage == "score_mass":
        return k_bytes + q_bytes + heads * N * 4
    if stage == "score_fused":
        return k_bytes + q_bytes + heads * N * 4
    if stage == "gather":
        return 4 * kept * d * es
    if stage == "del_stats":
        return active_heads * N * d * es
    if stage in ("keep_basis", "keep_cert"):
        return kept * d * es + heads * N * 4
    if stage == "select":
        return heads * N * 4 + kept * 4
    return 0.0


def path_bytes(cfg, budgets, active_heads: int) -> float:
    """Algorithmic bytes of the whole path: K and Q once, kept rows read and written, V only where OBF is active."""
    es = 2 if cfg.dtype == "bf16" else 4
    heads, N, d, R = cfg.n_heads, cfg.n_tokens, cfg.head_dim, cfg.rows
    kept = float(sum(min(int(b), N) for b in budgets.reshape(-1)))
    return heads * N * d * es + heads * R * d * es + 4 * kept * d * es + active_heads * N * d * es


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="3", help="config name from synth_inputs.CONFIGS (default: config 3)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU time budget of the oracle baseline (0: skip)")
    ap.add_argument("--layers", type=int, default=0, help="use only the first LAYERS layers (0: all)")
    ap.add_argument("--selector", choices=["head", "layer"], default="head",
                    help="granularity of the retention rule: per KV head (the headline path) or one index set per layer")
    ap.add_argument("--copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB before the timed region (a kernel of known "
                         "traffic that calibrates the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    ap.add_argument("--variant", default="none",
                    choices=["none", "no_projection", "max_p", "no_scaling", "naive", "attn_inject", "evr"],
                    help="ablation variant of App. D (not the headline path)")
    ap.add_argument("--sink", type=int, default=-1,
                    help="protect the first SINK tokens as the shared attention sink (the window entry point; -1: plain call)")
    ap.add_argument("--no-full-path", dest="full_path", action="store_false",
                    help="skip the extra timings of the full back-fill path (shadow config and paper shape) after the headline")
    ap.add_argument("--message", type=int, default=0,
                    help="also build the outgoing message [sink; retained rows; MESSAGE reasoning rows] in every step")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import synth_inputs as si
    from paper_2604_13349_amd import binding as B

    B.load_library()                      # fails loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    cfg = si.CONFIGS[args.workload]
    if args.layers:
        cfg = si.shrink(cfg, n_layers=args.layers, name=cfg.name)
    threads = min(16, os.cpu_count() or 1)
    t0 = time.time()
    calls = []
    for a in range(cfg.agents):           # config 5: sequential, independent agent hand-offs
        K, V, Q = si.make_cache(cfg, args.seed + a, threads=threads)
        bud = si.budgets(cfg, args.seed + a)
        def dev(x):
            if cfg.dtype == "bf16":
                return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
            return torch.from_numpy(x).cuda()
        calls.append({"K": dev(K), "V": dev(V), "Q": dev(Q), "bud": bud, "host": (K, V, Q) if a == 0 else None})
        if a > 0:
            del K, V, Q
    gen_s = time.time() - t0
    uniform = cfg.budget_range is None and cfg.budget_int_range is None
    layerwise = args.selector == "layer"
    if layerwise and not uniform:
        for c in calls:                   # one budget per layer: the first head's draw
            c["bud"] = c["bud"].reshape(cfg.n_layers, cfg.n_kv_heads)[:, :1].copy()
    max_budget = int(max(int(min(c["bud"].max(), cfg.n_tokens)) for c in calls))
    outs = [None] * len(calls)
    vflags = {"none": {}, "no_projection": {"no_projection": True}, "max_p": {"subspace": "all"}, "no_scaling": {"no_scaling": True},
              "naive": {"naive_aggregation": True}, "attn_inject": {"attn_inject": True}, "evr": {"subspace": "evr", "evr_tau": 0.35}}
    variant = B.make_variant(**vflags[args.variant]) if args.variant != "none" else None
    sink = args.sink if args.sink >= 0 else None
    if sink is not None:
        max_budget = min(max_budget, cfg.n_tokens - sink)
    gen_rows = None
    if args.message > 0:                  # stand-in for the reasoning states G of Sec. 3.3 (bit copies: values do not matter)
        gen_rows = [torch.zeros((cfg.n_layers, cfg.n_kv_heads, args.message, cfg.head_dim), dtype=calls[0]["K"].dtype,
                                device="cuda") for _ in range(2)]
    msg_ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]

    def step():
        for i, c in enumerate(calls):
            kw = dict(rank=cfg.rank, max_budget=max_budget, out=outs[i], ws=(outs[i] or {}).get("ws"),
                      want_diag=want_diag, layerwise=layerwise, variant=variant, sink=sink)
            if uniform:
                outs[i] = B.compress_relay(c["K"], c["V"], c["Q"], budget=int(c["bud"].flat[0]), **kw)
            else:
                outs[i] = B.compress_relay(c["K"], c["V"], c["Q"], budgets=c["bud"].reshape(-1), **kw)
            if gen_rows is not None:
                msg_ev[0].record()
                outs[i]["msg"] = B.append_message(c["K"], c["V"], None, outs[i]["K_out"], outs[i]["V_out"],
                                                  outs[i]["n_keep"].reshape(-1), gen_rows[0], gen_rows[1],
                                                  (sink or 0) + max_budget + args.message, prev_len_all=sink or 0)
                msg_ev[1].record()

    if args.copy_mib > 0:
        src = torch.empty(args.copy_mib << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                    # reads and writes copy_mib MiB once each
        torch.cuda.synchronize()
        del src, dst
    stages = B.profile_stages()

    def measure(step_fn, steps, warmup):
        """Warm-up, one step per stage with that stage's timing on (HIP events inside the library, on the launch stream), then `steps` timed
        steps: one wall-clock interval around all of them (the headline) and one HIP-event pair per step (the spread)."""
        for _ in range(max(1, warmup)):
            step_fn()
        torch.cuda.synchronize()
        stage_ms = {}
        for sid, name in enumerate(stages):
            B.profile_enable(sid)
            step_fn()
            ms, n = B.profile_read()
            stage_ms[name] = ms
        B.profile_enable(-1)
        dominant = max(stage_ms, key=stage_ms.get)
        B.profile_enable(stages.index(dominant))
        B.profile_read()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for e0, e1 in evs:
            e0.record()
            step_fn()
            e1.record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        dom_ms, dom_n = B.profile_read()
        B.profile_enable(-1)
        per = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
        return {"elapsed": t1 - t0, "stage_ms": stage_ms, "dominant": dominant, "dom_ms": dom_ms, "dom_n": dom_n,
                "step_ms": {"median": round(per[len(per) // 2], 4), "min": round(per[0], 4), "max": round(per[-1], 4)}}

    # one untimed step with the per-head diagnostics (how many heads ran the back-fill); the timed steps leave them
    # out, as a caller on the hot path would (they cost a pass over every head's scores)
    want_diag = True
    step()
    torch.cuda.synchronize()
    diag = B.diag_to_numpy(outs[0]["diag"])
    active_heads = int((diag["skipped"] == 0).sum())
    outs = [None] * len(calls)
    want_diag = False
    r = measure(step, args.steps, args.warmup)
    stage_ms, dominant, dom_ms, dom_n, elapsed = r["stage_ms"], r["dominant"], r["dom_ms"], r["dom_n"], r["elapsed"]
    ms_per_step = 1e3 * elapsed / args.steps
    head_tokens = cfg.n_heads * cfg.n_tokens * len(calls)
    value = head_tokens / (elapsed / args.steps)

    def roofline_of(r, cfg_, buds, active, steps, tname):
        """The dominant kernel against the HBM roofline (its algorithmic bytes over its own average launch time) and, as a
        separate object, the whole path (all algorithmic bytes of a step over the step time)."""
        lps = max(1, r["dom_n"] // max(1, steps))
        avg_ms = r["dom_ms"] / max(1, r["dom_n"])
        kbytes = sum(stage_bytes(r["dominant"], cfg_, b, active) for b in buds) / lps
        ach = kbytes / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else 0.0
        pb = sum(path_bytes(cfg_, b, active) for b in buds)
        step_s = r["elapsed"] / steps
        traffic = None
        tfile = os.path.join(ROOT, "profiles", f"traffic_config{tname}.json")
        if os.path.exists(tfile):
            with open(tfile) as f:
                traffic = json.load(f).get(r["dominant"])
        roof = {"bound": "hbm", "scope": "dominant kernel only (the whole path is the 'path' object)", "kernel": r["dominant"],
                "achieved": round(ach, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                "traffic": traffic, "kernel_ms": round(avg_ms, 4), "kernel_bytes": kbytes,
                "stage_ms": {k: round(v, 4) for k, v in r["stage_ms"].items()}}
        if r["dominant"] in ("keep_basis", "finalize", "select", "keep_cert"):
            roof["note"] = ("a per-head sequential factorisation / bisection: bound by the latency of its dependent steps, "
                            "the HBM fraction only says how far from streaming it is")
        path = {"bytes": pb, "GBps": round(pb / step_s / 1e9, 2), "frac": round(pb / step_s / 1e9 / HBM_PEAK_GBS, 4),
                "target_frac": 0.60, "unit": "GB/s of algorithmic bytes (K, Q once; retained rows read and written; V where the back-fill is active)"}
        return roof, path

    roofline, path = roofline_of(r, cfg, [c["bud"] for c in calls], active_heads, args.steps, cfg.name)
    # kept for readers of earlier lines
    roofline["path_bytes"], roofline["path_GBps"], roofline["path_frac"] = path["bytes"], path["GBps"], path["frac"]

    # The full Orthogonal BackFill path (budget below head_dim, every head injects), measured in the same run: the
    # same resident cache with budget 96 (shadow of this config) and the paper's own shape (N = 256, budget 32, rank 2).
    full_path = []
    plain = variant is None and sink is None and not layerwise and gen_rows is None and cfg.agents == 1
    if args.full_path and plain and cfg.name in ("3", "2", "4"):
        shadows = [(si.CONFIGS[cfg.name + "s"], calls[0])]
        pc = si.CONFIGS["paper"]
        if args.layers:
            pc = si.shrink(pc, n_layers=args.layers, name=pc.name)
        Kp, Vp, Qp = si.make_cache(pc, args.seed, threads=threads)
        shadows.append((pc, {"K": dev(Kp), "V": dev(Vp), "Q": dev(Qp), "bud": si.budgets(pc, args.seed), "host": (Kp, Vp, Qp)}))
        for scfg, c in shadows:
            if args.layers and scfg.name != "paper":
                scfg = si.shrink(scfg, n_layers=args.layers, name=scfg.name)
            sb = si.budgets(scfg, args.seed)
            holder = {"o": None}

            def sstep(c=c, scfg=scfg, sb=sb, holder=holder, wd=False):
                holder["o"] = B.compress_relay(c["K"], c["V"], c["Q"], budget=int(sb.flat[0]), rank=scfg.rank,
                                               max_budget=int(sb.max()), out=holder["o"], ws=(holder["o"] or {}).get("ws"),
                                               want_diag=wd)
            sstep(wd=True)
            torch.cuda.synchronize()
            act = int((B.diag_to_numpy(holder["o"]["diag"])["skipped"] == 0).sum())
            holder["o"] = None
            rr = measure(sstep, args.steps, args.warmup)
            roof_s, path_s = roofline_of(rr, scfg, [sb], act, args.steps, scfg.name)
            full_path.append({"workload": f"config {scfg.name}: {scfg.n_layers} layers x {scfg.n_kv_heads} KV heads, N={scfg.n_tokens}, "
                                          f"budget {int(sb.flat[0])}, rank {scfg.rank}", "active_obf_heads": act,
                              "ms_per_step": round(1e3 * rr["elapsed"] / args.steps, 4), "step_ms": rr["step_ms"],
                              "value": round(scfg.n_heads * scfg.n_tokens / (rr["elapsed"] / args.steps), 1), "unit": "head-tokens/s",
                              "path": path_s, "roofline": roof_s})
            c["shadow"] = (scfg, sb, holder["o"])
        # a batch of paper-shape samples through the batch entry point (three samples in flight on streams of the library)
        nb = 12
        if not args.layers:
            trip = [si.make_cache(pc, args.seed + 100 + j, threads=threads) for j in range(nb)]
            Kb, Vb, Qb = (dev(np.stack([t[j] for t in trip])) for j in range(3))
            del trip
            pb_ = int(si.budgets(pc, args.seed).flat[0])
            bo = {"o": None}

            def bstep():
                bo["o"] = B.compress_relay_batch(Kb, Vb, Qb, [pc.n_tokens] * nb, budget=pb_, rank=pc.rank, out=bo["o"])
            for _ in range(max(1, args.warmup)):
                bstep()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                bstep()
            torch.cuda.synchronize()
            bt = (time.perf_counter() - t0) / args.steps
            full_path.append({"workload": f"batch of {nb} samples of config {pc.name} (N={pc.n_tokens}, budget {pb_}, rank {pc.rank}) in one "
                                          "call of the batch entry point", "ms_per_step": round(1e3 * bt, 4),
                              "ms_per_sample": round(1e3 * bt / nb, 4),
                              "value": round(nb * pc.n_heads * pc.n_tokens / bt, 1), "unit": "head-tokens/s"})
            del Kb, Vb, Qb

    extra = {}
    if gen_rows is not None:
        row = cfg.head_dim * (2 if cfg.dtype == "bf16" else 4)
        nk = int(outs[0]["n_keep"].sum().item())
        copied = cfg.n_heads * ((sink or 0) + args.message) + nk                          # rows that carry data, per K or V
        written = cfg.n_heads * ((sink or 0) + max_budget + args.message)                 # all rows of the message buffers
        ms = msg_ev[0].elapsed_time(msg_ev[1])
        extra["message"] = {"ms": round(ms, 4), "read_bytes": 2 * row * copied, "written_bytes": 2 * row * written,
                            "GBps": round(2 * row * (copied + written) / (ms * 1e-3) / 1e9, 1)}
    ovar, osink = None, (sink or 0)
    cpu = None
    if args.cpu_seconds > 0 and layerwise:
        from oracle import obf_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = 1
        Kh, Vh, Qh = calls[0]["host"]
        bud = calls[0]["bud"].reshape(cfg.n_layers, -1)
        idx_host = outs[0]["idx"].cpu().numpy()
        done, mismatched, tc0 = 0, 0, time.perf_counter()
        for l in range(cfg.n_layers):
            ovar = O.Variant(**{{"naive_aggregation": "naive"}.get(k, k): v for k, v in vflags[args.variant].items()})
            ref_idx, _ = O.compress_layer(Kh[l], Vh[l], Qh[l], int(bud[l, 0]), cfg.rank, cfg.group, cfg.dtype, ovar, osink)
            done += 1
            mismatched += int(not np.array_equal(idx_host[l, 0, :len(ref_idx)], ref_idx))
            if time.perf_counter() - tc0 >= args.cpu_seconds:
                break
        tc = time.perf_counter() - tc0
        cpu = {"value": round(done * cfg.n_kv_heads * cfg.n_tokens / tc, 1), "unit": "head-tokens/s", "cores": int(cores),
               "kind": "oracle", "sample": f"first {done} of {cfg.n_layers} layers of call 0, {tc:.1f} s, fp64 numpy with exact SVD",
               "layers_index_mismatch": mismatched}
    elif args.cpu_seconds > 0:
        from oracle import obf_oracle as O
        from oracle import gram_baseline as G
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = 1

        def cpu_leg(kind, cfg_, host, bud_, idx_dev, seconds):
            """The oracle (kind "oracle": float64, exact SVD) or the single-precision Gram route of App. H (kind "gram32")
            on the first heads of a cache until `seconds` of CPU time are spent; also counts index sets that differ from
            the GPU's."""
            Kh, Vh, Qh = host
            idx_host = idx_dev.cpu().numpy()
            done, mismatched, tc0 = 0, 0, time.perf_counter()
            for l in range(cfg_.n_layers):
                for h in range(cfg_.n_kv_heads):
                    Qg = Qh[l, h * cfg_.group:(h + 1) * cfg_.group]
                    if kind == "oracle":
                        ovar = O.Variant(**{{"naive_aggregation": "naive"}.get(k, k): v for k, v in vflags[args.variant].items()})
                        ridx = O.compress_head(Kh[l, h], Vh[l, h], Qg, int(bud_[l, h]), cfg_.rank, cfg_.dtype, ovar, osink).idx
                    else:
                        ridx = G.compress_head_gram32(Kh[l, h], Vh[l, h], Qg, int(bud_[l, h]), cfg_.rank, cfg_.dtype)[0]
                    done += 1
                    mismatched += int(not np.array_equal(idx_host[l, h, :len(ridx)], ridx))
                    if time.perf_counter() - tc0 >= seconds:
                        break
                else:
                    continue
                break
            tc = time.perf_counter() - tc0
            what = "fp64 numpy with exact SVD" if kind == "oracle" else "fp32 numpy, QR + Gram/eigh route of App. H"
            return {"value": round(done * cfg_.n_tokens / tc, 1), "unit": "head-tokens/s", "cores": int(cores),
                    "host_cpus": os.cpu_count(), "kind": kind,
                    "sample": f"first {done} of {cfg_.n_heads} heads of config {cfg_.name}, {tc:.1f} s, {what}",
                    "heads_index_mismatch": mismatched}

        cpu = cpu_leg("oracle", cfg, calls[0]["host"], calls[0]["bud"], outs[0]["idx"], args.cpu_seconds)
        if full_path and "shadow" in calls[0]:
            # the same two CPU routes on the shadow workload, where the SVD of the residual actually runs
            scfg, sb, so = calls[0]["shadow"]
            extra["cpu_baseline_full_path"] = [cpu_leg("oracle", scfg, calls[0]["host"], sb, so["idx"], args.cpu_seconds / 2),
                                               cpu_leg("gram32", scfg, calls[0]["host"], sb, so["idx"], args.cpu_seconds / 2)]

    line = {
        "metric": METRIC, "value": round(value, 1), "unit": "head-tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"config {cfg.name}: {cfg.n_layers} layers x {cfg.n_kv_heads} KV heads, group {cfg.group}, "
                               f"head_dim {cfg.head_dim}, N={cfg.n_tokens}, window {cfg.window}, rank {cfg.rank}, "
                               f"budget {'per-head' if not uniform else cfg.budget}, {cfg.agents} call(s) per step"
                               + (", layerwise selector" if layerwise else "")
                               + (f", variant {args.variant}" if variant is not None else "")
                               + (f", sink {sink}" if sink is not None else "")
                               + (f", message with {args.message} reasoning rows" if gen_rows is not None else ""),
                   "heads": cfg.n_heads, "active_obf_heads": active_heads, "input_gen_s": round(gen_s, 1)},
        "step_ms": r["step_ms"], "roofline": roofline, "path": path, "full_path": full_path or None, "cpu_baseline": cpu, **extra,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
