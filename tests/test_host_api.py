"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the header
declares, sizes its workspace, and rejects bad arguments before anything is enqueued."""
import ctypes as C
import os
import re

import pytest

from paper_2604_13349_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.lib_path()):
        from paper_2604_13349_amd import build
        build.build(verbose=False)
    return B.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "obf_relay.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(obf_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"obf_score", "obf_select_topk", "obf_refine_boundary", "obf_gather", "obf_backfill",
            "obf_compress_relay", "obf_workspace_bytes", "obf_last_error"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in obf_relay.h but not exported"


def test_version_and_stage_names(lib):
    assert b"gfx950" in lib.obf_version()
    stages = B.profile_stages()
    assert stages[0] == "score_stats" and "gather" in stages and len(stages) == lib.obf_profile_stage_count()


def test_workspace_bytes_and_unsupported_shapes(lib):
    ok = B.make_shape(36, 8, 4, 128, 8192, 32, "bf16")
    need = B.workspace_bytes(ok, 1229, 8)
    assert need > 0 and need % 256 == 0
    assert B.workspace_bytes(B.make_shape(1, 1, 1, 100, 64, 1, "bf16"), 8, 1) == 0     # head_dim
    assert B.workspace_bytes(B.make_shape(1, 1, 1, 128, 40000, 1, "bf16"), 8, 1) == 0  # too many tokens
    assert B.workspace_bytes(B.make_shape(0, 1, 1, 128, 64, 1, "bf16"), 8, 1) == 0
    assert B.workspace_bytes(ok, -1, 1) == 0 and B.workspace_bytes(ok, 8, -1) == 0


def _status(lib, fn, *args):
    rc = fn(*args)
    return rc, lib.obf_last_error().decode()


def test_argument_errors_are_reported_before_any_device_work(lib):
    sh = B.make_shape(2, 2, 2, 64, 100, 4, "f32")
    fake = C.c_void_p(256 * 7)          # never dereferenced: every call below must fail on the host
    rc, msg = _status(lib, lib.obf_score, C.byref(sh), None, fake, fake, None, fake, 1 << 30, None)
    assert rc == 1 and "K" in msg
    rc, msg = _status(lib, lib.obf_score, C.byref(sh), fake, fake, fake, None, None, 0, None)
    assert rc == 1 and "workspace" in msg
    rc, msg = _status(lib, lib.obf_score, C.byref(sh), fake, fake, fake, None, C.c_void_p(257), 1 << 30, None)
    assert rc == 1 and "aligned" in msg
    rc, msg = _status(lib, lib.obf_score, C.byref(sh), fake, fake, fake, None, fake, 16, None)
    assert rc == 3 and "too small" in msg
    rc, msg = _status(lib, lib.obf_select_topk, C.byref(sh), fake, None, -1, 10, fake, fake, None, 0, None)
    assert rc == 1 and "budget" in msg
    rc, msg = _status(lib, lib.obf_select_topk, C.byref(sh), fake, None, 50, 10, fake, fake, None, 0, None)
    assert rc == 1 and "max_budget" in msg
    budgets = (C.c_int32 * 4)(1, 2, 300, 4)     # 300 > n_tokens clamps to 100 > max_budget 10
    rc, msg = _status(lib, lib.obf_select_topk, C.byref(sh), fake, C.cast(budgets, C.c_void_p), 0, 10, fake, fake, None, 0, None)
    assert rc == 1 and "budgets_host[2]" in msg
    rc, msg = _status(lib, lib.obf_gather, C.byref(sh), None, fake, fake, fake, 10, fake, None, None)
    assert rc == 1 and "K_out" in msg
    rc, msg = _status(lib, lib.obf_backfill, C.byref(sh), fake, fake, fake, fake, 10, -2, fake, None, None, fake, 1 << 30, None)
    assert rc == 1 and "rank" in msg
    bad = B.make_shape(2, 2, 2, 96, 100, 4, "f32")
    rc, msg = _status(lib, lib.obf_compress_relay, C.byref(bad), fake, fake, fake, None, 5, 5, 1, fake, fake, fake, fake,
                      None, None, None, fake, 1 << 30, None)
    assert rc == 2 and "head_dim" in msg
    rc, msg = _status(lib, lib.obf_compress_relay, None, fake, fake, fake, None, 5, 5, 1, fake, fake, fake, fake,
                      None, None, None, fake, 1 << 30, None)
    assert rc == 1 and "shape" in msg
    assert lib.obf_profile_enable(999) == 1


def test_variant_window_and_message_argument_errors(lib):
    sh = B.make_shape(2, 2, 2, 64, 100, 4, "f32")
    fake = C.c_void_p(256 * 7)          # never dereferenced
    tail = (fake, fake, fake, fake, None, None, None, fake, 1 << 30, None)
    for var, word in ((B.make_variant(subspace=5), "subspace"), (B.make_variant(subspace="evr", evr_tau=0.0), "evr_tau"),
                      (B.make_variant(subspace="evr", evr_tau=1.01), "evr_tau")):
        rc, msg = _status(lib, lib.obf_compress_relay_variant, C.byref(sh), fake, fake, fake, None, 5, 5, 1, 0, C.byref(var), *tail)
        assert rc == 1 and word in msg
        rc, msg = _status(lib, lib.obf_backfill_variant, C.byref(sh), fake, fake, fake, fake, 5, 1, C.byref(var), fake, None, None,
                          fake, 1 << 30, None)
        assert rc == 1 and word in msg
    for win, word in ((B._Window(99, 0), "token_stride"), (B._Window(0, 100), "sink"), (B._Window(0, -1), "sink")):
        rc, msg = _status(lib, lib.obf_compress_relay_window, C.byref(sh), C.byref(win), fake, fake, fake, None, 5, 5, 1, 0, None, *tail)
        assert rc == 1 and word in msg
    # a budget is counted in eligible tokens: 97 of them behind a sink of 3, so a budget of 98 keeps 97 > max_budget 96
    rc, msg = _status(lib, lib.obf_compress_relay_window, C.byref(sh), C.byref(B._Window(0, 3)), fake, fake, fake, None, 98, 96, 1, 0,
                      None, *tail)
    assert rc == 1 and "max_budget" in msg
    msg_args = dict(prev=(fake, fake, None, 4, 8), keep=(fake, fake, fake, 8), gen=(fake, fake, 2, 2))

    def append(n_heads=4, d=64, dtype=B.OBF_F32, prev=msg_args["prev"], keep=msg_args["keep"], gen=msg_args["gen"], out=(fake, fake, fake, 32)):
        return _status(lib, lib.obf_append_message, n_heads, d, dtype, *prev, *keep, *gen, *out, None)

    assert append(n_heads=0)[0] == 1
    assert append(d=96)[0] == 2
    assert append(dtype=7)[0] == 1
    rc, msg = append(prev=(fake, fake, None, 9, 8)); assert rc == 1 and "prev_len_all" in msg
    rc, msg = append(prev=(None, fake, None, 4, 8)); assert rc == 1 and "prev" in msg
    rc, msg = append(keep=(None, fake, fake, 8)); assert rc == 1 and "keep" in msg
    rc, msg = append(gen=(fake, fake, 3, 2)); assert rc == 1 and "n_gen" in msg
    rc, msg = append(gen=(None, fake, 2, 2)); assert rc == 1 and "gen" in msg
    rc, msg = append(out=(fake, fake, None, 32)); assert rc == 1 and "msg_len" in msg
    rc, msg = append(out=(fake, fake, fake, 0)); assert rc == 1
    rc, msg = append(keep=(None, None, None, 0), out=(fake, fake, fake, 5)); assert rc == 1 and "msg_stride" in msg


def test_binding_raises_without_library(monkeypatch, tmp_path):
    monkeypatch.setenv("OBF_RELAY_LIB", str(tmp_path / "missing.so"))
    monkeypatch.setattr(B, "_lib", None)
    with pytest.raises(ImportError):
        B.load_library()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_static_scratch_entry_point_refuses_oversized_shapes_on_the_host(lib):
    """obf_compress_relay_static: a shape whose workspace exceeds the built-in array is refused before any device call."""
    assert lib.obf_static_scratch_bytes() >= 32 << 20
    sh = B.make_shape(36, 8, 4, 128, 8192, 32, "bf16")
    assert B.workspace_bytes(sh, 1229, 8) > lib.obf_static_scratch_bytes()
    fake = C.c_void_p(256 * 7)
    rc = lib.obf_compress_relay_static(C.byref(sh), fake, fake, fake, None, 1229, 1229, 8, fake, fake, fake, fake, None)
    assert rc == 2 and "scratch" in lib.obf_last_error().decode()
    bad = B.make_shape(1, 1, 1, 100, 64, 1, "bf16")
    assert lib.obf_compress_relay_static(C.byref(bad), fake, fake, fake, None, 8, 8, 1, fake, fake, fake, fake, None) == 2


def test_batch_entry_point_checks_every_sample_on_the_host(lib):
    sh = B.make_shape(2, 2, 2, 128, 1, 8, "bf16")
    fake = C.c_void_p(256 * 9)
    lens = (C.c_int32 * 3)(100, 0, 50)
    call = lambda lens_, stride, sink, buds, budget, maxb, ws_bytes: lib.obf_compress_relay_batch(
        C.byref(sh), 3, lens_, stride, sink, fake, fake, fake, buds, budget, maxb, 2, fake, fake, fake, fake, None, fake, ws_bytes, None)
    assert call(lens, 128, 0, None, 16, 16, 1 << 30) == 1 and "n_tokens_host[1]" in lib.obf_last_error().decode()
    lens = (C.c_int32 * 3)(100, 200, 50)
    assert call(lens, 128, 0, None, 16, 16, 1 << 30) == 1                       # 200 tokens in a stride of 128
    lens = (C.c_int32 * 3)(100, 128, 50)
    assert call(lens, 128, 50, None, 16, 16, 1 << 30) == 1 and "eligible" in lib.obf_last_error().decode()
    buds = (C.c_int32 * 3)(16, 40, 16)
    assert call(lens, 128, 0, buds, 0, 16, 1 << 30) == 1 and "sample 1" in lib.obf_last_error().decode()
    need = lib.obf_workspace_bytes_batch(C.byref(sh), 3, 128, 40, 2)
    one = lib.obf_workspace_bytes_batch(C.byref(sh), 1, 128, 40, 2)
    assert one > 0 and one % 256 == 0 and need == 3 * one                       # a slot per sample in flight, three at most
    assert lib.obf_workspace_bytes_batch(C.byref(sh), 2, 128, 40, 2) == 2 * one
    assert lib.obf_workspace_bytes_batch(C.byref(sh), 9, 128, 40, 2) == 3 * one
    assert call(lens, 128, 0, buds, 0, 40, one // 2) == 3                       # OBF_ERR_WORKSPACE_TOO_SMALL
    assert lib.obf_workspace_bytes_batch(C.byref(sh), 3, 40000, 40, 2) == 0
