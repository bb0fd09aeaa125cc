"""ctypes binding of include/obf_relay.h: same names, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libobf_relay.so"
_lib = None

OBF_F32, OBF_BF16 = 0, 1
_STATUS = {1: "INVALID_ARG", 2: "UNSUPPORTED", 3: "WORKSPACE_TOO_SMALL", 4: "HIP"}

DIAG_DTYPE = np.dtype([("n_keep", "<i4"), ("r_keep", "<i4"), ("k_used", "<i4"), ("skipped", "<i4"),
                       ("a_keep", "<f4"), ("a_del", "<f4"), ("rcr", "<f4"), ("ivn", "<f4"),
                       ("pcr", "<f4"), ("pc", "<f4"), ("revr", "<f4"), ("dr", "<f4"),
                       ("select_flags", "<i4"), ("fast_err", "<f4")])


class ObfError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"obf_relay status {status} ({_STATUS.get(status, '?')}): {msg}")
        self.status = status


class _Shape(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_kv_heads", C.c_int32), ("group", C.c_int32), ("head_dim", C.c_int32),
                ("n_tokens", C.c_int32), ("window", C.c_int32), ("dtype", C.c_int32)]


class _Variant(C.Structure):
    """obf_variant_t."""
    _fields_ = [("no_projection", C.c_int32), ("subspace", C.c_int32), ("evr_tau", C.c_float),
                ("no_scaling", C.c_int32), ("naive_aggregation", C.c_int32), ("attn_inject", C.c_int32),
                ("subspace_iters", C.c_int32), ("per_token", C.c_int32)]


class _Window(C.Structure):
    """obf_window_t."""
    _fields_ = [("token_stride", C.c_int32), ("sink", C.c_int32)]


SUBSPACE = {"rank": 0, "all": 1, "evr": 2}
OBF_SELECT_BAND_OVERFLOW = 1


def make_variant(no_projection=False, subspace="rank", evr_tau=0.35, no_scaling=False, naive_aggregation=False,
                 attn_inject=False, subspace_iters=0, per_token=False) -> _Variant:
    """obf_variant_t from keywords (subspace by its name or its number)."""
    code = SUBSPACE[subspace] if isinstance(subspace, str) else int(subspace)
    return _Variant(int(no_projection), code, float(evr_tau), int(no_scaling), int(naive_aggregation), int(attn_inject),
                    int(subspace_iters), int(per_token))


def lib_path() -> str:
    return os.environ.get("OBF_RELAY_LIB") or os.path.join(_HERE, _LIB_NAME)


def load_library():
    """Loads the built library (torch first, so that both share one HIP runtime)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          f"or `python paper_2604_13349_amd/build.py` (there is no CPU fallback)")
    lib = C.CDLL(path)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    sp = C.POINTER(_Shape)
    lib.obf_workspace_bytes.restype = sz
    lib.obf_workspace_bytes.argtypes = [sp, i32, i32]
    lib.obf_score.restype = C.c_int
    lib.obf_score.argtypes = [sp, vp, vp, vp, vp, vp, sz, vp]
    lib.obf_select_topk.restype = C.c_int
    lib.obf_select_topk.argtypes = [sp, vp, vp, i32, i32, vp, vp, vp, sz, vp]
    lib.obf_refine_boundary.restype = C.c_int
    lib.obf_refine_boundary.argtypes = [sp, vp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
    lib.obf_gather.restype = C.c_int
    lib.obf_gather.argtypes = [sp, vp, vp, vp, vp, i32, vp, vp, vp]
    lib.obf_backfill.restype = C.c_int
    lib.obf_backfill.argtypes = [sp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.obf_compress_relay.restype = C.c_int
    lib.obf_compress_relay.argtypes = [sp, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.obf_compress_relay_layerwise.restype = C.c_int
    lib.obf_compress_relay_layerwise.argtypes = lib.obf_compress_relay.argtypes
    vr = C.POINTER(_Variant)
    lib.obf_backfill_variant.restype = C.c_int
    lib.obf_backfill_variant.argtypes = [sp, vp, vp, vp, vp, i32, i32, vr, vp, vp, vp, vp, sz, vp]
    lib.obf_compress_relay_variant.restype = C.c_int
    lib.obf_compress_relay_variant.argtypes = [sp, vp, vp, vp, vp, i32, i32, i32, i32, vr, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.obf_compress_relay_window.restype = C.c_int
    lib.obf_compress_relay_window.argtypes = [sp, C.POINTER(_Window), vp, vp, vp, vp, i32, i32, i32, i32, vr, vp, vp, vp, vp,
                                              vp, vp, vp, vp, sz, vp]
    lib.obf_workspace_bytes_batch.restype = sz
    lib.obf_workspace_bytes_batch.argtypes = [sp, i32, i32, i32, i32]
    lib.obf_compress_relay_batch.restype = C.c_int
    lib.obf_compress_relay_batch.argtypes = [sp, i32, vp, i32, i32, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.obf_quantize_rows.restype = C.c_int
    lib.obf_quantize_rows.argtypes = [vp, C.c_int64, i32, i32, i32, vp, vp, vp, vp]
    lib.obf_dequantize_rows.restype = C.c_int
    lib.obf_dequantize_rows.argtypes = [vp, vp, vp, C.c_int64, i32, i32, i32, vp, vp]
    lib.obf_cache_merge.restype = C.c_int
    lib.obf_cache_merge.argtypes = [sp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, sz, vp]
    lib.obf_compress_relay_merge.restype = C.c_int
    lib.obf_compress_relay_merge.argtypes = [sp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.obf_static_scratch_bytes.restype = sz
    lib.obf_static_scratch_bytes.argtypes = []
    lib.obf_compress_relay_static.restype = C.c_int
    lib.obf_compress_relay_static.argtypes = [sp, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp]
    lib.obf_append_message.restype = C.c_int
    lib.obf_append_message.argtypes = [i32, i32, i32, vp, vp, vp, i32, i32, vp, vp, vp, i32, vp, vp, i32, i32, vp, vp, vp, i32, vp]
    lib.obf_profile_enable.restype = C.c_int
    lib.obf_profile_enable.argtypes = [i32]
    lib.obf_profile_read.restype = C.c_int
    lib.obf_profile_read.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int32)]
    lib.obf_profile_stage_count.restype = i32
    lib.obf_profile_stage_name.restype = C.c_char_p
    lib.obf_profile_stage_name.argtypes = [i32]
    lib.obf_last_error.restype = C.c_char_p
    lib.obf_version.restype = C.c_char_p
    _lib = lib
    return lib


def _check(status: int):
    if status != 0:
        raise ObfError(status, load_library().obf_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return C.c_void_p(t.data_ptr())


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def shape_of(K: torch.Tensor, Qwin: torch.Tensor) -> _Shape:
    """Shape descriptor from K [L,H,N,d] and Qwin [L,H*group,W,d]."""
    L, H, N, d = K.shape
    Lq, Hq, W, dq = Qwin.shape
    if Lq != L or dq != d or Hq % H != 0:
        raise ValueError("Qwin does not match K")
    if K.dtype == torch.float32:
        dt = OBF_F32
    elif K.dtype == torch.bfloat16:
        dt = OBF_BF16
    else:
        raise ValueError("K must be float32 or bfloat16")
    if Qwin.dtype != K.dtype:
        raise ValueError("Qwin dtype differs from K")
    return _Shape(L, H, Hq // H, d, N, W, dt)


def make_shape(n_layers, n_kv_heads, group, head_dim, n_tokens, window, dtype) -> _Shape:
    """Shape descriptor from plain numbers; dtype is "bf16"/"f32" or a torch dtype."""
    if dtype in ("bf16", torch.bfloat16):
        dt = OBF_BF16
    elif dtype in ("f32", torch.float32):
        dt = OBF_F32
    else:
        raise ValueError("dtype must be bf16 or f32")
    return _Shape(n_layers, n_kv_heads, group, head_dim, n_tokens, window, dt)


def workspace_bytes(shape: _Shape, max_budget: int, rank: int) -> int:
    return int(load_library().obf_workspace_bytes(C.byref(shape), max_budget, rank))


def _ws(shape: _Shape, max_budget: int, rank: int, ws: Optional[torch.Tensor], device) -> torch.Tensor:
    need = workspace_bytes(shape, max_budget, rank)
    if need == 0:
        raise ObfError(2, "unsupported shape")
    if ws is None:
        ws = torch.empty(need, dtype=torch.uint8, device=device)
    return ws


def _budgets_arg(budgets: Optional[Sequence[int]]):
    if budgets is None:
        return None, None
    arr = np.ascontiguousarray(np.asarray(budgets, dtype=np.int32).reshape(-1))
    return arr, arr.ctypes.data_as(C.c_void_p)


def score(K, Qwin, scores=None, row_lse=None, ws=None):
    sh = shape_of(K, Qwin)
    L, H, N = sh.n_layers, sh.n_kv_heads, sh.n_tokens
    if scores is None:
        scores = torch.empty((L, H, N), dtype=torch.float32, device=K.device)
    if row_lse is None:
        row_lse = torch.empty((L, H, sh.group * sh.window), dtype=torch.float64, device=K.device)
    ws = _ws(sh, 0, 0, ws, K.device)
    _check(load_library().obf_score(C.byref(sh), _ptr(K), _ptr(Qwin), _ptr(scores), _ptr(row_lse), _ptr(ws),
                                    ws.numel(), _stream()))
    return scores, row_lse


def select_topk(shape: _Shape, scores, budget: int = 0, budgets=None, max_budget: Optional[int] = None,
                idx=None, n_keep=None):
    L, H = shape.n_layers, shape.n_kv_heads
    keep, bptr = _budgets_arg(budgets)
    if max_budget is None:
        max_budget = int(min(shape.n_tokens, max(keep) if keep is not None else budget))
    if idx is None:
        idx = torch.empty((L, H, max_budget), dtype=torch.int32, device=scores.device)
    if n_keep is None:
        n_keep = torch.empty((L, H), dtype=torch.int32, device=scores.device)
    _check(load_library().obf_select_topk(C.byref(shape), _ptr(scores), bptr, budget, max_budget, _ptr(idx), _ptr(n_keep),
                                          None, 0, _stream()))
    return idx, n_keep


def refine_boundary(K, Qwin, scores, row_lse, idx, n_keep, ws=None):
    sh = shape_of(K, Qwin)
    max_budget = idx.shape[-1]
    ws = _ws(sh, max_budget, 0, ws, K.device)
    _check(load_library().obf_refine_boundary(C.byref(sh), _ptr(K), _ptr(Qwin), _ptr(scores), _ptr(row_lse), max_budget,
                                              _ptr(idx), _ptr(n_keep), _ptr(ws), ws.numel(), _stream()))
    return idx


def gather(shape: _Shape, K, V, idx, n_keep, K_out=None, V_out=None):
    L, H, d = shape.n_layers, shape.n_kv_heads, shape.head_dim
    max_budget = idx.shape[-1]
    src = K if K is not None else V
    if K is not None and K_out is None:
        K_out = torch.empty((L, H, max_budget, d), dtype=src.dtype, device=src.device)
    if V is not None and V_out is None:
        V_out = torch.empty((L, H, max_budget, d), dtype=src.dtype, device=src.device)
    _check(load_library().obf_gather(C.byref(shape), _ptr(K), _ptr(V), _ptr(idx), _ptr(n_keep), max_budget, _ptr(K_out),
                                     _ptr(V_out), _stream()))
    return K_out, V_out


def backfill(shape: _Shape, V, scores, idx, n_keep, rank: int, V_out, delta_out=None, diag=None, ws=None,
             variant: Optional[_Variant] = None):
    max_budget = idx.shape[-1]
    ws = _ws(shape, max_budget, rank, ws, V.device)
    if variant is not None:
        _check(load_library().obf_backfill_variant(C.byref(shape), _ptr(V), _ptr(scores), _ptr(idx), _ptr(n_keep), max_budget,
                                                   rank, C.byref(variant), _ptr(V_out), _ptr(delta_out), _ptr(diag),
                                                   _ptr(ws), ws.numel(), _stream()))
        return V_out
    _check(load_library().obf_backfill(C.byref(shape), _ptr(V), _ptr(scores), _ptr(idx), _ptr(n_keep), max_budget, rank,
                                       _ptr(V_out), _ptr(delta_out), _ptr(diag), _ptr(ws), ws.numel(), _stream()))
    return V_out


def compress_relay(K, V, Qwin, budget: int = 0, rank: int = 0, budgets=None, max_budget: Optional[int] = None,
                   out=None, ws=None, want_scores=False, want_delta=False, want_diag=False, layerwise=False,
                   variant: Optional[_Variant] = None, n_tokens: Optional[int] = None, sink: Optional[int] = None):
    """Fused relay compression.  Returns a dict of output tensors (device).  layerwise: one index set per layer
    (budgets then holds one entry per layer).  variant: an obf_variant_t from make_variant (the variant entry point).
    n_tokens / sink: the window entry point; K and V are then right-padded storage [L,H,stride,d] of which the first
    n_tokens rows per head are real, the first `sink` of them the protected sink."""
    sh = shape_of(K, Qwin)
    window = None
    if n_tokens is not None or sink is not None:
        window = _Window(K.shape[2], int(sink or 0))
        if n_tokens is not None:
            sh.n_tokens = int(n_tokens)
    L, H, d, N = sh.n_layers, sh.n_kv_heads, sh.head_dim, sh.n_tokens
    keep, bptr = _budgets_arg(budgets)
    if max_budget is None:
        max_budget = int(min(N, max(keep) if keep is not None else budget))
    dev = K.device
    o = out if out is not None else {}
    if "K_out" not in o:
        o["K_out"] = torch.empty((L, H, max_budget, d), dtype=K.dtype, device=dev)
    if "V_out" not in o:
        o["V_out"] = torch.empty((L, H, max_budget, d), dtype=K.dtype, device=dev)
    if "idx" not in o:
        o["idx"] = torch.empty((L, H, max_budget), dtype=torch.int32, device=dev)
    if "n_keep" not in o:
        o["n_keep"] = torch.empty((L, H), dtype=torch.int32, device=dev)
    if want_scores and "scores" not in o:
        o["scores"] = torch.empty((L, H, N), dtype=torch.float32, device=dev)
    if want_delta and "delta" not in o:
        o["delta"] = torch.empty((L, H, d), dtype=torch.float32, device=dev)
    if want_diag and "diag" not in o:
        o["diag"] = torch.empty((L, H, DIAG_DTYPE.itemsize), dtype=torch.uint8, device=dev)
    ws = _ws(sh, max_budget, rank, ws, dev)
    if window is not None:
        _check(load_library().obf_compress_relay_window(
            C.byref(sh), C.byref(window), _ptr(K), _ptr(V), _ptr(Qwin), bptr, budget, max_budget, rank, int(bool(layerwise)),
            C.byref(variant) if variant is not None else None,
            _ptr(o["K_out"]), _ptr(o["V_out"]), _ptr(o["idx"]), _ptr(o["n_keep"]), _ptr(o.get("scores")), _ptr(o.get("delta")),
            _ptr(o.get("diag")), _ptr(ws), ws.numel(), _stream()))
        o["ws"] = ws
        return o
    if variant is not None:
        _check(load_library().obf_compress_relay_variant(
            C.byref(sh), _ptr(K), _ptr(V), _ptr(Qwin), bptr, budget, max_budget, rank, int(bool(layerwise)), C.byref(variant),
            _ptr(o["K_out"]), _ptr(o["V_out"]), _ptr(o["idx"]), _ptr(o["n_keep"]), _ptr(o.get("scores")), _ptr(o.get("delta")),
            _ptr(o.get("diag")), _ptr(ws), ws.numel(), _stream()))
        o["ws"] = ws
        return o
    fn = load_library().obf_compress_relay_layerwise if layerwise else load_library().obf_compress_relay
    _check(fn(
        C.byref(sh), _ptr(K), _ptr(V), _ptr(Qwin), bptr, budget, max_budget, rank, _ptr(o["K_out"]), _ptr(o["V_out"]),
        _ptr(o["idx"]), _ptr(o["n_keep"]), _ptr(o.get("scores")), _ptr(o.get("delta")), _ptr(o.get("diag")),
        _ptr(ws), ws.numel(), _stream()))
    o["ws"] = ws
    return o


def compress_relay_batch(K, V, Qwin, n_tokens, budget: int = 0, budgets=None, rank: int = 0, sink: int = 0,
                         max_budget: Optional[int] = None, want_diag=False, out=None, lanes=None):
    """obf_compress_relay_batch: K, V [S,L,H,stride,d] right-padded, Qwin [S,L,H*g,W,d], n_tokens the real length of each
    sample (host sequence), budgets one per sample.  Returns a dict of device tensors with a leading sample dimension.
    out: a dict returned by an earlier call of the same shape (its buffers and workspace are reused); lanes: hand over a
    workspace for that many samples in flight instead of what obf_workspace_bytes_batch() asks for."""
    S, L, H, stride, d = K.shape
    sh = shape_of(K[0], Qwin[0])
    lens = np.ascontiguousarray(np.asarray(n_tokens, dtype=np.int32).reshape(-1))
    keep, bptr = _budgets_arg(budgets)
    if max_budget is None:
        per = keep if keep is not None else np.full(S, budget)
        max_budget = int(max(min(int(b), int(n) - sink) for b, n in zip(per, lens)))
    dev = K.device
    lib = load_library()
    if out is not None:
        o, ws = out, out["ws"]
    else:
        o = {"K_out": torch.empty((S, L, H, max_budget, d), dtype=K.dtype, device=dev),
             "V_out": torch.empty((S, L, H, max_budget, d), dtype=K.dtype, device=dev),
             "idx": torch.empty((S, L, H, max_budget), dtype=torch.int32, device=dev),
             "n_keep": torch.empty((S, L, H), dtype=torch.int32, device=dev)}
        if want_diag:
            o["diag"] = torch.empty((S, L, H, DIAG_DTYPE.itemsize), dtype=torch.uint8, device=dev)
        nbytes = lib.obf_workspace_bytes_batch(C.byref(sh), S, stride, max_budget, rank)
        if lanes is not None:
            nbytes = min(nbytes, int(lanes) * lib.obf_workspace_bytes_batch(C.byref(sh), 1, stride, max_budget, rank))
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    _check(lib.obf_compress_relay_batch(C.byref(sh), S, lens.ctypes.data_as(C.c_void_p), stride, sink, _ptr(K), _ptr(V), _ptr(Qwin),
                                        bptr, budget, max_budget, rank, _ptr(o["K_out"]), _ptr(o["V_out"]), _ptr(o["idx"]),
                                        _ptr(o["n_keep"]), _ptr(o.get("diag")), _ptr(ws), ws.numel(), _stream()))
    o["ws"] = ws
    return o


def quantize_rows(X: torch.Tensor, bits: int = 8):
    """obf_quantize_rows on X [..., d]: returns (codes uint8, scale, zero) with scale / zero as float16 tensors."""
    d = X.shape[-1]
    rows = X.numel() // d
    dt = OBF_BF16 if X.dtype == torch.bfloat16 else OBF_F32
    codes = torch.empty((rows, d if bits == 8 else d // 2), dtype=torch.uint8, device=X.device)
    scale = torch.empty((rows,), dtype=torch.float16, device=X.device)
    zero = torch.empty((rows,), dtype=torch.float16, device=X.device)
    _check(load_library().obf_quantize_rows(_ptr(X), rows, d, dt, bits, _ptr(codes), _ptr(scale), _ptr(zero), _stream()))
    return codes, scale, zero


def dequantize_rows(codes, scale, zero, d: int, dtype: torch.dtype, bits: int = 8):
    rows = scale.numel()
    X = torch.empty((rows, d), dtype=dtype, device=codes.device)
    dt = OBF_BF16 if dtype == torch.bfloat16 else OBF_F32
    _check(load_library().obf_dequantize_rows(_ptr(codes), _ptr(scale), _ptr(zero), rows, d, dt, bits, _ptr(X), _stream()))
    return X


def cache_merge(shape: _Shape, K, V, scores, idx, n_keep, K_out, V_out, route=None, ws=None):
    """obf_cache_merge on gathered rows; V_out is updated in place.  Returns the route tensor if one was passed."""
    max_budget = idx.shape[-1]
    ws = _ws(shape, max_budget, 0, ws, K.device)
    _check(load_library().obf_cache_merge(C.byref(shape), _ptr(K), _ptr(V), _ptr(scores), _ptr(idx), _ptr(n_keep), max_budget,
                                          _ptr(K_out), _ptr(V_out), _ptr(route), _ptr(ws), ws.numel(), _stream()))
    return route


def compress_relay_merge(K, V, Qwin, budget: int = 0, budgets=None, max_budget: Optional[int] = None, want_scores=False,
                         want_route=False, ws=None):
    """obf_compress_relay_merge: the cache-merging comparison system (App. E) end to end.  Returns a dict of device tensors."""
    sh = shape_of(K, Qwin)
    L, H, d, N = sh.n_layers, sh.n_kv_heads, sh.head_dim, sh.n_tokens
    keep, bptr = _budgets_arg(budgets)
    if max_budget is None:
        max_budget = int(min(N, max(keep) if keep is not None else budget))
    dev = K.device
    o = {"K_out": torch.empty((L, H, max_budget, d), dtype=K.dtype, device=dev),
         "V_out": torch.empty((L, H, max_budget, d), dtype=K.dtype, device=dev),
         "idx": torch.empty((L, H, max_budget), dtype=torch.int32, device=dev),
         "n_keep": torch.empty((L, H), dtype=torch.int32, device=dev)}
    if want_scores:
        o["scores"] = torch.empty((L, H, N), dtype=torch.float32, device=dev)
    if want_route:
        o["route"] = torch.empty((L, H, N), dtype=torch.int32, device=dev)
    ws = _ws(sh, max_budget, 0, ws, dev)
    _check(load_library().obf_compress_relay_merge(C.byref(sh), _ptr(K), _ptr(V), _ptr(Qwin), bptr, budget, max_budget,
                                                   _ptr(o["K_out"]), _ptr(o["V_out"]), _ptr(o["idx"]), _ptr(o["n_keep"]),
                                                   _ptr(o.get("scores")), _ptr(o.get("route")), _ptr(ws), ws.numel(), _stream()))
    o["ws"] = ws
    return o


def compress_relay_static(K, V, Qwin, out, budget: int = 0, rank: int = 0, budgets=None):
    """obf_compress_relay_static: the fused call on the library's built-in scratch array.  `out` holds the caller's
    K_out, V_out [L,H,max_budget,d], idx [L,H,max_budget] and n_keep [L,H]; nothing is allocated here or in the library."""
    sh = shape_of(K, Qwin)
    keep, bptr = _budgets_arg(budgets)          # `keep` holds the host array until the call has returned
    max_budget = out["idx"].shape[-1]
    _check(load_library().obf_compress_relay_static(C.byref(sh), _ptr(K), _ptr(V), _ptr(Qwin), bptr, budget, max_budget, rank,
                                                    _ptr(out["K_out"]), _ptr(out["V_out"]), _ptr(out["idx"]),
                                                    _ptr(out["n_keep"]), _stream()))
    return out


def append_message(prev_K, prev_V, prev_len, keep_K, keep_V, n_keep, gen_K, gen_V, msg_stride: int, prev_len_all: int = 0):
    """M = [prev; keep; gen] per head (obf_append_message).  Parts are [..., rows, d] tensors (leading dims = heads) or None;
    prev_len / n_keep int32 device tensors (prev_len None: every head has prev_len_all rows).  Returns (msg_K, msg_V, msg_len)."""
    ref = next(t for t in (keep_K, prev_K, gen_K) if t is not None)
    d = ref.shape[-1]
    heads = int(np.prod(ref.shape[:-2]))
    dt = OBF_BF16 if ref.dtype == torch.bfloat16 else OBF_F32
    msg_K = torch.empty((heads, msg_stride, d), dtype=ref.dtype, device=ref.device)
    msg_V = torch.empty_like(msg_K)
    msg_len = torch.empty((heads,), dtype=torch.int32, device=ref.device)
    rows = lambda t: 0 if t is None else t.shape[-2]
    _check(load_library().obf_append_message(
        heads, d, dt, _ptr(prev_K), _ptr(prev_V), _ptr(prev_len), prev_len_all, rows(prev_K),
        _ptr(keep_K), _ptr(keep_V), _ptr(n_keep), rows(keep_K), _ptr(gen_K), _ptr(gen_V), rows(gen_K), rows(gen_K),
        _ptr(msg_K), _ptr(msg_V), _ptr(msg_len), msg_stride, _stream()))
    return msg_K, msg_V, msg_len


def diag_to_numpy(diag: torch.Tensor) -> np.ndarray:
    """Device diag bytes [L,H,sizeof(obf_diag_t)] -> structured numpy array [L,H]."""
    a = diag.cpu().numpy()
    return a.view(DIAG_DTYPE).reshape(a.shape[0], a.shape[1])


def profile_enable(stage: int) -> None:
    _check(load_library().obf_profile_enable(stage))


def profile_read():
    """(total milliseconds, launches) of the profiled stage since the last read."""
    ms, n = C.c_double(0.0), C.c_int32(0)
    _check(load_library().obf_profile_read(C.byref(ms), C.byref(n)))
    return ms.value, n.value


def profile_stages():
    lib = load_library()
    return [lib.obf_profile_stage_name(i).decode() for i in range(lib.obf_profile_stage_count())]
