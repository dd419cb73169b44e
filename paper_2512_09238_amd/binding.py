"""ctypes binding of libtca.so: argument marshalling only.

Every function has the name and the argument order of its C declaration in
include/tca.h (diagnostics: include/tca_diag.h).  Device arrays are torch CUDA tensors (used for memory and
streams only); host arrays are numpy.  Nothing here computes any step of the
method, and there is no CPU fallback: if the library is missing, importing
this module raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtca.so")

TCA_BF16, TCA_F32 = 0, 1
TCA_METRIC_HHI, TCA_METRIC_ENTROPY = 0, 1
TCA_SHARE_HEAD, TCA_SHARE_GROUP = 0, 1
TCA_KV_NATIVE, TCA_KV_FP8 = 0, 1
TCA_PART_ALL, TCA_PART_WINDOW, TCA_PART_GLOBAL = 0, 1, 2
TCA_ROPE_HALF, TCA_ROPE_INTERLEAVED = 0, 1
TCA_OK, TCA_ERR_INVALID, TCA_ERR_UNSUPPORTED, TCA_ERR_WORKSPACE, TCA_ERR_HIP = 0, -1, -2, -3, -4

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2512_09238_amd.build` "
        "(or __graft_entry__.build()).  There is no fallback path."
    )
# torch is imported before the library is loaded: the process must hold ONE HIP runtime, and
# torch ships its own copy.  Loaded in this order, libtca.so binds to the runtime torch has
# already mapped, so that streams and device pointers mean the same thing on both sides;
# loaded first, it would pull in a second runtime that does not see torch's device context.
import torch  # noqa: E402,F401

lib = C.CDLL(LIB_PATH)


class tca_params(C.Structure):
    _fields_ = [
        ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("block", C.c_int32), ("window", C.c_int32), ("dtype", C.c_int32),
        ("alpha", C.c_double), ("scale", C.c_double), ("metric", C.c_int32), ("share", C.c_int32),
    ]


class tca_cache(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("cap_rows", C.c_int64),
        ("idx", C.c_void_p), ("Kg", C.c_void_p), ("Vg", C.c_void_p), ("n_rows", C.c_void_p),
        ("ringK", C.c_void_p), ("ringV", C.c_void_p), ("length", C.c_void_p),
        ("kv_format", C.c_int32), ("Kg_scale", C.c_void_p), ("Vg_scale", C.c_void_p),
        ("ringK_scale", C.c_void_p), ("ringV_scale", C.c_void_p),
    ]


_P = C.POINTER
_dbl_p, _i64_p, _i32_p = _P(C.c_double), _P(C.c_int64), _P(C.c_int32)

EXPORTS = {
    "tca_selection_heads": (C.c_int, [_P(tca_params)]),
    "tca_num_counts": (C.c_int, [C.c_int]),
    "tca_make_candidates": (C.c_int, [C.c_int, C.c_int, C.c_double, _dbl_p]),
    "tca_config_from_budget": (C.c_int, [C.c_int, C.c_double, C.c_double, _dbl_p]),
    "tca_psi_counts": (C.c_int, [C.c_int, C.c_int64, _dbl_p, _i64_p]),
    "tca_select_rows": (C.c_int64, [_P(tca_params), C.c_int64, _dbl_p, _i64_p]),
    "tca_decode_budget": (C.c_int, [C.c_int, _dbl_p]),
    "tca_select_workspace_bytes": (C.c_size_t, [_P(tca_params), C.c_int64]),
    "tca_prefill_workspace_bytes": (C.c_size_t, [_P(tca_params), C.c_int64, C.c_int64]),
    "tca_decode_workspace_bytes": (C.c_size_t, [_P(tca_params), C.c_int, C.c_int64]),
    "tca_calibrate_workspace_bytes": (C.c_size_t, [_P(tca_params), C.c_int64, C.c_int]),
    "tca_probe_workspace_bytes": (C.c_size_t, []),
    "tca_probe_mfma": (C.c_int, [C.c_int, C.c_int, _dbl_p, _dbl_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "tca_select": (C.c_int, [_P(tca_params), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                             C.c_int64, _dbl_p, _i64_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                             C.c_void_p, C.c_size_t, C.c_void_p]),
    "tca_prefill": (C.c_int, [_P(tca_params), C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p,
                              C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, _i64_p, C.c_void_p,
                              C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "tca_prefill_part": (C.c_int, [_P(tca_params), C.c_int, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p,
                                   C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, _i64_p, C.c_void_p,
                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "tca_prefill_merge": (C.c_int, [_P(tca_params), C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_void_p]),
    "tca_select_prefill_overlapped": (C.c_int, [_P(tca_params), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                C.c_int64, C.c_int64, C.c_int64, _dbl_p, _i64_p, C.c_void_p,
                                                C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t,
                                                C.c_void_p, C.c_void_p]),
    "tca_cache_load_window": (C.c_int, [_P(tca_params), _P(tca_cache), C.c_int, C.c_void_p, C.c_void_p,
                                        C.c_int64, C.c_int64, C.c_void_p]),
    "tca_cache_load_global": (C.c_int, [_P(tca_params), _P(tca_cache), C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                        _i64_p, C.c_void_p, C.c_void_p]),
    "tca_decode": (C.c_int, [_P(tca_params), _P(tca_cache), _i64_p, C.c_void_p, C.c_void_p, C.c_void_p,
                             _dbl_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "tca_decode_static": (C.c_int, [_P(tca_params), _P(tca_cache), _i64_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                    _dbl_p, C.c_void_p, C.c_void_p]),
    "tca_calibrate_budgets": (C.c_int, [_P(tca_params), C.c_void_p, C.c_void_p, C.c_int64, C.c_int,
                                        C.c_double, C.c_double, _dbl_p, _i32_p, _dbl_p, _i64_p, _i32_p,
                                        C.c_void_p, C.c_size_t, C.c_void_p]),
    "tca_diag_prefill_clocks": (None, [C.c_int]),
    "tca_diag_prefill_variant": (C.c_int, [C.c_int]),
    "tca_diag_prefill_xcd_plan": (C.c_int64, [_P(tca_params), C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_void_p]),
    "tca_calibrate_layers": (C.c_int, [_P(tca_params), C.c_int, _P(C.c_void_p), _P(C.c_void_p), C.c_int64, C.c_int,
                                       C.c_double, C.c_double, _dbl_p, _i32_p, _dbl_p, _i64_p, _i32_p,
                                       C.c_void_p, C.c_size_t, C.c_void_p]),
    "tca_rope": (C.c_int, [_P(tca_params), C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_double, C.c_int, C.c_void_p]),
    "tca_qkv_project": (C.c_int, [_P(tca_params), C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                  C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p]),
    "tca_strerror": (C.c_char_p, [C.c_int]),
    "tca_last_error": (C.c_char_p, []),
}
for _name, (_res, _args) in EXPORTS.items():
    _f = getattr(lib, _name)
    _f.restype, _f.argtypes = _res, _args


class TcaError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"{lib.tca_strerror(code).decode()} ({code}): {lib.tca_last_error().decode()}")


def _check(rc: int) -> int:
    if rc < 0:
        raise TcaError(int(rc))
    return int(rc)


def _dp(t):
    """Device pointer of a torch tensor (None -> NULL; an int is taken as a device address)."""
    if t is None:
        return None
    if isinstance(t, int):                      # a device address (a row inside a caller's buffer)
        return C.c_void_p(t)
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("device arguments must be contiguous CUDA tensors")
    return C.c_void_p(t.data_ptr())


def _host(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def _stream(stream):
    if stream is not None:
        return C.c_void_p(int(stream))
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_params(n_q_heads, n_kv_heads, head_dim, block, window, dtype, alpha=0.5, scale=0.0,
                metric=TCA_METRIC_HHI, share=TCA_SHARE_HEAD) -> tca_params:
    return tca_params(n_q_heads, n_kv_heads, head_dim, block, window, dtype, alpha, scale, metric, share)


# ---------------------------------------------------------------- host --
def tca_selection_heads(prm: tca_params) -> int:
    return _check(lib.tca_selection_heads(C.byref(prm)))


def tca_num_counts(b: int) -> int:
    return _check(lib.tca_num_counts(b))


def tca_make_candidates(b: int, M: int, sigma: float) -> np.ndarray:
    out = np.empty((M, tca_num_counts(b)), np.float64)
    _check(lib.tca_make_candidates(b, M, sigma, out.ctypes.data_as(_dbl_p)))
    return out


def tca_config_from_budget(b: int, sigma: float, frac: float) -> np.ndarray:
    out = np.empty(tca_num_counts(b), np.float64)
    _check(lib.tca_config_from_budget(b, sigma, frac, out.ctypes.data_as(_dbl_p)))
    return out


def tca_psi_counts(b: int, m: int, p) -> np.ndarray:
    p = _host(p, np.float64)
    out = np.empty(tca_num_counts(b), np.int64)
    _check(lib.tca_psi_counts(b, m, p.ctypes.data_as(_dbl_p), out.ctypes.data_as(_i64_p)))
    return out


def tca_select_rows(prm: tca_params, n_blocks: int, p):
    p = _host(p, np.float64)
    rows = np.empty(tca_selection_heads(prm), np.int64)
    total = _check(lib.tca_select_rows(C.byref(prm), n_blocks, p.ctypes.data_as(_dbl_p), rows.ctypes.data_as(_i64_p)))
    return total, rows


def tca_decode_budget(b: int, p) -> int:
    p = _host(p, np.float64)
    return _check(lib.tca_decode_budget(b, p.ctypes.data_as(_dbl_p)))


def tca_select_workspace_bytes(prm, n_tokens: int) -> int:
    return int(lib.tca_select_workspace_bytes(C.byref(prm), n_tokens))


def tca_prefill_workspace_bytes(prm, n_queries: int, cap_rows: int) -> int:
    return int(lib.tca_prefill_workspace_bytes(C.byref(prm), n_queries, cap_rows))


def tca_decode_workspace_bytes(prm, batch: int, max_head_rows: int) -> int:
    return int(lib.tca_decode_workspace_bytes(C.byref(prm), batch, max_head_rows))


def tca_calibrate_workspace_bytes(prm, L_cal: int, M: int) -> int:
    return int(lib.tca_calibrate_workspace_bytes(C.byref(prm), L_cal, M))


# -------------------------------------------------------------- device --
def _ws_args(ws):
    if ws is None:
        return None, 0
    return _dp(ws), ws.numel() * ws.element_size()


def tca_select(prm, q_last, K, V, kv_stride, pos0, n_tokens, p, offs, n_rows, idx, Kg, Vg, ws, stream=None):
    p = _host(p, np.float64)
    offs = _host(offs, np.int64)
    wsp, wsb = _ws_args(ws)
    _check(lib.tca_select(C.byref(prm), _dp(q_last), _dp(K), _dp(V), kv_stride, pos0, n_tokens,
                          p.ctypes.data_as(_dbl_p), offs.ctypes.data_as(_i64_p), _dp(n_rows), _dp(idx),
                          _dp(Kg), _dp(Vg), wsp, wsb, _stream(stream)))


def tca_prefill(prm, Q, q_pos0, n_queries, K, V, kv_stride, idx, Kg, Vg, offs, n_rows, O, lse, ws, stream=None):
    offs = _host(offs, np.int64)
    wsp, wsb = _ws_args(ws)
    _check(lib.tca_prefill(C.byref(prm), _dp(Q), q_pos0, n_queries, _dp(K), _dp(V), kv_stride, _dp(idx),
                           _dp(Kg), _dp(Vg), offs.ctypes.data_as(_i64_p), _dp(n_rows), _dp(O), _dp(lse),
                           wsp, wsb, _stream(stream)))


def tca_prefill_part(prm, part, Q, q_pos0, n_queries, K, V, kv_stride, idx, Kg, Vg, offs, n_rows, O, lse, ws, stream=None):
    offs = _host(offs, np.int64)
    wsp, wsb = _ws_args(ws)
    _check(lib.tca_prefill_part(C.byref(prm), part, _dp(Q), q_pos0, n_queries, _dp(K), _dp(V), kv_stride, _dp(idx),
                                _dp(Kg), _dp(Vg), offs.ctypes.data_as(_i64_p), _dp(n_rows), _dp(O), _dp(lse),
                                wsp, wsb, _stream(stream)))


def tca_prefill_merge(prm, n_queries, O_a, lse_a, O_b, lse_b, lse_out=None, stream=None):
    _check(lib.tca_prefill_merge(C.byref(prm), n_queries, _dp(O_a), _dp(lse_a), _dp(O_b), _dp(lse_b), _dp(lse_out),
                                 _stream(stream)))


def tca_select_prefill_overlapped(prm, q_last, Q, K, V, kv_stride, pos0, n_tokens, p, offs, n_rows, idx, Kg, Vg, O,
                                  O_part, lse_parts, ws_select, ws_prefill, side_stream, stream=None):
    p = _host(p, np.float64)
    offs = _host(offs, np.int64)
    wsp, wsb = _ws_args(ws_select)
    wpp, wpb = _ws_args(ws_prefill)
    _check(lib.tca_select_prefill_overlapped(C.byref(prm), _dp(q_last), _dp(Q), _dp(K), _dp(V), kv_stride, pos0,
                                             n_tokens, p.ctypes.data_as(_dbl_p), offs.ctypes.data_as(_i64_p),
                                             _dp(n_rows), _dp(idx), _dp(Kg), _dp(Vg), _dp(O), _dp(O_part),
                                             _dp(lse_parts), wsp, wsb, wpp, wpb, _stream(stream),
                                             C.c_void_p(int(side_stream))))


def make_cache(batch, cap_rows, idx, Kg, Vg, n_rows, ringK, ringV, length, kv_format=TCA_KV_NATIVE,
               Kg_scale=None, Vg_scale=None, ringK_scale=None, ringV_scale=None) -> tca_cache:
    ptr = lambda t: None if t is None else t.data_ptr()
    return tca_cache(batch, cap_rows, idx.data_ptr(), Kg.data_ptr(), Vg.data_ptr(), n_rows.data_ptr(),
                     ringK.data_ptr(), ringV.data_ptr(), length.data_ptr(), kv_format,
                     ptr(Kg_scale), ptr(Vg_scale), ptr(ringK_scale), ptr(ringV_scale))


def tca_cache_load_window(prm, cache, seq, K, V, kv_stride, L, stream=None):
    _check(lib.tca_cache_load_window(C.byref(prm), C.byref(cache), seq, _dp(K), _dp(V), kv_stride, L,
                                     _stream(stream)))


def tca_cache_load_global(prm, cache, seq, idx, Kg, Vg, offs, n_rows, stream=None):
    offs = _host(offs, np.int64)
    _check(lib.tca_cache_load_global(C.byref(prm), C.byref(cache), seq, _dp(idx), _dp(Kg), _dp(Vg),
                                     offs.ctypes.data_as(_i64_p), _dp(n_rows), _stream(stream)))


def tca_decode(prm, cache, offs, q, k_new, v_new, p, O, ws, stream=None):
    p = _host(p, np.float64)
    offs = _host(offs, np.int64)
    wsp, wsb = _ws_args(ws)
    _check(lib.tca_decode(C.byref(prm), C.byref(cache), offs.ctypes.data_as(_i64_p), _dp(q), _dp(k_new),
                          _dp(v_new), p.ctypes.data_as(_dbl_p), _dp(O), wsp, wsb, _stream(stream)))


TCA_DECODE_STATIC_BYTES = 32 << 20


def tca_decode_static(prm, cache, offs, q, k_new, v_new, p, O, stream=None):
    p = _host(p, np.float64)
    offs = _host(offs, np.int64)
    _check(lib.tca_decode_static(C.byref(prm), C.byref(cache), offs.ctypes.data_as(_i64_p), _dp(q), _dp(k_new),
                                 _dp(v_new), p.ctypes.data_as(_dbl_p), _dp(O), _stream(stream)))


def tca_calibrate_budgets(prm, Qcal, Kcal, L_cal, M, sigma, tau, ws, stream=None):
    """Returns dict(p_star [Hs,nk], cand_idx [Hs], a [Hs,M], n [Hs,M], fallback [Hs])."""
    Hq, nk = tca_selection_heads(prm), tca_num_counts(prm.block)
    p_star = np.empty((Hq, nk), np.float64)
    cand = np.empty(Hq, np.int32)
    a = np.empty((Hq, M), np.float64)
    n = np.empty((Hq, M), np.int64)
    fb = np.empty(Hq, np.int32)
    wsp, wsb = _ws_args(ws)
    _check(lib.tca_calibrate_budgets(C.byref(prm), _dp(Qcal), _dp(Kcal), L_cal, M, sigma, tau,
                                     p_star.ctypes.data_as(_dbl_p), cand.ctypes.data_as(_i32_p),
                                     a.ctypes.data_as(_dbl_p), n.ctypes.data_as(_i64_p),
                                     fb.ctypes.data_as(_i32_p), wsp, wsb, _stream(stream)))
    return {"p_star": p_star, "cand_idx": cand, "a": a, "n": n, "fallback": fb}


def tca_calibrate_layers(prm, Qcals, Kcals, L_cal, M, sigma, tau, ws, stream=None):
    """Qcals, Kcals: one device tensor per layer.  Returns dict(p_star [layers,Hs,nk], cand_idx [layers,Hs],
    a [layers,Hs,M], n [layers,Hs,M], fallback [layers,Hs])."""
    nl, Hs, nk = len(Qcals), tca_selection_heads(prm), tca_num_counts(prm.block)
    qp = (C.c_void_p * nl)(*[_dp(t) for t in Qcals])
    kp = (C.c_void_p * nl)(*[_dp(t) for t in Kcals])
    p_star = np.empty((nl, Hs, nk), np.float64)
    cand = np.empty((nl, Hs), np.int32)
    a = np.empty((nl, Hs, M), np.float64)
    n = np.empty((nl, Hs, M), np.int64)
    fb = np.empty((nl, Hs), np.int32)
    wsp, wsb = _ws_args(ws)
    _check(lib.tca_calibrate_layers(C.byref(prm), nl, qp, kp, L_cal, M, sigma, tau,
                                    p_star.ctypes.data_as(_dbl_p), cand.ctypes.data_as(_i32_p),
                                    a.ctypes.data_as(_dbl_p), n.ctypes.data_as(_i64_p), fb.ctypes.data_as(_i32_p),
                                    wsp, wsb, _stream(stream)))
    return {"p_star": p_star, "cand_idx": cand, "a": a, "n": n, "fallback": fb}


def tca_rope(prm, X, n_heads, n_rows, pos0, base=10000.0, pairing=TCA_ROPE_HALF, stream=None):
    _check(lib.tca_rope(C.byref(prm), _dp(X), n_heads, n_rows, pos0, base, pairing, _stream(stream)))


def tca_qkv_project(prm, X, n_tokens, hidden, W, bias, Q, q_token_stride, q_head_stride, K, V, kv_token_stride,
                    kv_head_stride, stream=None):
    _check(lib.tca_qkv_project(C.byref(prm), _dp(X), n_tokens, hidden, _dp(W), _dp(bias) if bias is not None else None,
                               _dp(Q), q_token_stride, q_head_stride, _dp(K), _dp(V), kv_token_stride,
                               kv_head_stride, _stream(stream)))


# --------------------------------------------------------- diagnostics --
def tca_probe_workspace_bytes() -> int:
    return int(lib.tca_probe_workspace_bytes())


def tca_probe_mfma(random_operands: bool, iters: int, ws, stream=None):
    """Returns (TFLOP/s reached by a register-only bf16 MFMA loop, shader clock in GHz)."""
    tf, ghz = C.c_double(0.0), C.c_double(0.0)
    wsp, wsb = _ws_args(ws)
    _check(lib.tca_probe_mfma(int(bool(random_operands)), int(iters), C.byref(tf), C.byref(ghz), wsp, wsb,
                              _stream(stream)))
    return tf.value, ghz.value


def tca_diag_prefill_clocks(enable: bool) -> None:
    lib.tca_diag_prefill_clocks(int(bool(enable)))


def tca_diag_prefill_variant(variant: int) -> None:
    _check(lib.tca_diag_prefill_variant(int(variant)))


def tca_diag_prefill_xcd_plan(prm, offs, q_pos0: int, n_queries: int, part: int = 0, gather_free: bool = False):
    """Returns (start[9], workgroups): the ranges of the (head, query tile) sequence the eight XCDs take."""
    offs = np.ascontiguousarray(offs, dtype=np.int64)
    start = np.zeros(9, dtype=np.int32)
    n = lib.tca_diag_prefill_xcd_plan(C.byref(prm), offs.ctypes.data_as(C.c_void_p), q_pos0, n_queries, part,
                                      int(bool(gather_free)), start.ctypes.data_as(C.c_void_p))
    if n < 0:
        raise ValueError("tca_diag_prefill_xcd_plan: not a bf16 call with a head count that is a multiple of 8")
    return start, int(n)


def prefill_shader_clock_ghz(ws) -> float:
    """Average shader clock during the last completed bf16 tca_prefill that used `ws`
    (a torch uint8 tensor) while tca_diag_prefill_clocks was on: its first two uint64 are
    cycle and 100 MHz tick sums."""
    torch.cuda.synchronize()
    c = ws[:16].view(torch.int64).cpu().numpy()
    return float(c[0]) / (float(c[1]) * 10.0) if c[1] else 0.0
