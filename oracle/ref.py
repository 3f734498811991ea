"""numpy-facing wrapper of the C oracle (oracle/moe_oracle.c). Test infrastructure only.

bf16 tensors are numpy uint16 arrays of raw bits; everything is a host array.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB if os.path.exists(_build.LIB) else _build.build()
        _lib = C.CDLL(path)
        for name in ("moe_ref_logits", "moe_ref_logits_f64", "moe_ref_topk", "moe_ref_permute",
                     "moe_ref_gather", "moe_ref_layer_tokens", "moe_ref_expert_ffn",
                     "moe_ref_combine", "moe_ref_combine_bf16", "moe_ref_layer_staged"):
            getattr(_lib, name).restype = C.c_int
        _lib.moe_ref_num_threads.restype = C.c_int
    return _lib


def _p(a, dtype):
    if a is None:
        return None
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype)
    return a.ctypes.data_as(C.c_void_p)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what}: invalid argument (rc={rc})")


def num_threads() -> int:
    return lib().moe_ref_num_threads()


def set_threads(n: int) -> None:
    lib().moe_ref_set_threads(C.c_int(n))


def logits(x, w_router, bias=None):
    T, d = x.shape
    E = w_router.shape[1]
    out = np.empty((T, E), np.float32)
    _check(lib().moe_ref_logits(_p(x, np.uint16), _p(w_router, np.float32), _p(bias, np.float32),
                                T, d, E, _p(out, np.float32)), "logits")
    return out


def logits_f64(x, w_router, bias=None):
    T, d = x.shape
    E = w_router.shape[1]
    out = np.empty((T, E), np.float64)
    _check(lib().moe_ref_logits_f64(_p(x, np.uint16), _p(w_router, np.float32),
                                    _p(bias, np.float32), T, d, E, _p(out, np.float64)), "logits_f64")
    return out


def topk(lg, k):
    T, E = lg.shape
    idx = np.empty((T, k), np.int32)
    g = np.empty((T, k), np.float32)
    _check(lib().moe_ref_topk(_p(lg, np.float32), T, E, k, _p(idx, np.int32), _p(g, np.float32)),
           "topk")
    return idx, g


def permute(topk_idx, E):
    R = topk_idx.size
    counts = np.empty(E, np.int32)
    offsets = np.empty(E + 1, np.int32)
    perm = np.empty(R, np.int32)
    inv = np.empty(R, np.int32)
    flat = np.ascontiguousarray(topk_idx.reshape(-1))
    _check(lib().moe_ref_permute(_p(flat, np.int32), R, E, _p(counts, np.int32),
                                 _p(offsets, np.int32), _p(perm, np.int32), _p(inv, np.int32)),
           "permute")
    return counts, offsets, perm, inv


def gather(x, perm, k):
    R = perm.size
    d = x.shape[1]
    out = np.empty((R, d), np.uint16)
    _check(lib().moe_ref_gather(_p(x, np.uint16), _p(perm, np.int32), R, d, k, _p(out, np.uint16)),
           "gather")
    return out


def layer_tokens(x, w_router, bias, W1, W3, W2, k, tokens=None):
    """y[n,d] float64 (+ idx[n,k], g[n,k]) for the listed tokens (all if None)."""
    T, d = x.shape
    E, f, _ = W1.shape
    if tokens is None:
        n, tok = T, None
    else:
        tok = np.ascontiguousarray(np.asarray(tokens, np.int32))
        n = tok.size
    y = np.empty((n, d), np.float64)
    idx = np.empty((n, k), np.int32)
    g = np.empty((n, k), np.float32)
    _check(lib().moe_ref_layer_tokens(_p(x, np.uint16), _p(w_router, np.float32),
                                      _p(bias, np.float32), _p(W1, np.uint16), _p(W3, np.uint16),
                                      _p(W2, np.uint16), T, d, f, E, k, _p(tok, np.int32), n,
                                      _p(y, np.float64), _p(idx, np.int32), _p(g, np.float32)),
           "layer_tokens")
    return y, idx, g


def expert_ffn(x_perm, offsets, W1, W3, W2, rows=None, want_h=False):
    R, d = x_perm.shape
    E, f, _ = W1.shape
    if rows is None:
        n, rw = R, None
    else:
        rw = np.ascontiguousarray(np.asarray(rows, np.int32))
        n = rw.size
    y = np.empty((n, d), np.float64)
    h = np.empty((n, f), np.float64) if want_h else None
    _check(lib().moe_ref_expert_ffn(_p(x_perm, np.uint16), _p(offsets, np.int32), R, d, f, E,
                                    _p(W1, np.uint16), _p(W3, np.uint16), _p(W2, np.uint16),
                                    _p(rw, np.int32), n, _p(y, np.float64), _p(h, np.float64)),
           "expert_ffn")
    return (y, h) if want_h else y


def combine(y_perm, inv_perm, topk_w):
    T, k = topk_w.shape
    d = y_perm.shape[1]
    y = np.empty((T, d), np.float64)
    flat = np.ascontiguousarray(inv_perm.reshape(-1))
    if y_perm.dtype == np.uint16:
        fn, dt = lib().moe_ref_combine_bf16, np.uint16
    else:
        fn, dt = lib().moe_ref_combine, np.float64
    _check(fn(_p(y_perm, dt), _p(flat, np.int32), _p(topk_w, np.float32), T, d, k,
              _p(y, np.float64)), "combine")
    return y


def layer_staged(x, w_router, bias, W1, W3, W2, k, m):
    T, d = x.shape
    E, f, _ = W1.shape
    y = np.empty((T, d), np.float64)
    _check(lib().moe_ref_layer_staged(_p(x, np.uint16), _p(w_router, np.float32),
                                      _p(bias, np.float32), _p(W1, np.uint16), _p(W3, np.uint16),
                                      _p(W2, np.uint16), T, d, f, E, k, m, _p(y, np.float64)),
           "layer_staged")
    return y
