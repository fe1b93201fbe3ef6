"""ctypes front end of the CPU oracle in ``moe_oracle.c`` (TEST INFRASTRUCTURE).

The oracle is the plain fp64 definition of the sparse MoE layer the DAOP paper
(arXiv 2501.10375) wraps: gating and top-k selection (Sec. II-A), per-sequence
expert activation counts (Sec. IV-B, Algorithm 1), next-layer prediction by the
next layer's gate on the same hidden state (Sec. III observation 3, Sec. IV-C)
and expert execution with the weighted combine (Sec. II-A, Algorithm 1's local
expert execution step).

Only tests, ``__graft_entry__.smoke()`` and the benchmark's ``cpu_baseline`` leg
may import this module.  It imports nothing from the GPU package and the GPU
package imports nothing from here.

Arrays are numpy.  A tensor's storage type is one of float32, float64 or
uint16 (bf16 bit patterns); all tensors of one call share it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")
_lib = None

_DTYPE_CODE = {np.dtype(np.float32): 0, np.dtype(np.uint16): 1, np.dtype(np.float64): 2}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, ip = ctypes.c_void_p, ctypes.c_int
        lib.oracle_route.argtypes = [ip, ip, ip, ip, ip, vp, vp, vp, vp, vp, vp, vp, vp, ip]
        lib.oracle_route.restype = ip
        lib.oracle_expert_ffn.argtypes = [ip, ip, ip, ip, ip, ip, vp, vp, vp, vp, vp, vp, vp, ip, vp]
        lib.oracle_expert_ffn.restype = ip
        lib.oracle_expert_ffn_precalc.argtypes = [ip, ip, ip, ip, ip, ip, vp, vp, vp, vp, vp, vp, vp, vp, vp, ip, vp]
        lib.oracle_expert_ffn_precalc.restype = ip
        lib.oracle_num_threads.restype = ip
        lib.oracle_set_num_threads.argtypes = [ip]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def _code(*arrays) -> int:
    dts = {a.dtype for a in arrays}
    if len(dts) != 1:
        raise TypeError(f"all tensors of one call must share a storage type, got {dts}")
    dt = dts.pop()
    if dt not in _DTYPE_CODE:
        raise TypeError(f"unsupported storage type {dt}")
    return _DTYPE_CODE[dt]


def _c(a):
    return np.ascontiguousarray(a)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def route(x, wg, bias=None, k=2, counts=None):
    """Gate, softmax, top-k, renormalised weights, counts and near-tie margin.

    x [T,H], wg [E,H]; bias [E] or None.  ``counts`` (int32 [E]) is added to
    when given, else a fresh histogram is returned.
    Returns dict(idx int32 [T,k], w float64 [T,k], p float32 [T,E],
    margin float32 [T], counts int32 [E]).
    """
    x, wg = _c(x), _c(wg)
    T, H = x.shape
    E, H2 = wg.shape
    if H2 != H:
        raise ValueError("gate width does not match hidden size")
    code = _code(x, wg)
    b = None if bias is None else _c(np.asarray(bias, dtype=np.float64))
    idx = np.empty((T, k), dtype=np.int32)
    w = np.empty((T, k), dtype=np.float64)
    p = np.empty((T, E), dtype=np.float32)
    margin = np.empty((T,), dtype=np.float32)
    accumulate = counts is not None
    if counts is None:
        counts = np.zeros((E,), dtype=np.int32)
    elif counts.dtype != np.int32 or counts.shape != (E,) or not counts.flags.c_contiguous:
        raise ValueError("counts must be a contiguous int32 [E] array")
    rc = _load().oracle_route(T, H, E, k, code, _ptr(x), _ptr(wg), _ptr(b), _ptr(idx), _ptr(w),
                              _ptr(p), _ptr(margin), _ptr(counts), int(accumulate))
    if rc != 0:
        raise ValueError("oracle_route rejected its arguments")
    return {"idx": idx, "w": w, "p": p, "margin": margin, "counts": counts}


def expert_ffn(x, idx, w, w1, w3, w2, tokens=None):
    """SwiGLU experts and weighted combine for the listed tokens (all if None).

    x [T,H]; idx int32 [T,k]; w [T,k]; w1, w3 [E,F,H]; w2 [E,H,F].
    Returns y float64 [len(tokens), H].
    """
    x, w1, w3, w2 = _c(x), _c(w1), _c(w3), _c(w2)
    T, H = x.shape
    E, F, H1 = w1.shape
    if H1 != H or w3.shape != (E, F, H) or w2.shape != (E, H, F):
        raise ValueError("expert weight shapes do not match")
    code = _code(x, w1, w3, w2)
    idx = _c(np.asarray(idx, dtype=np.int32))
    k = idx.shape[1]
    w = _c(np.asarray(w, dtype=np.float64))
    if idx.shape != (T, k) or w.shape != (T, k):
        raise ValueError("idx / w must be [T,k]")
    if tokens is None:
        tok = np.arange(T, dtype=np.int32)
    else:
        tok = _c(np.asarray(tokens, dtype=np.int32))
    y = np.empty((tok.shape[0], H), dtype=np.float64)
    rc = _load().oracle_expert_ffn(T, H, F, E, k, code, _ptr(x), _ptr(idx), _ptr(w), _ptr(w1),
                                   _ptr(w3), _ptr(w2), _ptr(tok), tok.shape[0], _ptr(y))
    if rc != 0:
        raise ValueError("oracle_expert_ffn rejected its arguments")
    return y


def expert_ffn_precalc(x, x_stale, stale, idx, w, w1, w3, w2, tokens=None):
    """Expert execution where some selections were pre-calculated on an earlier hidden state (Sec. IV-C):
    selection (t, j) is evaluated on x_stale[t] where stale[t, j] is non-zero, on x[t] otherwise.

    x, x_stale [T,H]; stale [T,k] (bool / uint8); the rest as in ``expert_ffn``.
    Returns y float64 [len(tokens), H].
    """
    x, x_stale, w1, w3, w2 = _c(x), _c(x_stale), _c(w1), _c(w3), _c(w2)
    T, H = x.shape
    E, F, H1 = w1.shape
    if x_stale.shape != (T, H) or H1 != H or w3.shape != (E, F, H) or w2.shape != (E, H, F):
        raise ValueError("shapes do not match")
    code = _code(x, x_stale, w1, w3, w2)
    idx = _c(np.asarray(idx, dtype=np.int32))
    k = idx.shape[1]
    w = _c(np.asarray(w, dtype=np.float64))
    stale = _c((np.asarray(stale) != 0).astype(np.uint8))
    if idx.shape != (T, k) or w.shape != (T, k) or stale.shape != (T, k):
        raise ValueError("idx / w / stale must be [T,k]")
    tok = np.arange(T, dtype=np.int32) if tokens is None else _c(np.asarray(tokens, dtype=np.int32))
    y = np.empty((tok.shape[0], H), dtype=np.float64)
    rc = _load().oracle_expert_ffn_precalc(T, H, F, E, k, code, _ptr(x), _ptr(x_stale), _ptr(stale), _ptr(idx), _ptr(w),
                                           _ptr(w1), _ptr(w3), _ptr(w2), _ptr(tok), tok.shape[0], _ptr(y))
    if rc != 0:
        raise ValueError("oracle_expert_ffn_precalc rejected its arguments")
    return y


def predict_next(x, wg_next, bias_next=None, k=2):
    """Predicted experts of the next layer: that layer's gate applied to this
    layer's gate input.  Same outputs as ``route``; ``idx`` is the prediction."""
    return route(x, wg_next, bias_next, k)


def layer(x, wg, bias, w1, w3, w2, k=2, wg_next=None, bias_next=None, tokens=None):
    """One MoE layer: route, optional next-layer prediction, experts, combine."""
    r = route(x, wg, bias, k)
    out = {"idx": r["idx"], "w": r["w"], "p": r["p"], "margin": r["margin"], "counts": r["counts"]}
    if wg_next is not None:
        pr = predict_next(x, wg_next, bias_next, k)
        out["pred_idx"], out["pred_w"] = pr["idx"], pr["w"]
        out["pred_margin"], out["pred_counts"] = pr["margin"], pr["counts"]
    out["y"] = expert_ffn(x, r["idx"], r["w"], w1, w3, w2, tokens)
    return out
