"""ctypes binding of include/daop_policy.h: the count-driven policy steps of DAOP on the device.

Argument marshalling only; every computation runs in the HIP library.  Tensors are contiguous CUDA
tensors; outputs are allocated here for convenience and returned.
"""
from __future__ import annotations

import ctypes

import torch

from . import moe
from .moe import _check, _p, _stream

EXPORTS = ("daop_similarity", "daop_window_variation", "daop_plan_swaps", "daop_memory_init", "daop_predict_degraded")
_ready = False


def lib() -> ctypes.CDLL:
    global _ready
    L = moe.lib()
    if not _ready:
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        L.daop_similarity.argtypes = [i32, i32, vp, vp, vp, vp]
        L.daop_window_variation.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp]
        L.daop_plan_swaps.argtypes = [i32, i32, vp, vp, ctypes.c_double, vp, vp, vp]
        L.daop_memory_init.argtypes = [i32, i32, vp, i32, vp, vp]
        L.daop_predict_degraded.argtypes = [ctypes.POINTER(moe.MoeShape), i32, vp, vp, vp, vp, vp, vp, vp]
        for name in EXPORTS:
            getattr(L, name).restype = ctypes.c_int
        _ready = True
    return L


def daop_similarity(counts_p: torch.Tensor, counts_d: torch.Tensor):
    """Eq. 1 on int32 [L, E] count matrices.  Returns (similarity, per-layer cosines) as fp64 tensors on the GPU."""
    L, E = counts_p.shape
    out = torch.empty(1 + L, dtype=torch.float64, device=counts_p.device)
    _check(lib().daop_similarity(L, E, _p(counts_p, torch.int32, (L, E), "counts_p"),
                                 _p(counts_d, torch.int32, (L, E), "counts_d"), _p(out), _stream()), "daop_similarity")
    return out[0], out[1:]


def daop_window_variation(idx: torch.Tensor, n_experts: int, window: int = 15):
    """Sec. VI-B on int32 [L, S, k] selections of S decode steps.  Returns (mean similarity of consecutive
    windows, per-pair similarities) as fp64 tensors on the GPU."""
    L, S, k = idx.shape
    n_pairs = max(S // window - 1, 0)
    out = torch.empty(2 + n_pairs, dtype=torch.float64, device=idx.device)   # one spare element keeps it non-empty
    _check(lib().daop_window_variation(L, n_experts, S, k, int(window), _p(idx, torch.int32, (L, S, k), "idx"), _p(out),
                                       _stream()), "daop_window_variation")
    return out[0], out[1:1 + n_pairs]


def daop_plan_swaps(counts: torch.Tensor, on_gpu: torch.Tensor, swap_in_out: float = 1.05):
    """Algorithm 1 over all layers; updates `on_gpu` (uint8 [L, E]) in place.
    Returns (swaps int32 [L, E // 2, 2], n_swaps int32 [L])."""
    L, E = counts.shape
    swaps = torch.empty((L, max(E // 2, 1), 2), dtype=torch.int32, device=counts.device)
    n_swaps = torch.empty(L, dtype=torch.int32, device=counts.device)
    _check(lib().daop_plan_swaps(L, E, _p(counts, torch.int32, (L, E), "counts"), _p(on_gpu, torch.uint8, (L, E), "on_gpu"),
                                 float(swap_in_out), _p(swaps) if E >= 2 else None, _p(n_swaps), _stream()),
           "daop_plan_swaps")
    return swaps[:, : E // 2], n_swaps


def daop_memory_init(calib_counts: torch.Tensor, slots: int) -> torch.Tensor:
    """Initial expert cache (uint8 [L, E]) from calibration counts and a number of GPU slots."""
    L, E = calib_counts.shape
    on_gpu = torch.empty((L, E), dtype=torch.uint8, device=calib_counts.device)
    _check(lib().daop_memory_init(L, E, _p(calib_counts, torch.int32, (L, E), "calib_counts"), int(slots), _p(on_gpu),
                                  _stream()), "daop_memory_init")
    return on_gpu


def daop_predict_degraded(shape: moe.MoeShape, x, w_gate_next, gate_bias_next, on_gpu, pred_idx, pred_w=None):
    """Next-layer prediction with graceful degradation; on_gpu is the next layer's uint8 [E] row."""
    T = x.shape[0]
    _check(lib().daop_predict_degraded(ctypes.byref(shape), T, _p(x), _p(w_gate_next), _p(gate_bias_next, torch.float32),
                                       _p(on_gpu, torch.uint8, (shape.n_experts,), "on_gpu"),
                                       _p(pred_idx, torch.int32, (T, shape.top_k), "pred_idx"),
                                       _p(pred_w, torch.float32, (T, shape.top_k), "pred_w"), _stream()),
           "daop_predict_degraded")
