"""Thin ctypes binding of libmoe_hip.so (see include/moe.h for the contract).

Argument marshalling only: every function here takes torch tensors that live on
the GPU, checks dtypes/shapes, passes their device pointers and the current HIP
stream to the C entry point of the same name, and raises on a non-zero status.
No step of the MoE layer is computed in Python or by torch, and there is no CPU
fallback: if the shared library has not been built the import of the library
raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_hip.so")

MOE_F32, MOE_BF16 = 0, 1
MOE_OK, MOE_ERR_NULL, MOE_ERR_SHAPE, MOE_ERR_DTYPE, MOE_ERR_WORKSPACE, MOE_ERR_ALIGN, MOE_ERR_DEVICE = 0, -1, -2, -3, -4, -5, -6
MOE_ERR_TOO_LARGE = -7
MOE_STATIC_SCRATCH_BYTES = 16 << 20
STATUS = {0: "MOE_OK", -1: "MOE_ERR_NULL", -2: "MOE_ERR_SHAPE", -3: "MOE_ERR_DTYPE", -4: "MOE_ERR_WORKSPACE",
          -5: "MOE_ERR_ALIGN", -6: "MOE_ERR_DEVICE", -7: "MOE_ERR_TOO_LARGE"}

EXPORTS = ("moe_status_string", "moe_workspace_bytes", "moe_route_workspace_bytes", "moe_route",
           "moe_predict_next", "moe_expert_ffn", "moe_expert_ffn_precalc", "moe_layer", "moe_layer_static", "moe_decode_status",
           # include/moe_measure.h
           "moe_stage_timing_begin", "moe_stage_timing_end", "moe_calibrate_mfma", "moe_calibrate_read_stream",
           "moe_measure_set_decode_spin_limit")
STAGES = ("route", "permute", "gemm1", "gemm2", "combine", "fused")


class MoeShape(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_int32), ("ffn", ctypes.c_int32), ("n_experts", ctypes.c_int32),
                ("top_k", ctypes.c_int32), ("dtype", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class MoeError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS.get(status, status)} ({lib().moe_status_string(status).decode()})")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2501_10375_amd.build` "
                               "(or __graft_entry__.build()); there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        sp = ctypes.POINTER(MoeShape)
        L.moe_status_string.argtypes = [ctypes.c_int]
        L.moe_status_string.restype = ctypes.c_char_p
        for name in ("moe_workspace_bytes", "moe_route_workspace_bytes"):
            getattr(L, name).argtypes = [sp, i32, ctypes.POINTER(sz)]
            getattr(L, name).restype = ctypes.c_int
        L.moe_route.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, i32, vp, sz, vp]
        L.moe_route.restype = ctypes.c_int
        L.moe_predict_next.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.moe_predict_next.restype = ctypes.c_int
        L.moe_expert_ffn.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.moe_expert_ffn.restype = ctypes.c_int
        L.moe_expert_ffn_precalc.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.moe_expert_ffn_precalc.restype = ctypes.c_int
        L.moe_layer.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
        L.moe_layer.restype = ctypes.c_int
        L.moe_layer_static.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp]
        L.moe_layer_static.restype = ctypes.c_int
        L.moe_decode_status.argtypes = [vp, sz, i32, ctypes.POINTER(i32), vp]
        L.moe_decode_status.restype = ctypes.c_int
        L.moe_measure_set_decode_spin_limit.argtypes = [i32]
        L.moe_measure_set_decode_spin_limit.restype = ctypes.c_int
        L.moe_stage_timing_begin.argtypes = [i32]
        L.moe_stage_timing_begin.restype = ctypes.c_int
        L.moe_stage_timing_end.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32)]
        L.moe_stage_timing_end.restype = ctypes.c_int
        L.moe_calibrate_mfma.argtypes = [i32, i32, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double),
                                         ctypes.POINTER(ctypes.c_float), vp]
        L.moe_calibrate_mfma.restype = ctypes.c_int
        L.moe_calibrate_read_stream.argtypes = [vp, sz, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double), vp]
        L.moe_calibrate_read_stream.restype = ctypes.c_int
        _lib = L
    return _lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return MOE_F32
    if t.dtype == torch.bfloat16:
        return MOE_BF16
    raise TypeError(f"unsupported storage dtype {t.dtype}")


def make_shape(hidden: int, ffn: int, n_experts: int, top_k: int, dtype: torch.dtype) -> MoeShape:
    code = MOE_F32 if dtype == torch.float32 else MOE_BF16 if dtype == torch.bfloat16 else -1
    return MoeShape(hidden, ffn, n_experts, top_k, code, 0)


def _p(t, dtype=None, shape=None, name="tensor"):
    """Device pointer of a contiguous CUDA tensor (None -> NULL), with dtype/shape checks."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous GPU tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int, where: str):
    if status != 0:
        raise MoeError(status, where)


def moe_workspace_bytes(shape: MoeShape, max_tokens: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().moe_workspace_bytes(ctypes.byref(shape), max_tokens, ctypes.byref(out)), "moe_workspace_bytes")
    return out.value


def moe_route_workspace_bytes(shape: MoeShape, max_tokens: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().moe_route_workspace_bytes(ctypes.byref(shape), max_tokens, ctypes.byref(out)),
           "moe_route_workspace_bytes")
    return out.value


def alloc_workspace(shape: MoeShape, max_tokens: int, device="cuda", route_only: bool = False) -> torch.Tensor:
    n = moe_route_workspace_bytes(shape, max_tokens) if route_only else moe_workspace_bytes(shape, max_tokens)
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device)


def moe_route(shape: MoeShape, x, w_gate, gate_bias, topk_idx, topk_w, counts, accumulate: bool, workspace):
    T, E, k, H = x.shape[0], shape.n_experts, shape.top_k, shape.hidden
    dt = x.dtype
    _check(lib().moe_route(ctypes.byref(shape), T, _p(x, None, (T, H), "x"), _p(w_gate, dt, (E, H), "w_gate"),
                           _p(gate_bias, torch.float32, (E,), "gate_bias"),
                           _p(topk_idx, torch.int32, (T, k), "topk_idx"), _p(topk_w, torch.float32, (T, k), "topk_w"),
                           _p(counts, torch.int32, (E,), "counts"), int(bool(accumulate)),
                           _p(workspace, torch.uint8, None, "workspace"), workspace.numel(), _stream()), "moe_route")


def moe_predict_next(shape: MoeShape, x, w_gate_next, gate_bias_next, pred_idx, pred_w, pred_counts, workspace):
    T, E, k, H = x.shape[0], shape.n_experts, shape.top_k, shape.hidden
    dt = x.dtype
    _check(lib().moe_predict_next(ctypes.byref(shape), T, _p(x, None, (T, H), "x"),
                                  _p(w_gate_next, dt, (E, H), "w_gate_next"),
                                  _p(gate_bias_next, torch.float32, (E,), "gate_bias_next"),
                                  _p(pred_idx, torch.int32, (T, k), "pred_idx"),
                                  _p(pred_w, torch.float32, (T, k), "pred_w"),
                                  _p(pred_counts, torch.int32, (E,), "pred_counts"),
                                  _p(workspace, torch.uint8, None, "workspace"), workspace.numel(), _stream()),
           "moe_predict_next")


def moe_expert_ffn(shape: MoeShape, x, topk_idx, topk_w, w1, w3, w2, y, workspace):
    T, E, k, H, F = x.shape[0], shape.n_experts, shape.top_k, shape.hidden, shape.ffn
    dt = x.dtype
    _check(lib().moe_expert_ffn(ctypes.byref(shape), T, _p(x, None, (T, H), "x"),
                                _p(topk_idx, torch.int32, (T, k), "topk_idx"),
                                _p(topk_w, torch.float32, (T, k), "topk_w"), _p(w1, dt, (E, F, H), "w1"),
                                _p(w3, dt, (E, F, H), "w3"), _p(w2, dt, (E, H, F), "w2"), _p(y, dt, (T, H), "y"),
                                _p(workspace, torch.uint8, None, "workspace"), workspace.numel(), _stream()),
           "moe_expert_ffn")


def moe_expert_ffn_precalc(shape: MoeShape, x, x_stale, stale, topk_idx, topk_w, w1, w3, w2, y, workspace):
    """moe_expert_ffn where selection (t, j) is evaluated on x_stale[t] if stale[t, j] (uint8) is non-zero."""
    T, E, k, H, F = x.shape[0], shape.n_experts, shape.top_k, shape.hidden, shape.ffn
    dt = x.dtype
    _check(lib().moe_expert_ffn_precalc(ctypes.byref(shape), T, _p(x, None, (T, H), "x"), _p(x_stale, dt, (T, H), "x_stale"),
                                        _p(stale, torch.uint8, (T, k), "stale"),
                                        _p(topk_idx, torch.int32, (T, k), "topk_idx"),
                                        _p(topk_w, torch.float32, (T, k), "topk_w"), _p(w1, dt, (E, F, H), "w1"),
                                        _p(w3, dt, (E, F, H), "w3"), _p(w2, dt, (E, H, F), "w2"), _p(y, dt, (T, H), "y"),
                                        _p(workspace, torch.uint8, None, "workspace"), workspace.numel(), _stream()),
           "moe_expert_ffn_precalc")


def moe_layer(shape: MoeShape, x, w_gate, gate_bias, w_gate_next, gate_bias_next, w1, w3, w2, y, topk_idx, topk_w,
              counts, accumulate: bool, pred_idx, workspace):
    T, E, k, H, F = x.shape[0], shape.n_experts, shape.top_k, shape.hidden, shape.ffn
    dt = x.dtype
    _check(lib().moe_layer(ctypes.byref(shape), T, _p(x, None, (T, H), "x"), _p(w_gate, dt, (E, H), "w_gate"),
                           _p(gate_bias, torch.float32, (E,), "gate_bias"),
                           _p(w_gate_next, dt, (E, H), "w_gate_next"),
                           _p(gate_bias_next, torch.float32, (E,), "gate_bias_next"), _p(w1, dt, (E, F, H), "w1"),
                           _p(w3, dt, (E, F, H), "w3"), _p(w2, dt, (E, H, F), "w2"), _p(y, dt, (T, H), "y"),
                           _p(topk_idx, torch.int32, (T, k), "topk_idx"), _p(topk_w, torch.float32, (T, k), "topk_w"),
                           _p(counts, torch.int32, (E,), "counts"), int(bool(accumulate)),
                           _p(pred_idx, torch.int32, (T, k), "pred_idx"),
                           _p(workspace, torch.uint8, None, "workspace"), workspace.numel(), _stream()), "moe_layer")


def moe_layer_static(shape: MoeShape, x, w_gate, gate_bias, w_gate_next, gate_bias_next, w1, w3, w2, y, topk_idx, topk_w,
                     counts, accumulate: bool, pred_idx):
    """moe_layer on the library's static scratch buffer (no workspace argument, nothing allocated)."""
    T, E, k, H, F = x.shape[0], shape.n_experts, shape.top_k, shape.hidden, shape.ffn
    dt = x.dtype
    _check(lib().moe_layer_static(ctypes.byref(shape), T, _p(x, None, (T, H), "x"), _p(w_gate, dt, (E, H), "w_gate"),
                                  _p(gate_bias, torch.float32, (E,), "gate_bias"),
                                  _p(w_gate_next, dt, (E, H), "w_gate_next"),
                                  _p(gate_bias_next, torch.float32, (E,), "gate_bias_next"),
                                  _p(w1, dt, (E, F, H), "w1"), _p(w3, dt, (E, F, H), "w3"), _p(w2, dt, (E, H, F), "w2"),
                                  _p(y, dt, (T, H), "y"), _p(topk_idx, torch.int32, (T, k), "topk_idx"),
                                  _p(topk_w, torch.float32, (T, k), "topk_w"), _p(counts, torch.int32, (E,), "counts"),
                                  int(bool(accumulate)), _p(pred_idx, torch.int32, (T, k), "pred_idx"), _stream()),
           "moe_layer_static")


def moe_decode_status(workspace: torch.Tensor | None, reset: bool = False) -> bool:
    """True if a decode-size call on this workspace (None: the static scratch of moe_layer_static) gave
    up a rendezvous since the last reset (synchronises)."""
    out = ctypes.c_int32(0)
    _check(lib().moe_decode_status(_p(workspace, torch.uint8, None, "workspace"),
                                   0 if workspace is None else workspace.numel(), int(bool(reset)),
                                   ctypes.byref(out), _stream()), "moe_decode_status")
    return bool(out.value)


def moe_measure_set_decode_spin_limit(polling_rounds: int):
    _check(lib().moe_measure_set_decode_spin_limit(int(polling_rounds)), "moe_measure_set_decode_spin_limit")


class PreparedLayerCall:
    """A moe_layer call whose arguments were checked and marshalled once, for loops that repeat it on
    the same buffers (a decode step of about 100 microseconds leaves no room for per-call argument
    checks in Python).  Calling the object enqueues the call on the current stream."""

    def __init__(self, shape: MoeShape, d: dict, out: "LayerOutputs", accumulate: bool = False, predict: bool = True):
        x = d["x"]
        T, E, k, H, F = x.shape[0], shape.n_experts, shape.top_k, shape.hidden, shape.ffn
        dt = x.dtype
        pred = out.pred_idx[:T] if (predict and d.get("wg_next") is not None) else None
        y, idx, w = out.y[:T], out.topk_idx[:T], out.topk_w[:T]
        self._keep = (shape, d, out, y, idx, w, pred)   # the tensors behind the raw pointers
        self._fn = lib().moe_layer
        self._args = (ctypes.byref(shape), T, _p(x, None, (T, H), "x"), _p(d["wg"], dt, (E, H), "w_gate"),
                      _p(d.get("bias"), torch.float32, (E,), "gate_bias"),
                      _p(d.get("wg_next") if pred is not None else None, dt, (E, H), "w_gate_next"),
                      _p(d.get("bias_next") if pred is not None else None, torch.float32, (E,), "gate_bias_next"),
                      _p(d["w1"], dt, (E, F, H), "w1"), _p(d["w3"], dt, (E, F, H), "w3"), _p(d["w2"], dt, (E, H, F), "w2"),
                      _p(y, dt, (T, H), "y"), _p(idx, torch.int32, (T, k), "topk_idx"),
                      _p(w, torch.float32, (T, k), "topk_w"), _p(out.counts, torch.int32, (E,), "counts"),
                      int(bool(accumulate)), _p(pred, torch.int32, (T, k), "pred_idx"),
                      _p(out.workspace, torch.uint8, None, "workspace"), out.workspace.numel())
        self.result = {"y": y, "idx": idx, "w": w, "counts": out.counts, "pred_idx": pred}

    def __call__(self):
        status = self._fn(*self._args, _stream())
        if status != 0:
            raise MoeError(status, "moe_layer")
        return self.result


def moe_stage_timing_begin(max_calls: int):
    _check(lib().moe_stage_timing_begin(max_calls), "moe_stage_timing_begin")


def moe_stage_timing_end() -> dict:
    """{stage name: (mean ms per launch, launches)} for the calls since moe_stage_timing_begin."""
    ms = (ctypes.c_float * len(STAGES))()
    n = (ctypes.c_int32 * len(STAGES))()
    _check(lib().moe_stage_timing_end(ms, n), "moe_stage_timing_end")
    return {name: (float(ms[i]), int(n[i])) for i, name in enumerate(STAGES)}


def moe_calibrate_mfma(random_operands: bool, iterations: int = 20000, stream=None) -> dict:
    """Register-only bf16 MFMA loop on every CU; returns {"ms", "flop", "tflops", "ghz"} of the timed launch."""
    ms, flop, ghz = ctypes.c_float(0.0), ctypes.c_double(0.0), ctypes.c_float(0.0)
    s = torch.cuda.current_stream() if stream is None else stream
    _check(lib().moe_calibrate_mfma(int(bool(random_operands)), int(iterations), ctypes.byref(ms), ctypes.byref(flop),
                                    ctypes.byref(ghz), ctypes.c_void_p(s.cuda_stream)), "moe_calibrate_mfma")
    return {"ms": float(ms.value), "flop": float(flop.value), "tflops": float(flop.value) / (ms.value * 1e-3) / 1e12,
            "ghz": float(ghz.value)}


def moe_calibrate_read_stream(buffer: torch.Tensor, stream=None) -> dict:
    """Plain read stream over a device tensor; returns {"ms", "bytes", "GBps"} of the timed launch."""
    assert buffer.is_cuda and buffer.is_contiguous()
    ms, nbytes = ctypes.c_float(0.0), ctypes.c_double(0.0)
    s = torch.cuda.current_stream() if stream is None else stream
    _check(lib().moe_calibrate_read_stream(ctypes.c_void_p(buffer.data_ptr()), buffer.numel() * buffer.element_size(),
                                           ctypes.byref(ms), ctypes.byref(nbytes), ctypes.c_void_p(s.cuda_stream)),
           "moe_calibrate_read_stream")
    return {"ms": float(ms.value), "bytes": float(nbytes.value), "GBps": float(nbytes.value) / (ms.value * 1e-3) / 1e9}


class LayerOutputs:
    """Output buffers of one moe_layer call, allocated once and reused."""

    def __init__(self, shape: MoeShape, max_tokens: int, dtype: torch.dtype, device="cuda", predict: bool = True):
        k, E, H = shape.top_k, shape.n_experts, shape.hidden
        self.y = torch.empty((max_tokens, H), dtype=dtype, device=device)
        self.topk_idx = torch.empty((max_tokens, k), dtype=torch.int32, device=device)
        self.topk_w = torch.empty((max_tokens, k), dtype=torch.float32, device=device)
        self.counts = torch.zeros((E,), dtype=torch.int32, device=device)
        self.pred_idx = torch.empty((max_tokens, k), dtype=torch.int32, device=device) if predict else None
        self.workspace = alloc_workspace(shape, max_tokens, device)


def run_layer(shape: MoeShape, d: dict, out: LayerOutputs, accumulate: bool = False, predict: bool = True):
    """moe_layer on a dict of tensors as made by synth.moe_layer_inputs; returns views sized to the call."""
    T = d["x"].shape[0]
    pred = out.pred_idx[:T] if (predict and d.get("wg_next") is not None) else None
    moe_layer(shape, d["x"], d["wg"], d.get("bias"), d.get("wg_next") if pred is not None else None,
              d.get("bias_next") if pred is not None else None, d["w1"], d["w3"], d["w2"], out.y[:T],
              out.topk_idx[:T], out.topk_w[:T], out.counts, accumulate, pred, out.workspace)
    return {"y": out.y[:T], "idx": out.topk_idx[:T], "w": out.topk_w[:T], "counts": out.counts, "pred_idx": pred}
