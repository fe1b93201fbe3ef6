"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "moe.h")
MEASURE_HEADER = os.path.join(ROOT, "include", "moe_measure.h")
POLICY_HEADER = os.path.join(ROOT, "include", "daop_policy.h")


@pytest.fixture(scope="module")
def L():
    from paper_2501_10375_amd import build, moe

    if not os.path.exists(moe.LIB_PATH):
        build.build()
    return moe.lib()


def _declared_functions(header=HEADER, prefix="moe_"):
    text = open(header).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(" + prefix + r"[a-z_]+)\s*\(", text)))


def test_header_declares_the_four_entry_points():
    names = _declared_functions()
    for required in ("moe_route", "moe_expert_ffn", "moe_predict_next", "moe_layer", "moe_workspace_bytes"):
        assert required in names


def test_library_exports_every_declared_symbol(L):
    from paper_2501_10375_amd import moe

    layer, measure = _declared_functions(), _declared_functions(MEASURE_HEADER)
    for name in layer + measure:
        assert hasattr(L, name), name
    assert set(moe.EXPORTS) == set(layer) | set(measure)
    # the layer's header declares nothing that allocates, keeps state or times itself
    assert not [n for n in layer if n.startswith(("moe_stage_", "moe_calibrate_", "moe_measure_"))]
    from paper_2501_10375_amd import policy

    declared = _declared_functions(POLICY_HEADER, "daop_")
    assert len(declared) == 5
    for name in declared:
        assert hasattr(L, name), name
    assert set(policy.EXPORTS) == set(declared)


def test_policy_calls_reject_bad_arguments_on_the_host(L):
    from paper_2501_10375_amd import moe, policy

    P = policy.lib()
    fake = ctypes.c_void_p(0x1000)   # aligned, never dereferenced: validation fails first
    assert P.daop_similarity(0, 8, fake, fake, fake, None) == moe.MOE_ERR_SHAPE
    assert P.daop_similarity(4, 65, fake, fake, fake, None) == moe.MOE_ERR_SHAPE
    assert P.daop_similarity(4, 8, None, fake, fake, None) == moe.MOE_ERR_NULL
    assert P.daop_similarity(4, 8, ctypes.c_void_p(0x1004), fake, fake, None) == moe.MOE_ERR_ALIGN
    assert P.daop_window_variation(4, 8, 60, 2, 0, fake, fake, None) == moe.MOE_ERR_SHAPE
    assert P.daop_window_variation(4, 8, 60, 9, 15, fake, fake, None) == moe.MOE_ERR_SHAPE
    assert P.daop_window_variation(4, 8, 60, 2, 15, None, fake, None) == moe.MOE_ERR_NULL
    assert P.daop_window_variation(4, 8, 60, 2, 15, fake, ctypes.c_void_p(0x1008), None) == moe.MOE_ERR_ALIGN
    assert P.daop_plan_swaps(4, 8, fake, fake, -1.0, None, None, None) == moe.MOE_ERR_SHAPE
    assert P.daop_plan_swaps(4, 8, fake, fake, float("nan"), None, None, None) == moe.MOE_ERR_SHAPE
    assert P.daop_plan_swaps(4, 8, fake, None, 1.05, None, None, None) == moe.MOE_ERR_NULL
    assert P.daop_memory_init(2000, 8, fake, 3, fake, None) == moe.MOE_ERR_SHAPE
    assert P.daop_memory_init(4, 8, None, 3, fake, None) == moe.MOE_ERR_NULL
    s = _shape()
    assert P.daop_predict_degraded(ctypes.byref(s), 4, fake, fake, None, None, fake, None, None) == moe.MOE_ERR_NULL
    assert P.daop_predict_degraded(ctypes.byref(s), -1, fake, fake, None, fake, fake, None, None) == moe.MOE_ERR_SHAPE
    assert P.daop_predict_degraded(ctypes.byref(s), 0, None, fake, None, fake, None, None, None) == moe.MOE_OK


def test_status_strings(L):
    for code in range(0, -8, -1):
        s = L.moe_status_string(code)
        assert s and b"unknown" not in s
    assert b"unknown" in L.moe_status_string(-99)


def _shape(**kw):
    from paper_2501_10375_amd import moe

    base = dict(hidden=256, ffn=512, n_experts=8, top_k=2, dtype=moe.MOE_BF16, reserved=0)
    base.update(kw)
    return moe.MoeShape(**base)


def test_workspace_sizes(L):
    n = ctypes.c_size_t(0)
    s = _shape()
    assert L.moe_workspace_bytes(ctypes.byref(s), 64, ctypes.byref(n)) == 0
    full = n.value
    assert L.moe_route_workspace_bytes(ctypes.byref(s), 64, ctypes.byref(n)) == 0
    assert 0 < n.value < full
    # must at least hold act [A,F] bf16 and out [A,H] fp32
    assert full >= 64 * 2 * 512 * 2 + 64 * 2 * 256 * 4
    big = _shape(hidden=4096, ffn=14336)
    assert L.moe_workspace_bytes(ctypes.byref(big), 4096, ctypes.byref(n)) == 0
    assert n.value >= 8192 * 14336 * 2 + 8192 * 4096 * 4
    assert L.moe_workspace_bytes(ctypes.byref(s), 64, None) == -1
    assert L.moe_workspace_bytes(None, 64, ctypes.byref(n)) == -1
    assert L.moe_workspace_bytes(ctypes.byref(s), -1, ctypes.byref(n)) == -2
    assert L.moe_workspace_bytes(ctypes.byref(s), (1 << 20) + 1, ctypes.byref(n)) == -2


@pytest.mark.parametrize("kw,code", [
    (dict(hidden=100), -2), (dict(ffn=0), -2), (dict(ffn=96), -2), (dict(n_experts=65), -2), (dict(n_experts=0), -2),
    (dict(top_k=0), -2), (dict(top_k=9, n_experts=16), -2), (dict(top_k=3, n_experts=2), -2), (dict(dtype=7), -3),
    (dict(reserved=1), -2),
])
def test_bad_shapes_are_rejected(L, kw, code):
    n = ctypes.c_size_t(0)
    s = _shape(**kw)
    assert L.moe_workspace_bytes(ctypes.byref(s), 16, ctypes.byref(n)) == code
    fake = ctypes.c_void_p(0x1000)
    assert L.moe_route(ctypes.byref(s), 4, fake, fake, None, fake, fake, fake, 0, fake, 1 << 30, None) == code


def test_entry_points_validate_before_any_device_work(L):
    # Fake, never dereferenced addresses: every call below must fail in host-side validation.
    s = _shape()
    ok = ctypes.c_void_p(0x10000)
    odd = ctypes.c_void_p(0x10008)
    big = 1 << 40
    sp = ctypes.byref(s)
    assert L.moe_route(sp, 4, None, ok, None, ok, ok, ok, 0, ok, big, None) == -1
    assert L.moe_route(sp, 4, ok, ok, None, ok, ok, None, 0, ok, big, None) == -1
    assert L.moe_route(sp, 4, ok, ok, None, ok, ok, ok, 0, None, big, None) == -1
    assert L.moe_route(sp, 4, odd, ok, None, ok, ok, ok, 0, ok, big, None) == -5
    assert L.moe_route(sp, 4, ok, ok, odd, ok, ok, ok, 0, ok, big, None) == -5
    assert L.moe_route(sp, -1, ok, ok, None, ok, ok, ok, 0, ok, big, None) == -2
    assert L.moe_route(sp, 4, ok, ok, None, ok, ok, ok, 0, ok, 8, None) == -4
    assert L.moe_predict_next(sp, 4, ok, None, None, ok, None, None, ok, big, None) == -1
    assert L.moe_predict_next(sp, 4, ok, ok, None, None, None, None, ok, big, None) == -1
    assert L.moe_predict_next(sp, 4, ok, ok, None, ok, odd, None, ok, big, None) == -5
    assert L.moe_predict_next(sp, 4, ok, ok, None, ok, None, None, ok, 0, None) == -4
    assert L.moe_expert_ffn(sp, 4, ok, ok, ok, ok, None, ok, ok, ok, big, None) == -1
    assert L.moe_expert_ffn(sp, 4, ok, ok, ok, ok, ok, ok, odd, ok, big, None) == -5
    n = ctypes.c_size_t(0)
    L.moe_route_workspace_bytes(sp, 4, ctypes.byref(n))
    assert L.moe_expert_ffn(sp, 4, ok, ok, ok, ok, ok, ok, ok, ok, n.value, None) == -4  # route-only size is not enough
    args = [ok] * 14
    assert L.moe_layer(sp, 4, ok, ok, None, ok, None, ok, ok, ok, ok, ok, ok, ok, 0, None, ok, big, None) == -1
    assert L.moe_layer(sp, 4, ok, ok, None, None, None, ok, ok, None, ok, ok, ok, ok, 0, None, ok, big, None) == -1
    assert L.moe_layer(sp, 4, ok, ok, None, None, None, ok, ok, ok, ok, ok, ok, ok, 0, None, ok, 16, None) == -4
    assert L.moe_layer(None, 4, ok, ok, None, None, None, ok, ok, ok, ok, ok, ok, ok, 0, None, ok, big, None) == -1
    # zero tokens with nothing to clear is accepted without touching the device
    assert L.moe_expert_ffn(sp, 0, ok, ok, ok, ok, ok, ok, ok, ok, big, None) == 0
    assert L.moe_predict_next(sp, 0, ok, ok, None, ok, None, None, ok, big, None) == 0


def test_binding_refuses_cpu_tensors():
    import torch
    from paper_2501_10375_amd import moe

    s = moe.make_shape(256, 512, 8, 2, torch.bfloat16)
    x = torch.zeros((4, 256), dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        moe.moe_route(s, x, x, None, x, x, x, False, x)


def test_binding_raises_when_the_library_is_missing(monkeypatch, tmp_path):
    """No fallback: without the built HIP library the binding refuses to work at all."""
    from paper_2501_10375_amd import moe

    monkeypatch.setattr(moe, "_lib", None)
    monkeypatch.setattr(moe, "LIB_PATH", str(tmp_path / "libmoe_hip.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        moe.lib()


def test_product_code_never_touches_the_oracle():
    """The oracle is test infrastructure: nothing in the package (Python or C++) names it, and only
    the benchmark's CPU-baseline leg and the smoke check import it outside tests/."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = os.path.join(root, "paper_2501_10375_amd")
    for folder, _, files in os.walk(pkg):
        for name in files:
            if name.endswith((".py", ".hip", ".h", ".cpp", ".c")):
                text = open(os.path.join(folder, name), errors="replace").read()
                assert "oracle" not in text.lower(), f"{os.path.join(folder, name)} mentions the oracle"
    # bench.py: one import, inside the block that times the CPU baseline
    lines = open(os.path.join(root, "bench.py")).read().split("\n")
    hits = [i for i, line in enumerate(lines) if re.search(r"^\s*(from|import)\s+oracle\b", line)]
    assert len(hits) == 1 and "no_cpu_baseline" in lines[hits[0] - 1], "bench.py may use the oracle for cpu_baseline only"
    # __graft_entry__.py: build() compiles the checker, smoke() checks against it
    current = ""
    for line in open(os.path.join(root, "__graft_entry__.py")).read().split("\n"):
        if line.startswith("def "):
            current = line
        if re.search(r"^\s*(from|import)\s+oracle\b", line):
            assert current.startswith(("def build", "def smoke")), f"oracle imported inside `{current}`"


def test_calibration_call_validates_on_the_host(L):
    ms, flop = ctypes.c_float(0), ctypes.c_double(0)
    L.moe_calibrate_mfma.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_float),
                                     ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_float), ctypes.c_void_p]
    L.moe_calibrate_mfma.restype = ctypes.c_int
    assert L.moe_calibrate_mfma(1, 8, ctypes.byref(ms), ctypes.byref(flop), None, None) == -2       # too few iterations (MOE_ERR_SHAPE)
    assert L.moe_calibrate_mfma(1, 1 << 23, ctypes.byref(ms), ctypes.byref(flop), None, None) == -2  # too many
    assert L.moe_calibrate_mfma(0, 4096, None, ctypes.byref(flop), None, None) == -2                 # NULL output


def test_read_stream_call_validates_on_the_host(L):
    ms, nbytes = ctypes.c_float(0), ctypes.c_double(0)
    L.moe_calibrate_read_stream.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_float),
                                            ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
    L.moe_calibrate_read_stream.restype = ctypes.c_int
    assert L.moe_calibrate_read_stream(None, 1 << 30, ctypes.byref(ms), ctypes.byref(nbytes), None) == -1      # NULL buffer
    assert L.moe_calibrate_read_stream(ctypes.c_void_p(4096), 1 << 30, None, ctypes.byref(nbytes), None) == -1  # NULL output
    assert L.moe_calibrate_read_stream(ctypes.c_void_p(4100), 1 << 30, ctypes.byref(ms), ctypes.byref(nbytes), None) == -5  # alignment


def test_decode_status_call_validates_on_the_host(L):
    from paper_2501_10375_amd import moe

    out = ctypes.c_int32(7)
    fake = ctypes.c_void_p(0x1000)
    assert L.moe_decode_status(fake, 1 << 20, 0, None, None) == moe.MOE_ERR_NULL
    assert L.moe_decode_status(None, 0, 0, None, None) == moe.MOE_ERR_NULL
    assert L.moe_decode_status(ctypes.c_void_p(0x1004), 1 << 20, 0, ctypes.byref(out), None) == moe.MOE_ERR_ALIGN
    assert L.moe_decode_status(fake, 64, 0, ctypes.byref(out), None) == moe.MOE_ERR_WORKSPACE
    assert out.value == 7
    assert L.moe_measure_set_decode_spin_limit(-1) == moe.MOE_ERR_SHAPE


def test_workspace_keeps_flags_and_counters_at_fixed_offsets(L):
    """The decode kernel's launch count and arrival flags and the GEMMs' counters sit at the start of
    the workspace whatever the call size, so a long call can never put other data over them: the
    smallest workspace (0 tokens) already holds both blocks, and every size's routing part starts
    with them."""
    n0, n = ctypes.c_size_t(0), ctypes.c_size_t(0)
    s = _shape()
    assert L.moe_route_workspace_bytes(ctypes.byref(s), 0, ctypes.byref(n0)) == 0
    assert n0.value >= (2 * 256 + 16) * 4 + 2 * (8 + 8 * 32) * 4
    for T in (1, 16, 17, 1024, 4096):
        assert L.moe_route_workspace_bytes(ctypes.byref(s), T, ctypes.byref(n)) == 0
        assert n.value >= n0.value


def test_static_scratch_entry_point_validates_on_the_host(L):
    """moe_layer_static checks its arguments and the size limit of its static buffer before any device work."""
    from paper_2501_10375_amd import moe

    fake = ctypes.c_void_p(0x1000)
    s = _shape()

    def call(shape, T, x=fake, counts=fake, pred=None, wg_next=None):
        return L.moe_layer_static(ctypes.byref(shape) if shape is not None else None, T, x, fake, None, wg_next, None,
                                  fake, fake, fake, fake, fake, fake, counts, 0, pred, None)

    assert call(None, 4) == moe.MOE_ERR_NULL
    assert call(s, -1) == moe.MOE_ERR_SHAPE
    assert call(s, 4, x=None) == moe.MOE_ERR_NULL
    assert call(s, 4, counts=ctypes.c_void_p(0x1008)) == moe.MOE_ERR_ALIGN
    assert call(s, 4, wg_next=fake) == moe.MOE_ERR_NULL            # prediction asked for, nowhere to put it
    assert call(_shape(dtype=9), 4) == moe.MOE_ERR_DTYPE
    # bf16 calls of more than 32 tokens need 64 MiB of K-split pieces: never inside the static buffer
    assert call(s, 33) == moe.MOE_ERR_TOO_LARGE
    big = _shape(hidden=4096, ffn=14336, dtype=moe.MOE_F32)
    assert call(big, 256) == moe.MOE_ERR_TOO_LARGE
    n = ctypes.c_size_t(0)
    for shape, T in ((_shape(hidden=4096, ffn=14336), 32), (_shape(hidden=4096, ffn=6400, n_experts=16), 32)):
        assert L.moe_workspace_bytes(ctypes.byref(shape), T, ctypes.byref(n)) == 0
        assert n.value <= moe.MOE_STATIC_SCRATCH_BYTES    # decode steps at the shapes of Table III fit
    assert b"static" in L.moe_status_string(moe.MOE_ERR_TOO_LARGE)
