"""Parity of the HIP library (through its C ABI) with the CPU oracle, element by element,
at sizes the oracle finishes in seconds: several tiles, ragged tails, degenerate cases."""
import numpy as np
import pytest
import torch

from paper_2501_10375_amd import moe, synth
from parity_util import check_layer, check_routing, host, output_error, to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _run(T, H, F, E, k, dtype, seed=0, zipf=1.2, predict=True):
    d = synth.moe_layer_inputs(T, H, F, E, dtype, DEV, seed=seed, zipf_s=zipf, with_next=predict)
    shape = moe.make_shape(H, F, E, k, dtype)
    out = moe.LayerOutputs(shape, max(T, 1), dtype, DEV, predict=predict)
    res = moe.run_layer(shape, d, out, predict=predict)
    return d, shape, out, res


def test_config0_tiny_fp32_layer(oracle):
    d, shape, out, res = _run(64, 256, 512, 8, 2, torch.float32)
    r = check_layer(oracle, d, shape, res, torch.float32, label="config0")
    print("config0", r)
    assert r["compared_tokens"] >= 60


@pytest.mark.parametrize("T,H,F,E,k", [
    (300, 256, 512, 8, 2),     # several 128-slot tiles per expert, ragged tails
    (129, 128, 192, 4, 2),     # F not a multiple of the 128 feature tile
    (77, 64, 64, 16, 2),       # smallest legal widths, many cold experts
    (200, 256, 256, 8, 1),     # top-1
    (50, 128, 256, 8, 4),      # top-4
    (40, 128, 128, 64, 8),     # widest router, top-8
    (17, 256, 512, 8, 2),      # just above the decode threshold
    (90, 192, 128, 32, 3),     # two 16-expert blocks in the router
    (40, 8192, 128, 8, 2),     # hidden dimension longer than one register chunk of the router
    (60, 128, 128, 12, 3),     # expert count that is not a power of two
    (32, 256, 512, 8, 2), (33, 256, 320, 16, 2), (64, 256, 512, 8, 2), (65, 256, 512, 8, 2),   # weight-streaming sizes and the first size past them
])
def test_bf16_prefill_path(oracle, T, H, F, E, k):
    d, shape, out, res = _run(T, H, F, E, k, torch.bfloat16)
    r = check_layer(oracle, d, shape, res, torch.bfloat16, label=f"bf16 T={T}")
    print(r)


@pytest.mark.parametrize("T,H,F,E,k", [
    (1100, 256, 512, 2, 2),    # ~9 slot tiles of 256, everything in one round whose tiles are split along K
    (700, 512, 384, 1, 1),     # one expert, top-1: a dense SwiGLU MLP; F = 3 feature tiles of gemm1
    (1300, 320, 448, 2, 2),    # F ends in a half feature tile, K = 5 steps of 64 (odd number of ring turns)
    (2100, 1024, 320, 4, 2),   # 16 K steps: the weight ring wraps 5 times; ragged last slot tiles
    (3000, 256, 2048, 2, 2),   # more tiles than compute units: one full round, then a split round
])
def test_bf16_full_tile_flavour_every_token(oracle, T, H, F, E, k):
    """Calls with at least 512 routed rows per expert run both GEMMs in the full-tile flavour (256-slot
    tiles, three weight stages and two slot stages), the one long prefill calls run.  Narrow layers let
    the oracle check every token, so every wavefront's fragment rows and every epilogue position of
    the 256 x 256 tile is compared, including tiles whose K range is split between workgroups."""
    assert T * k >= E * 512
    d, shape, out, res = _run(T, H, F, E, k, torch.bfloat16)
    r = check_layer(oracle, d, shape, res, torch.bfloat16, label=f"bf16 full tiles T={T}")
    print(r)
    assert r["compared_tokens"] >= T - r["excluded"] - 2


@pytest.mark.parametrize("T,H,F,E,k,seed", [
    (200, 256, 256, 2, 2, 0),    # 200 rows per expert: gemm1 in the full-tile flavour, gemm2 in the ragged one
    (150, 256, 384, 4, 4, 1),    # hot expert: a full slot tile and a short one; cold experts: one or two fragments
    (330, 320, 448, 2, 2, 2),    # both GEMMs full-tile, second slot tile of every expert ragged
    (140, 128, 640, 1, 1, 3),    # one expert with 140 rows: 5 valid fragments, 3 and 2 per wavefront group
    (520, 192, 256, 8, 2, 4),    # 130 rows per expert on average: cold experts far below one fragment per group
    (300, 256, 512, 2, 1, 5),    # top-1, about 150 rows per expert
])
def test_bf16_ragged_fragments_of_full_tiles_every_token(oracle, T, H, F, E, k, seed):
    """From 128 routed rows per expert on gemm1 runs in the full-tile flavour, whose ragged slot tiles
    issue only the MFMAs of their valid 32-slot fragments (a main loop per fragment count, chosen per
    wavefront), while gemm2 stays in the ragged flavour below 320 rows per expert.  Every token is
    compared, so every fragment count a wavefront can have (1 to 4) is exercised over these shapes."""
    assert E * 128 <= T * k
    d, shape, out, res = _run(T, H, F, E, k, torch.bfloat16, seed=seed)
    counts = res["counts"].cpu().tolist()
    r = check_layer(oracle, d, shape, res, torch.bfloat16, label=f"bf16 T={T} ragged fragments")
    print(r, "rows per expert:", counts)
    assert r["compared_tokens"] >= T - r["excluded"] - 2


@pytest.mark.parametrize("T,H,F,E,k", [
    (1, 256, 512, 8, 2), (5, 256, 512, 8, 2), (16, 256, 512, 8, 2), (8, 512, 1600, 16, 2), (3, 64, 64, 4, 1),
    (16, 128, 320, 8, 8), (7, 2048, 1024, 8, 2), (4, 128, 128, 64, 8), (9, 192, 256, 32, 2), (6, 8192, 128, 8, 2),
    (5, 128, 128, 6, 2),
])
def test_bf16_decode_path(oracle, T, H, F, E, k):
    d, shape, out, res = _run(T, H, F, E, k, torch.bfloat16)
    r = check_layer(oracle, d, shape, res, torch.bfloat16, label=f"decode T={T}")
    print(r)


def _random_shapes(n, seed):
    """Seeded sweep over legal shapes: token counts on both sides of every path boundary (16, 32,
    256), widths that do not divide the tile sizes, few and many experts, every top_k."""
    rng = np.random.default_rng(seed)
    shapes = []
    for i in range(n):
        T = int(rng.choice([1, 2, 3, 7, 15, 16, 17, 24, 31, 32, 33, 48, 63, 64, 80, 127, 200, 255, 256, 257, 300]))
        H = 64 * int(rng.integers(1, 9))
        F = 64 * int(rng.integers(1, 25))
        E = int(rng.choice([1, 2, 3, 4, 5, 8, 11, 16, 24, 32, 64]))
        k = int(rng.integers(1, min(E, 8) + 1))
        shapes.append((T, H, F, E, k, i))
    return shapes


@pytest.mark.parametrize("T,H,F,E,k,seed", _random_shapes(36, 20250110))
def test_bf16_random_shapes(oracle, T, H, F, E, k, seed):
    d, shape, out, res = _run(T, H, F, E, k, torch.bfloat16, seed=seed, zipf=1.2 if seed % 3 else None)
    r = check_layer(oracle, d, shape, res, torch.bfloat16, label=f"bf16 random T={T} H={H} F={F} E={E} k={k}")
    print(r)


@pytest.mark.parametrize("T,H,F,E,k", [(100, 128, 192, 8, 2), (5, 64, 128, 4, 2), (130, 256, 64, 16, 3)])
def test_fp32_path(oracle, T, H, F, E, k):
    d, shape, out, res = _run(T, H, F, E, k, torch.float32)
    r = check_layer(oracle, d, shape, res, torch.float32, label=f"fp32 T={T}")
    print(r)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("T", [9, 30, 64, 150])
def test_layer_equals_route_predict_ffn_bitwise(dtype, T):
    H, F, E, k = 256, 512, 8, 2
    d, shape, out, res = _run(T, H, F, E, k, dtype)
    idx = torch.empty((T, k), dtype=torch.int32, device=DEV)
    w = torch.empty((T, k), dtype=torch.float32, device=DEV)
    counts = torch.full((E,), -7, dtype=torch.int32, device=DEV)
    pidx = torch.empty((T, k), dtype=torch.int32, device=DEV)
    pw = torch.empty((T, k), dtype=torch.float32, device=DEV)
    pcounts = torch.full((E,), -7, dtype=torch.int32, device=DEV)
    y = torch.empty((T, H), dtype=dtype, device=DEV)
    ws = moe.alloc_workspace(shape, T)
    moe.moe_route(shape, d["x"], d["wg"], d["bias"], idx, w, counts, False, ws)
    moe.moe_predict_next(shape, d["x"], d["wg_next"], d["bias_next"], pidx, pw, pcounts, ws)
    moe.moe_expert_ffn(shape, d["x"], idx, w, d["w1"], d["w3"], d["w2"], y, ws)
    torch.cuda.synchronize()
    assert torch.equal(idx, res["idx"]) and torch.equal(w, res["w"]) and torch.equal(counts, res["counts"])
    assert torch.equal(pidx, res["pred_idx"])
    assert torch.equal(y.view(torch.uint8), res["y"].view(torch.uint8))
    assert pcounts.sum().item() == T * k
    assert torch.equal(pcounts, torch.bincount(pidx.flatten().long(), minlength=E).int())
    assert torch.all((pw.sum(1) - 1).abs() < 1e-5)


@pytest.mark.parametrize("T", [8, 48, 260])
def test_repeatable_and_independent_of_workspace_contents(T):
    H, F, E, k, dtype = 256, 512, 8, 2, torch.bfloat16
    d, shape, out, res = _run(T, H, F, E, k, dtype)
    y0, i0, c0 = res["y"].clone(), res["idx"].clone(), res["counts"].clone()
    for fill in (0xFF, 0x7F, 0x00):
        out.workspace.fill_(fill)   # 0xFF.. is NaN in bf16 and fp32 and -1 as an index
        out.y.fill_(0)
        res = moe.run_layer(shape, d, out)
        torch.cuda.synchronize()
        assert torch.equal(res["y"].view(torch.int16), y0.view(torch.int16))
        assert torch.equal(res["idx"], i0) and torch.equal(res["counts"], c0)


@pytest.mark.parametrize("T,H,F,E,k", [(1, 256, 512, 8, 2), (6, 256, 512, 8, 2), (16, 128, 320, 8, 8), (3, 64, 64, 4, 1),
                                       (24, 256, 512, 8, 2), (300, 256, 512, 8, 2), (600, 1024, 2048, 8, 2)])
def test_sequence_of_calls_on_one_workspace_small_shapes(T, H, F, E, k):
    """Calls with changing inputs share one workspace at sizes where everything stays in the caches
    between launches: what an earlier call left there (intermediate values, K-split pieces,
    rendezvous flags and counters) must never be what a later call reads.  Every call is compared
    bit for bit with the same call on a fresh workspace filled with a byte pattern."""
    dtype = torch.bfloat16
    d = synth.moe_layer_inputs(T, H, F, E, dtype, DEV, seed=3, zipf_s=1.2, with_next=True)
    shape = moe.make_shape(H, F, E, k, dtype)
    shared = moe.LayerOutputs(shape, T, dtype, DEV, predict=True)
    for step in range(8):
        call = dict(d, x=synth.normal((T, H), 3000 + step, synth.TID_X, 1.0, dtype, DEV))
        got = moe.run_layer(shape, call, shared, predict=True)
        y, idx, pred = got["y"].clone(), got["idx"].clone(), got["pred_idx"].clone()
        fresh = moe.LayerOutputs(shape, T, dtype, DEV, predict=True)
        fresh.workspace.fill_(0x5A)
        ref = moe.run_layer(shape, call, fresh, predict=True)
        torch.cuda.synchronize()
        assert torch.equal(idx, ref["idx"]) and torch.equal(pred, ref["pred_idx"]), f"step {step}"
        assert torch.equal(y.view(torch.int16), ref["y"].view(torch.int16)), f"step {step}"


def test_alternating_long_and_decode_calls_on_one_workspace():
    """A serving loop alternates prefill-size and single-token calls on one workspace.  The decode
    kernel derives its rendezvous epoch from a launch count it keeps in the workspace, and flags left
    by its previous launch carry the previous epoch; a long call in between must leave both alone
    (they sit at fixed offsets ahead of everything whose size depends on the call).  Every call is
    compared bit for bit with the same call on a fresh workspace filled with a byte pattern."""
    H, F, E, k, dtype = 256, 512, 8, 2, torch.bfloat16
    d = synth.moe_layer_inputs(1024, H, F, E, dtype, DEV, seed=11, zipf_s=1.2, with_next=True)
    shape = moe.make_shape(H, F, E, k, dtype)
    shared = moe.LayerOutputs(shape, 1024, dtype, DEV, predict=True)
    shared.workspace.zero_()
    for step, T in enumerate([1, 1024, 1, 1, 1024, 300, 1, 24, 1, 1024, 1]):
        call = dict(d, x=synth.normal((T, H), 4000 + step, synth.TID_X, 1.0, dtype, DEV))
        got = moe.run_layer(shape, call, shared, predict=True)
        y, idx = got["y"].clone(), got["idx"].clone()
        fresh = moe.LayerOutputs(shape, T, dtype, DEV, predict=True)
        fresh.workspace.fill_(0x5A)
        ref = moe.run_layer(shape, call, fresh, predict=True)
        torch.cuda.synchronize()
        assert torch.equal(idx, ref["idx"]), f"step {step} T={T}"
        assert torch.equal(y.view(torch.int16), ref["y"].view(torch.int16)), f"step {step} T={T}"
    assert not moe.moe_decode_status(shared.workspace)


def test_decode_rendezvous_reports_when_it_gives_up(oracle):
    """The decode-size kernel's workgroups wait for one another with a bounded spin.  Normally nobody
    gives up and the status word stays clear.  With the spin bound lowered to zero from the host every
    rendezvous gives up at once (all kernels still run to their end): the call then reports it through
    moe_decode_status and marks its output with NaN instead of returning numbers computed from an
    intermediate that may not have been written yet."""
    T, H, F, E, k, dtype = 4, 256, 512, 8, 2, torch.bfloat16
    d, shape, out, res = _run(T, H, F, E, k, dtype)
    torch.cuda.synchronize()
    good = res["y"].clone()
    assert not moe.moe_decode_status(out.workspace, reset=True)
    try:
        moe.moe_measure_set_decode_spin_limit(0)
        res = moe.run_layer(shape, d, out)
        torch.cuda.synchronize()
        assert torch.isnan(res["y"].float()).all()
        assert moe.moe_decode_status(out.workspace)            # reported ...
        assert moe.moe_decode_status(out.workspace, reset=True)  # ... and sticky until reset
        assert not moe.moe_decode_status(out.workspace)
    finally:
        moe.moe_measure_set_decode_spin_limit(1 << 22)
    res = moe.run_layer(shape, d, out)
    torch.cuda.synchronize()
    assert torch.equal(res["y"].view(torch.int16), good.view(torch.int16))
    assert not moe.moe_decode_status(out.workspace)
    r = check_layer(oracle, d, shape, res, dtype, label="after a reported give-up")
    print(r)


@pytest.mark.parametrize("T,H,F,E,k,dtype", [
    (1, 256, 512, 8, 2, torch.bfloat16), (8, 512, 1024, 8, 2, torch.bfloat16), (16, 128, 320, 8, 8, torch.bfloat16),
    (24, 256, 512, 8, 2, torch.bfloat16),      # two column groups of the streaming kernel
    (6, 8192, 128, 8, 2, torch.bfloat16),      # hidden size past the register-resident token operand
    (300, 256, 512, 8, 2, torch.bfloat16),     # ragged 128-slot tiles
    (1100, 256, 512, 2, 2, torch.bfloat16),    # full 256-slot tiles, split-K round
    (64, 256, 512, 8, 2, torch.float32), (5, 64, 128, 4, 2, torch.float32),
])
def test_expert_ffn_with_precalculated_selections(oracle, T, H, F, E, k, dtype):
    """Sec. IV-C pre-calculation as one library call: selections flagged stale are evaluated on an
    earlier hidden state, the rest on the true input, in one pass over the weights.  Compared with the
    oracle's definition at the layer's own tolerance; an all-zero mask must equal moe_expert_ffn."""
    d = synth.moe_layer_inputs(T, H, F, E, dtype, DEV, seed=31, zipf_s=1.2, with_next=False)
    x_stale = synth.normal((T, H), 4242, synth.TID_X, 1.0, dtype, DEV)
    shape = moe.make_shape(H, F, E, k, dtype)
    ws = moe.alloc_workspace(shape, T)
    idx = torch.empty((T, k), dtype=torch.int32, device=DEV)
    w = torch.empty((T, k), dtype=torch.float32, device=DEV)
    counts = torch.zeros((E,), dtype=torch.int32, device=DEV)
    moe.moe_route(shape, d["x"], d["wg"], d["bias"], idx, w, counts, False, ws)
    g = torch.Generator(device="cpu").manual_seed(T * 7 + H)
    stale = (torch.rand((T, k), generator=g) < 0.4).to(torch.uint8)
    stale[0, 0] = 1
    if k > 1:
        stale[0, 1] = 0
    stale = stale.to(DEV)
    y = torch.empty((T, H), dtype=dtype, device=DEV)
    moe.moe_expert_ffn_precalc(shape, d["x"], x_stale, stale, idx, w, d["w1"], d["w3"], d["w2"], y, ws)
    torch.cuda.synchronize()
    h = host(dict(d, x_stale=x_stale))
    ref = oracle.expert_ffn_precalc(h["x"], h["x_stale"], stale.cpu().numpy(), idx.cpu().numpy(),
                                    w.cpu().numpy().astype(np.float64), h["w1"], h["w3"], h["w2"])
    err = output_error(to_f64(y), ref)
    print("precalc", T, H, F, E, k, dtype, "err", err)
    assert err <= {torch.bfloat16: 2e-2, torch.float32: 1e-4}[dtype]
    # the mask matters: the plain call differs where a selection is stale
    y_plain = torch.empty_like(y)
    moe.moe_expert_ffn(shape, d["x"], idx, w, d["w1"], d["w3"], d["w2"], y_plain, ws)
    y_zero = torch.empty_like(y)
    moe.moe_expert_ffn_precalc(shape, d["x"], x_stale, torch.zeros_like(stale), idx, w, d["w1"], d["w3"], d["w2"], y_zero, ws)
    torch.cuda.synchronize()
    assert torch.equal(y_zero.view(torch.uint8), y_plain.view(torch.uint8))
    assert not torch.equal(y[0], y_plain[0])


def test_prepared_call_equals_run_layer():
    """The binding's pre-marshalled call object enqueues the same call as run_layer."""
    T, H, F, E, k, dtype = 6, 256, 512, 8, 2, torch.bfloat16
    d, shape, out, res = _run(T, H, F, E, k, dtype)
    y, idx, pred, counts = res["y"].clone(), res["idx"].clone(), res["pred_idx"].clone(), res["counts"].clone()
    out2 = moe.LayerOutputs(shape, T, dtype, DEV, predict=True)
    call = moe.PreparedLayerCall(shape, d, out2, predict=True)
    for _ in range(3):
        got = call()
    torch.cuda.synchronize()
    assert torch.equal(got["idx"], idx) and torch.equal(got["pred_idx"], pred) and torch.equal(got["counts"], counts)
    assert torch.equal(got["y"].view(torch.int16), y.view(torch.int16))


def test_counts_accumulate_over_calls_and_zero_tokens(oracle):
    H, F, E, k, dtype = 256, 512, 8, 2, torch.bfloat16
    d, shape, out, res = _run(40, H, F, E, k, dtype)
    c1 = res["counts"].clone()
    moe.run_layer(shape, d, out, accumulate=True)
    torch.cuda.synchronize()
    assert torch.equal(out.counts, 2 * c1)
    # decode-size call adds its own tokens
    d1 = dict(d)
    d1["x"] = d["x"][:3].contiguous()
    moe.run_layer(shape, d1, out, accumulate=True)
    torch.cuda.synchronize()
    assert out.counts.sum().item() == (40 * 2 + 3) * k
    # 17 to 32 tokens: the weight-streaming kernel counts the selections of the routing kernel before it
    d2 = dict(d)
    d2["x"] = d["x"][:20].contiguous()
    before = out.counts.clone()
    r2 = moe.run_layer(shape, d2, out, accumulate=True)
    torch.cuda.synchronize()
    hist = torch.bincount(r2["idx"].flatten().long(), minlength=E).to(torch.int32)
    assert torch.equal(out.counts, before + hist)
    moe.run_layer(shape, d2, out, accumulate=False)
    torch.cuda.synchronize()
    assert torch.equal(out.counts, hist)
    moe.run_layer(shape, d, out, accumulate=False)
    moe.run_layer(shape, d, out, accumulate=True)
    moe.run_layer(shape, d1, out, accumulate=True)
    torch.cuda.synchronize()
    # zero tokens: counts untouched with accumulate, cleared without
    d0 = dict(d)
    d0["x"] = d["x"][:0]
    before = out.counts.clone()
    moe.run_layer(shape, d0, out, accumulate=True)
    torch.cuda.synchronize()
    assert torch.equal(out.counts, before)
    moe.run_layer(shape, d0, out, accumulate=False)
    torch.cuda.synchronize()
    assert out.counts.sum().item() == 0
    ws = moe.alloc_workspace(shape, 1, route_only=True)
    cnt = torch.full((E,), 5, dtype=torch.int32, device=DEV)
    moe.moe_route(shape, d0["x"], d["wg"], None, out.topk_idx[:0], out.topk_w[:0], cnt, False, ws)
    torch.cuda.synchronize()
    assert cnt.sum().item() == 0


def test_all_tokens_to_one_expert_equals_its_dense_ffn(oracle):
    # the degenerate grouping: one expert owns every slot (k = 1, +50 bias), both paths
    H, F, E, dtype = 256, 512, 8, torch.bfloat16
    for T in (12, 16, 17, 32, 33, 64, 65, 300):
        d = synth.moe_layer_inputs(T, H, F, E, dtype, DEV, zipf_s=None, with_next=False)
        d["bias"] = torch.zeros(E, dtype=torch.float32, device=DEV)
        d["bias"][5] = 50.0
        shape = moe.make_shape(H, F, E, 1, dtype)
        out = moe.LayerOutputs(shape, T, dtype, DEV, predict=False)
        res = moe.run_layer(shape, d, out, predict=False)
        torch.cuda.synchronize()
        assert torch.all(res["idx"] == 5) and res["counts"][5].item() == T
        assert torch.all(res["w"] == 1.0)
        x64 = to_f64(d["x"])
        w1, w3, w2 = to_f64(d["w1"][5]), to_f64(d["w3"][5]), to_f64(d["w2"][5])
        g = x64 @ w1.T
        dense = ((g / (1 + np.exp(-g))) * (x64 @ w3.T)) @ w2.T
        assert output_error(to_f64(res["y"]), dense) <= 2e-2


def test_routing_entry_points_alone(oracle):
    T, H, E, k = 1000, 512, 16, 2
    for dtype in (torch.float32, torch.bfloat16):
        d = synth.moe_layer_inputs(T, H, 64, E, dtype, DEV, zipf_s=1.5)
        shape = moe.make_shape(H, 64, E, k, dtype)
        ws = moe.alloc_workspace(shape, T, route_only=True)
        idx = torch.empty((T, k), dtype=torch.int32, device=DEV)
        w = torch.empty((T, k), dtype=torch.float32, device=DEV)
        counts = torch.zeros((E,), dtype=torch.int32, device=DEV)
        moe.moe_route(shape, d["x"], d["wg"], d["bias"], idx, w, counts, False, ws)
        torch.cuda.synchronize()
        h = host(d)
        ref = oracle.route(h["x"], h["wg"], h["bias"], k)
        n_excl, _ = check_routing(idx, w, counts, ref, E, "moe_route")
        assert n_excl < 0.02 * T
        # same gate as "next" gate: the prediction equals the routing
        pidx = torch.empty((T, k), dtype=torch.int32, device=DEV)
        moe.moe_predict_next(shape, d["x"], d["wg"], d["bias"], pidx, None, None, ws)
        torch.cuda.synchronize()
        assert torch.equal(pidx, idx)


def test_mfma_calibration_probe_is_sane():
    """The register-only MFMA loop: plausible rates, and constant operands never slower than random ones."""
    const = moe.moe_calibrate_mfma(False, 4096)
    rnd = moe.moe_calibrate_mfma(True, 4096)
    assert const["flop"] == rnd["flop"] > 0
    assert 500 < rnd["tflops"] <= const["tflops"] * 1.05 and const["tflops"] < 2600
    assert 0.5 < rnd["ghz"] <= const["ghz"] * 1.05 and const["ghz"] < 2.6


def test_read_stream_probe_is_sane():
    """The plain read stream: a plausible rate, and the bytes it reports are what it was given (rounded down)."""
    buf = torch.empty(1 << 29, dtype=torch.uint8, device=DEV).fill_(1)     # 512 MB
    r = moe.moe_calibrate_read_stream(buf)
    assert 0.9 * buf.numel() <= r["bytes"] <= buf.numel()
    assert 1000 < r["GBps"] < 8000
