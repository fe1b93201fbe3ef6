"""moe_layer_static: the whole layer on the library's static device scratch (for callers that cannot
allocate).  It must give what moe_layer gives on a caller's workspace, bit for bit, and that must
match the oracle; the array is shared by all calls on the GPU and keeps the last call's contents, so
each case runs two calls in a row, the second on a smaller input."""
import pytest
import torch

from paper_2501_10375_amd import moe, synth
from parity_util import check_layer

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _both(shape, d, T, dtype):
    call = dict(d, x=d["x"][:T].contiguous())
    ref_out = moe.LayerOutputs(shape, T, dtype, DEV)
    ref_out.workspace.fill_(0x5A)
    ref = moe.run_layer(shape, call, ref_out)
    E, k, H = shape.n_experts, shape.top_k, shape.hidden
    y = torch.full((T, H), 7, dtype=dtype, device=DEV)
    idx = torch.full((T, k), -1, dtype=torch.int32, device=DEV)
    w = torch.zeros((T, k), dtype=torch.float32, device=DEV)
    counts = torch.full((E,), -5, dtype=torch.int32, device=DEV)
    pred = torch.full((T, k), -1, dtype=torch.int32, device=DEV)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    moe.moe_layer_static(shape, call["x"], d["wg"], d["bias"], d["wg_next"], d["bias_next"], d["w1"], d["w3"], d["w2"],
                         y, idx, w, counts, False, pred)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    got = {"y": y, "idx": idx, "w": w, "counts": counts, "pred_idx": pred}
    for key in ("idx", "w", "counts", "pred_idx"):
        assert torch.equal(got[key], ref[key]), key
    assert torch.equal(y.view(torch.uint8), ref["y"].view(torch.uint8))
    return call, got


@pytest.mark.parametrize("dtype,H,F,E,k,sizes", [
    (torch.bfloat16, 512, 1024, 8, 2, (16, 3)),      # one-kernel decode path, then fewer tokens
    (torch.bfloat16, 256, 512, 8, 2, (32, 17)),      # streaming kernel with separate routing kernels
    (torch.bfloat16, 4096, 14336, 8, 2, (8, 1)),     # Table III Mixtral shape at decode sizes
    (torch.float32, 256, 512, 8, 2, (64, 20)),       # fp32 path: permutation, both GEMMs and combine use the scratch
])
def test_static_scratch_layer_matches_workspace_layer_and_oracle(oracle, dtype, H, F, E, k, sizes):
    d = synth.moe_layer_inputs(max(sizes), H, F, E, dtype, DEV, seed=21, zipf_s=1.2)
    shape = moe.make_shape(H, F, E, k, dtype)
    for T in sizes:     # two calls in a row on the shared array, the second smaller
        assert moe.moe_workspace_bytes(shape, T) <= moe.MOE_STATIC_SCRATCH_BYTES
        call, got = _both(shape, d, T, dtype)
        r = check_layer(oracle, call, shape, got, dtype, label=f"static scratch T={T}")
        print(T, r, flush=True)
    assert not moe.moe_decode_status(None)


def test_static_scratch_rejects_calls_that_do_not_fit():
    H, F, E, k, dtype = 256, 512, 8, 2, torch.bfloat16
    T = 33   # bf16 calls past the streaming sizes need 64 MiB of K-split pieces
    d = synth.moe_layer_inputs(T, H, F, E, dtype, DEV, seed=21)
    shape = moe.make_shape(H, F, E, k, dtype)
    assert moe.moe_workspace_bytes(shape, T) > moe.MOE_STATIC_SCRATCH_BYTES
    y = torch.zeros((T, H), dtype=dtype, device=DEV)
    idx = torch.zeros((T, k), dtype=torch.int32, device=DEV)
    w = torch.zeros((T, k), dtype=torch.float32, device=DEV)
    counts = torch.zeros((E,), dtype=torch.int32, device=DEV)
    with pytest.raises(moe.MoeError) as err:
        moe.moe_layer_static(shape, d["x"], d["wg"], d["bias"], None, None, d["w1"], d["w3"], d["w2"], y, idx, w, counts,
                             False, None)
    assert err.value.status == moe.MOE_ERR_TOO_LARGE
    torch.cuda.synchronize()
    assert not y.any() and not counts.any()   # nothing was enqueued
