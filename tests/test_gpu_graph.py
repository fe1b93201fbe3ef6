"""A moe_layer call recorded into a HIP graph (stream capture) replays correctly: the library's
kernels take nothing from the host that changes between calls.  Each graph is replayed several
times with new inputs written into its static input buffer, with eager calls and synchronisations
between the replays, and every replay is compared bit for bit with the eager call on the same input."""
import pytest
import torch

from paper_2501_10375_amd import moe, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("T,H,F,E,k", [
    (1, 256, 512, 8, 2),      # one kernel: routing, experts, prediction
    (8, 512, 1600, 16, 2),    # decode size, tiles that do not divide the grid
    (24, 256, 512, 8, 2),     # routing kernels + the streaming expert kernel
    (300, 256, 512, 8, 2),    # prefill path: routing, permutation, grouped GEMMs with a split last round, combine
])
def test_layer_call_replays_from_a_graph(T, H, F, E, k):
    dtype = torch.bfloat16
    d = synth.moe_layer_inputs(T, H, F, E, dtype, DEV, seed=5, zipf_s=1.2, with_next=True)
    shape = moe.make_shape(H, F, E, k, dtype)
    x_static = d["x"].clone()
    graph_out = moe.LayerOutputs(shape, T, dtype, DEV, predict=True)
    eager_out = moe.LayerOutputs(shape, T, dtype, DEV, predict=True)
    call = moe.PreparedLayerCall(shape, dict(d, x=x_static), graph_out, predict=True)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(2):      # warm-up outside the capture (one-time kernel attribute calls)
            call()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call()
    torch.cuda.synchronize()

    for step in range(5):
        x = synth.normal((T, H), 4000 + step, synth.TID_X, 1.0, dtype, DEV)
        ref = moe.run_layer(shape, dict(d, x=x), eager_out, predict=True)      # eager work between the replays
        ref = {key: v.clone() for key, v in ref.items() if v is not None}
        torch.cuda.synchronize()
        x_static.copy_(x)
        g.replay()
        torch.cuda.synchronize()
        got = call.result
        assert torch.equal(got["idx"], ref["idx"]), f"replay {step}"
        assert torch.equal(got["pred_idx"], ref["pred_idx"]), f"replay {step}"
        assert torch.equal(got["counts"], ref["counts"]), f"replay {step}"
        assert torch.equal(got["y"].view(torch.int16), ref["y"].view(torch.int16)), f"replay {step}"
