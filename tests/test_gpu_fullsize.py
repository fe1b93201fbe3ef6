"""Parity at the benchmark's full sizes (Table III shapes), in the launch configuration bench.py
times: routing, counts and prediction on every token; layer outputs on sampled tokens the oracle
can compute one by one; count invariants on everything."""
import numpy as np
import pytest
import torch

from paper_2501_10375_amd import moe, synth
from parity_util import check_layer, tile_aware_sample

pytestmark = pytest.mark.gpu
DEV = "cuda"

MIXTRAL = dict(H=4096, F=14336, E=8, k=2, zipf=1.2)
PHI = dict(H=4096, F=6400, E=16, k=2, zipf=1.5)


@pytest.fixture(scope="module")
def mixtral():
    c = MIXTRAL
    d = synth.moe_layer_inputs(4096, c["H"], c["F"], c["E"], torch.bfloat16, DEV, seed=0, zipf_s=c["zipf"])
    yield d
    del d
    torch.cuda.empty_cache()


@pytest.fixture(scope="module")
def phi():
    c = PHI
    d = synth.moe_layer_inputs(2048, c["H"], c["F"], c["E"], torch.bfloat16, DEV, seed=0, zipf_s=c["zipf"])
    yield d
    del d
    torch.cuda.empty_cache()


def _layer(oracle, d, c, T, n_sample, label, tile_aware=False):
    shape = moe.make_shape(c["H"], c["F"], c["E"], c["k"], torch.bfloat16)
    call = dict(d, x=d["x"][:T].contiguous())
    out = moe.LayerOutputs(shape, T, torch.bfloat16, DEV)
    res = moe.run_layer(shape, call, out)
    torch.cuda.synchronize()
    assert int(res["counts"].sum().item()) == T * c["k"]
    if n_sample >= T:
        tokens = None
    elif tile_aware:
        tokens = tile_aware_sample(res["idx"].cpu().numpy(), c["E"], n_sample)
    else:
        tokens = np.unique(np.linspace(0, T - 1, n_sample).astype(int))
    r = check_layer(oracle, call, shape, res, torch.bfloat16, tokens=tokens, label=label)
    print(label, r, "counts", res["counts"].tolist(), flush=True)
    assert r["excluded"] <= max(2, 0.01 * T)
    return r, res


@pytest.mark.parametrize("T", [1, 8, 16])
def test_mixtral_decode(oracle, mixtral, T):
    _layer(oracle, mixtral, MIXTRAL, T, T, f"mixtral decode T={T}")


@pytest.mark.parametrize("T", [32, 64, 100])
def test_mixtral_mid_sizes(oracle, mixtral, T):
    _layer(oracle, mixtral, MIXTRAL, T, 32, f"mixtral T={T}")


@pytest.mark.parametrize("T", [512, 2048, 4096])
def test_mixtral_prefill(oracle, mixtral, T):
    """The three prefill lengths of the benchmark.  The output is compared on every token of the two
    least-used experts, both ends of every slot tile, every fragment position of the busiest expert's
    first and last tile, and an even sample: several hundred tokens per length."""
    r, res = _layer(oracle, mixtral, MIXTRAL, T, 256, f"mixtral prefill T={T}", tile_aware=True)
    assert r["compared_tokens"] >= 250
    share = res["counts"].float() / res["counts"].sum()
    assert share[0] > 0.3 and share[-1] < 0.06  # the Zipf(1.2) skew of the benchmark recipe


def test_phi_prefill_and_decode(oracle, phi):
    r, res = _layer(oracle, phi, PHI, 2048, 256, "phi prefill T=2048", tile_aware=True)
    assert r["compared_tokens"] >= 250
    top4 = torch.sort(res["counts"], descending=True).values[:4].sum().item() / res["counts"].sum().item()
    assert top4 > 0.8  # four experts take most tokens (load-imbalance stress)
    _layer(oracle, phi, PHI, 1, 1, "phi decode T=1")


@pytest.mark.parametrize("T", [1, 5])
def test_mixtral_decode_sequence_on_one_workspace(mixtral, T):
    """Decode steps share one workspace: the intermediate of an earlier step must never be what a
    later step reads (its caches may still hold it), and the barrier flags need no clearing."""
    c = MIXTRAL
    shape = moe.make_shape(c["H"], c["F"], c["E"], c["k"], torch.bfloat16)
    shared = moe.LayerOutputs(shape, T, torch.bfloat16, DEV, predict=False)
    for step in range(6):
        x = synth.normal((T, c["H"]), 2000 + step, synth.TID_X, 1.0, torch.bfloat16, DEV)
        call = dict(mixtral, x=x, wg_next=None, bias_next=None)
        got = moe.run_layer(shape, call, shared, predict=False)
        y, idx = got["y"].clone(), got["idx"].clone()
        fresh = moe.LayerOutputs(shape, T, torch.bfloat16, DEV, predict=False)
        fresh.workspace.fill_(0xA5)
        ref = moe.run_layer(shape, call, fresh, predict=False)
        torch.cuda.synchronize()
        assert torch.equal(idx, ref["idx"]), f"step {step}"
        assert torch.equal(y.view(torch.int16), ref["y"].view(torch.int16)), f"step {step}"


@pytest.mark.parametrize("T,dtype", [(20000, torch.bfloat16), (20000, torch.float32), (1 << 20, torch.bfloat16)])
def test_long_calls_up_to_the_token_limit(oracle, T, dtype):
    """More than 1024 routing blocks take the two-kernel counts/permutation path; 2^20 tokens is the
    documented maximum.  Narrow layers keep the oracle's share in seconds."""
    H, F, E, k = 64, 64, 8, 2
    d = synth.moe_layer_inputs(T, H, F, E, dtype, DEV, seed=5, zipf_s=1.2)
    shape = moe.make_shape(H, F, E, k, dtype)
    out = moe.LayerOutputs(shape, T, dtype, DEV)
    res = moe.run_layer(shape, d, out)
    torch.cuda.synchronize()
    assert int(res["counts"].sum().item()) == T * k
    tokens = np.unique(np.linspace(0, T - 1, 48).astype(int))
    r = check_layer(oracle, d, shape, res, dtype, tokens=tokens, label=f"long call T={T}")
    print(r, flush=True)
    assert r["excluded"] <= 0.01 * T
    # the permutation is a bijection between assignments and slots, grouped by expert in token order
    idx = res["idx"].flatten().long()
    order = torch.argsort(idx, stable=True)
    assert torch.equal(torch.bincount(idx, minlength=E).int(), res["counts"])
    del order
