"""The multi-layer harness (paper_2501_10375_amd/stack.py): teacher-forced per-layer parity with the
oracle (each layer's oracle sees the GPU's actual layer input, because bf16 drift through a stack
legitimately changes selections), count matrices, agreement rates and Eq. 1."""
import numpy as np
import pytest
import torch

from paper_2501_10375_amd import moe, policy, stack, synth
from parity_util import check_layer, check_routing, host, output_error, tile_aware_sample

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_small_stack_teacher_forced_parity(oracle):
    from oracle import daop_policy as pol

    L, H, F, E, k, T = 4, 256, 512, 8, 2, 40
    st = stack.MoeStack(L, H, F, E, k, torch.bfloat16, DEV, zipf_s=1.2, max_tokens=T)
    h0 = synth.normal((T, H), 500, synth.TID_X, 1.0, torch.float32, DEV)
    prefill = st.new_counts()
    out = st.forward(h0, prefill, keep_inputs=True, keep_outputs=True)
    torch.cuda.synchronize()
    idx = out["idx"].clone()
    pred = out["pred"].clone()
    excluded = 0
    ref_idx = []
    for l in range(L):
        d = dict(st.layers[l], x=out["inputs"][l])
        nxt = st.layers[l + 1] if l + 1 < L else None
        d["wg_next"], d["bias_next"] = (nxt["wg"], nxt["bias"]) if nxt else (None, None)
        y, w = out["outputs"][l]
        res = {"y": y, "idx": idx[l], "w": w, "counts": prefill[l, :E], "pred_idx": pred[l] if nxt else None}
        r = check_layer(oracle, d, st.shape, res, torch.bfloat16, label=f"stack layer {l}", predict=nxt is not None)
        excluded += r["excluded"] + r["excluded_pred"]
        hd = host(d)
        ref_idx.append(oracle.route(hd["x"], hd["wg"], hd["bias"], k)["idx"])
    assert excluded <= 2
    assert prefill[:, :E].sum(1).tolist() == [T * k] * L

    # agreement rates: the harness's numbers equal the ones recomputed on the host from its own outputs,
    # and the oracle's (teacher-forced) unless a near-tie token was excluded
    exact, overlap = stack.agreement(pred, idx)
    pi, ai = pred.cpu().numpy(), idx.cpu().numpy()
    for l in range(L - 1):
        same = [set(pi[l, t]) == set(ai[l + 1, t]) for t in range(T)]
        ov = [len(set(pi[l, t]) & set(ai[l + 1, t])) / k for t in range(T)]
        assert abs(exact[l].item() - np.mean(same)) < 1e-12 and abs(overlap[l].item() - np.mean(ov)) < 1e-12
    assert 0.0 <= exact.min().item() and overlap.max().item() <= 1.0

    # decode steps accumulate into their own count matrix; Eq. 1 between the two matrices
    decode = st.new_counts()
    for step in range(6):
        h = synth.normal((1, H), 1000 + step, synth.TID_X, 1.0, torch.float32, DEV)
        st.forward(h, decode)
    torch.cuda.synchronize()
    assert decode[:, :E].sum(1).tolist() == [6 * k] * L
    P = prefill[:, :E].contiguous()
    D = decode[:, :E].contiguous()
    sim, per = policy.daop_similarity(P, D)
    ref_sim, ref_per = pol.similarity(P.cpu().numpy(), D.cpu().numpy())
    assert abs(sim.item() - ref_sim) < 1e-14 and np.allclose(per.cpu().numpy(), ref_per, atol=1e-15)

    # the counts drive Algorithm 1: plan on the prefill counts from a calibrated cache of half the experts
    cache = policy.daop_memory_init(D, L * E // 2)
    before = cache.clone()
    swaps, n = policy.daop_plan_swaps(P, cache)
    torch.cuda.synchronize()
    ref_swaps, ref_mask = pol.plan_swaps_all(P.cpu().numpy(), before.cpu().numpy())
    assert np.array_equal(cache.cpu().numpy().astype(bool), ref_mask)
    assert n.cpu().tolist() == [len(s) for s in ref_swaps]
    covered_before = (P * before.int()).sum().item()
    covered_after = (P * cache.int()).sum().item()
    assert covered_after >= covered_before   # more prefill tokens hit GPU-resident experts after the swaps


@pytest.mark.timeout(900)
def test_full_size_stack_teacher_forced_parity(oracle):
    """The benchmark's multi-layer workload at its real size: 32 resident Mixtral-shaped layers
    (Table III; 90 GB of expert weights), a 1024-token prefill and one single-token decode step.
    Teacher-forced: each layer's oracle sees the input the GPU's layer saw.  Routing, counts and the
    prediction are compared on every token of every layer; layer outputs on layers 0, 1, 4, 15 and 31
    (sampled prefill tokens chosen by slot-tile position, and the decode token)."""
    L, H, F, E, k, T = 32, 4096, 14336, 8, 2, 1024
    free, _ = torch.cuda.mem_get_info()
    need = L * E * 3 * H * F * 2 + (8 << 30)
    if free < need:
        pytest.skip(f"needs {need >> 30} GiB of free device memory, {free >> 30} GiB available")
    st = stack.MoeStack(L, H, F, E, k, torch.bfloat16, DEV, zipf_s=1.2, max_tokens=T)
    assert abs(st.weight_bytes() / 1e9 - 90.2) < 0.1
    sampled_layers = (0, 1, 4, 15, 31)
    for phase, tokens, seed in (("prefill", T, 999), ("decode", 1, 1000)):
        h0 = synth.normal((tokens, H), seed, synth.TID_X, 1.0, torch.float32, DEV)
        counts = st.new_counts()
        out = st.forward(h0, counts, keep_inputs=True, keep_outputs=True)
        torch.cuda.synchronize()
        assert counts[:, :E].sum(1).tolist() == [tokens * k] * L
        idx, pred = out["idx"].clone(), out["pred"].clone()
        excluded = 0
        for l in range(L):
            nxt = st.layers[l + 1] if l + 1 < L else None
            y, w = out["outputs"][l]
            label = f"full stack {phase} layer {l}"
            print(label, flush=True)
            if l in sampled_layers:
                d = dict(st.layers[l], x=out["inputs"][l])
                d["wg_next"], d["bias_next"] = (nxt["wg"], nxt["bias"]) if nxt else (None, None)
                res = {"y": y, "idx": idx[l], "w": w, "counts": counts[l, :E], "pred_idx": pred[l] if nxt else None}
                sample = None if tokens <= 64 else tile_aware_sample(idx[l].cpu().numpy(), E, 32, n_cold=1)
                r = check_layer(oracle, d, st.shape, res, torch.bfloat16, tokens=sample, label=label,
                                predict=nxt is not None)
                print(label, r, flush=True)
                assert r["compared_tokens"] >= min(tokens, 32)
                excluded += r["excluded"] + r["excluded_pred"]
            else:
                x = synth.to_numpy(out["inputs"][l])
                d = st.layers[l]
                ref = oracle.route(x, synth.to_numpy(d["wg"]), synth.to_numpy(d["bias"]), k)
                n, _ = check_routing(idx[l], w, counts[l, :E], ref, E, label)
                excluded += n
                if nxt is not None:
                    pref = oracle.predict_next(x, synth.to_numpy(nxt["wg"]), synth.to_numpy(nxt["bias"]), k)
                    n, _ = check_routing(pred[l], None, None, pref, E, label + " (prediction)")
                    excluded += n
        assert excluded <= 0.01 * 2 * L * tokens + 2
        del out
    del st
    torch.cuda.empty_cache()


def test_precalculation_variant(oracle):
    """DAOP's decode approximation on a small stack: exact when no layer is predicted; per layer the
    mix of fresh and stale expert inputs matches the oracle evaluated the same way; the output
    error against the exact stack shrinks as the cache grows."""
    L, H, F, E, k, T = 6, 256, 512, 8, 2, 12
    st = stack.MoeStack(L, H, F, E, k, torch.bfloat16, DEV, zipf_s=1.2, max_tokens=T)
    h0 = synth.normal((T, H), 77, synth.TID_X, 1.0, torch.float32, DEV)
    exact = st.forward(h0, st.new_counts())["h"].clone()

    none = torch.zeros((L, E), dtype=torch.uint8, device=DEV)
    same = stack.forward_precalc(st, h0, none, first_predicted_layer=L)
    assert same["stale_selections"] == 0 and torch.equal(same["h"], exact)

    errs = []
    for slots in (0, L * E // 4, L * E // 2, L * E):
        cache = policy.daop_memory_init(torch.ones((L, E), dtype=torch.int32, device=DEV).cumsum(1).int().contiguous(), slots)
        r = stack.forward_precalc(st, h0, cache, first_predicted_layer=2, keep_layers=True)
        torch.cuda.synchronize()
        errs.append(((r["h"] - exact).norm() / exact.norm()).item())
        if slots == L * E:
            assert r["stale_selections"] == 0
        # one predicted layer against the oracle: fresh experts on u_l, stale ones on u_{l-1}
        l = 3
        u_prev, u, idx, w, stale, out = r["layers"][l]
        d = st.layers[l]
        hd = host(dict(w1=d["w1"], w3=d["w3"], w2=d["w2"], u=u, u_prev=u_prev))
        idx_h, w_h, st_h = idx.cpu().numpy(), w.cpu().numpy().astype(np.float64), stale.cpu().numpy() != 0
        ref = oracle.expert_ffn_precalc(hd["u"], hd["u_prev"], st_h, idx_h, w_h, hd["w1"], hd["w3"], hd["w2"])
        assert output_error(out.double().cpu().numpy(), ref) <= 2e-2
        # the cache decides which selections are stale
        assert np.array_equal(st_h, cache[l].cpu().numpy()[idx_h] == 0)
    print("relative error of the final hidden state vs cache slots:", errs)
    assert errs[-1] <= errs[0] + 1e-6 and errs[0] > 0


def test_decode_step_replays_from_a_graph():
    """The whole stack's decode step as one HIP graph: every replay equals the eager pass on the same
    hidden state bit for bit (final hidden state, selections, predictions) and the counts add up."""
    L, H, F, E, k = 5, 256, 512, 8, 2
    st = stack.MoeStack(L, H, F, E, k, torch.bfloat16, DEV, zipf_s=1.2, max_tokens=4)
    graph_counts, eager_counts = st.new_counts(), st.new_counts()
    step = stack.CapturedStep(st, 1, graph_counts)
    for i in range(5):
        h = synth.normal((1, H), 7000 + i, synth.TID_X, 1.0, torch.float32, DEV)
        ref = st.forward(h, eager_counts)                      # eager work between the replays
        ref = {key: ref[key].clone() for key in ("h", "idx", "pred")}
        torch.cuda.synchronize()
        step.h_in.copy_(h)
        got = step.replay()
        torch.cuda.synchronize()
        for key in ("h", "idx", "pred"):
            assert torch.equal(got[key], ref[key]), f"replay {i}: {key}"
        assert torch.equal(graph_counts, eager_counts), f"replay {i}: counts"
    assert graph_counts[:, :E].sum(1).tolist() == [5 * k] * L
