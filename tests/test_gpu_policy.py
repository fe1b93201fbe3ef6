"""Parity of the policy kernels (include/daop_policy.h) with the policy oracle: integer and index
results bit-exact, Eq. 1 to a few ulps of fp64."""
import numpy as np
import pytest
import torch

from paper_2501_10375_amd import moe, policy, synth
from parity_util import host

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _counts(rng, L, E, zero_rows=False, hi=500):
    c = rng.integers(0, hi, size=(L, E)).astype(np.int32)
    c[rng.random((L, E)) < 0.15] = 0
    if zero_rows and L > 2:
        c[1] = 0
    return c


@pytest.mark.parametrize("L,E", [(32, 8), (32, 16), (5, 64), (1, 3), (300, 7)])
def test_similarity_matches_eq1_oracle(L, E):
    from oracle import daop_policy as pol

    rng = np.random.default_rng(L * 100 + E)
    P, D = _counts(rng, L, E, zero_rows=True), _counts(rng, L, E)
    mean, per = policy.daop_similarity(torch.from_numpy(P).to(DEV), torch.from_numpy(D).to(DEV))
    torch.cuda.synchronize()
    ref_mean, ref_per = pol.similarity(P, D)
    assert np.allclose(per.cpu().numpy(), ref_per, rtol=0, atol=4e-16)
    assert abs(mean.item() - ref_mean) <= 4e-16 * max(1, L) ** 0.5 + 1e-15
    same, _ = policy.daop_similarity(torch.from_numpy(P).to(DEV), torch.from_numpy(P).to(DEV))
    nz = (P.sum(1) > 0).mean()
    assert abs(same.item() - nz) < 1e-14      # identical patterns: 1 per layer that saw tokens


@pytest.mark.parametrize("L,E,k,S,W", [(32, 8, 2, 128, 15), (32, 16, 2, 100, 15), (3, 64, 8, 47, 5), (1, 3, 1, 6, 2),
                                       (300, 7, 3, 31, 15), (4, 8, 2, 29, 15), (4, 8, 2, 14, 15), (2, 8, 2, 0, 15)])
def test_window_variation_matches_oracle(L, E, k, S, W):
    """Sec. VI-B: Eq. 1 between consecutive decode windows, bit for bit up to the rounding of the
    roots and quotients (the counts and their products are exact on both sides)."""
    from oracle import daop_policy as pol

    rng = np.random.default_rng(L * 1000 + E * 10 + S)
    # a drifting skew, so the windows differ by a realistic amount
    idx = np.zeros((L, S, k), dtype=np.int32)
    for l in range(L):
        for s in range(S):
            p = np.exp(-0.4 * ((np.arange(E) + s // 9 + l) % E))
            idx[l, s] = rng.choice(E, size=k, replace=False, p=p / p.sum())
    mean, per = policy.daop_window_variation(torch.from_numpy(idx).to(DEV), E, W)
    torch.cuda.synchronize()
    ref_mean, ref_per = pol.window_variation(idx, E, W)
    assert per.shape[0] == ref_per.shape[0] == max(S // W - 1, 0)
    assert np.allclose(per.cpu().numpy(), ref_per, rtol=0, atol=4e-16 * max(1, L) ** 0.5 + 1e-15)
    assert abs(mean.item() - ref_mean) <= 1e-15 * max(1, per.shape[0]) + 1e-15
    if S // W >= 2:
        assert 0.0 < ref_mean <= 1.0 + 1e-15


def test_window_variation_hand_worked_on_the_gpu():
    idx = torch.tensor([[[0], [0], [1], [0], [2], [1]]], dtype=torch.int32, device=DEV)
    mean, per = policy.daop_window_variation(idx, 3, 2)
    torch.cuda.synchronize()
    assert abs(per[0].item() - 2 / (2 * 2 ** 0.5)) < 1e-15 and abs(per[1].item() - 0.5) < 1e-15
    assert abs(mean.item() - (per[0].item() + per[1].item()) / 2) < 1e-15


@pytest.mark.parametrize("L,E,thr", [(32, 8, 1.05), (32, 16, 1.05), (7, 64, 1.05), (9, 5, 1.0), (4, 2, 1.05),
                                     (3, 1, 1.05), (16, 8, 0.0), (16, 8, 1e9)])
def test_plan_swaps_matches_algorithm1_oracle(L, E, thr):
    from oracle import daop_policy as pol

    rng = np.random.default_rng(L * 1000 + E)
    counts = _counts(rng, L, E, hi=40)          # small range: many ties and threshold-equal pairs
    mask = (rng.random((L, E)) < rng.random((L, 1))).astype(np.uint8)
    on_gpu = torch.from_numpy(mask.copy()).to(DEV)
    swaps, n_swaps = policy.daop_plan_swaps(torch.from_numpy(counts).to(DEV), on_gpu, thr)
    torch.cuda.synchronize()
    ref_swaps, ref_mask = pol.plan_swaps_all(counts, mask, thr)
    assert np.array_equal(on_gpu.cpu().numpy().astype(bool), ref_mask)
    sw, ns = swaps.cpu().numpy(), n_swaps.cpu().numpy()
    for l in range(L):
        assert ns[l] == len(ref_swaps[l])
        assert [tuple(p) for p in sw[l, : ns[l]].tolist()] == ref_swaps[l]
        assert (sw[l, ns[l]:] == -1).all()


def test_plan_swaps_golden_cases_on_the_gpu():
    from test_oracle_policy import _cases

    for counts, mask, expected in _cases():
        E = len(counts)
        on_gpu = torch.tensor([mask], dtype=torch.uint8, device=DEV)
        swaps, n = policy.daop_plan_swaps(torch.tensor([counts], dtype=torch.int32, device=DEV), on_gpu, 1.05)
        torch.cuda.synchronize()
        got = [tuple(p) for p in swaps[0, : int(n[0])].tolist()]
        assert got == expected, (counts, mask)


@pytest.mark.parametrize("L,E,slots", [(32, 8, 120), (32, 8, 64), (32, 16, 96), (3, 5, 7), (4, 4, 0), (4, 4, 16),
                                       (4, 4, 99), (40, 64, 1000), (6, 3, 5)])
def test_memory_init_matches_oracle(L, E, slots):
    from oracle import daop_policy as pol

    rng = np.random.default_rng(L * 7 + E + slots)
    calib = _counts(rng, L, E, zero_rows=True, hi=30)   # ties and an empty layer
    got = policy.daop_memory_init(torch.from_numpy(calib).to(DEV), slots)
    torch.cuda.synchronize()
    ref = pol.memory_init(calib, slots)
    assert np.array_equal(got.cpu().numpy().astype(bool), ref)
    assert int(got.sum().item()) == min(max(slots, 0), L * E)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("T,H,E,k", [(1, 256, 8, 2), (13, 512, 8, 2), (40, 256, 16, 2), (16, 128, 64, 4), (7, 4096, 8, 2)])
def test_predict_degraded_matches_oracle(oracle, dtype, T, H, E, k):
    from oracle import daop_policy as pol

    d = synth.moe_layer_inputs(T, H, 64, E, dtype, DEV, seed=3, zipf_s=1.2, with_next=True)
    shape = moe.make_shape(H, 64, E, k, dtype)
    h = host(d)
    ref = oracle.route(h["x"], h["wg_next"], h["bias_next"], k)
    p = np.asarray(ref["p"], dtype=np.float64)
    rng = np.random.default_rng(T + E)
    changed = 0
    for trial, frac in enumerate((0.0, 0.3, 0.6, 1.0)):
        mask = (rng.random(E) < frac).astype(np.uint8)
        idx = torch.full((T, k), -1, dtype=torch.int32, device=DEV)
        w = torch.zeros((T, k), dtype=torch.float32, device=DEV)
        policy.daop_predict_degraded(shape, d["x"], d["wg_next"], d["bias_next"], torch.from_numpy(mask).to(DEV), idx, w)
        torch.cuda.synchronize()
        gi, gw = idx.cpu().numpy(), w.cpu().numpy()
        skipped = 0
        for t in range(T):
            want_idx, want_w = pol.degrade_selection(p[t], k, mask)
            # near ties (Q5 margin rule) in the plain top-k or between the replacement candidates are not compared
            ps = np.sort(p[t])[::-1]
            gaps = [ps[r] - ps[r + 1] for r in range(min(k, E - 1))]
            res = np.sort(p[t][mask.astype(bool)])[::-1]
            if len(res) > 1:
                gaps.append(res[0] - res[1])
            if min(gaps) < 1e-4:
                skipped += 1
                continue
            assert gi[t].tolist() == want_idx, (trial, t)
            assert np.allclose(gw[t], want_w, rtol=0, atol=5e-5)
            changed += want_idx != list(np.argsort(-p[t], kind="stable")[:k])
            assert len(set(gi[t].tolist())) == k
        assert skipped <= max(1, T // 8)
        if frac in (0.0, 1.0):   # nothing / everything resident: identical to the plain prediction
            plain = torch.empty((T, k), dtype=torch.int32, device=DEV)
            ws = moe.alloc_workspace(shape, T)
            moe.moe_predict_next(shape, d["x"], d["wg_next"], d["bias_next"], plain, None, None, ws)
            torch.cuda.synchronize()
            if T <= 16:
                assert torch.equal(plain, idx)
    print("tokens whose selection was degraded:", changed)
