"""Pins of the policy oracle (oracle/daop_policy.py): hand-worked cases, closed forms, invariants,
brute force on tiny inputs.  No GPU."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import daop_policy as pol

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _cases():
    out = []
    for line in open(os.path.join(GOLDEN, "alg1_cases.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        c, m, s = [part.strip() for part in line.split("|")]
        swaps = [tuple(int(v) for v in tok.split(">")) for tok in s.split()]
        out.append(([int(v) for v in c.split()], [int(v) for v in m.split()], swaps))
    return out


@pytest.mark.parametrize("counts,mask,expected", _cases())
def test_algorithm1_hand_worked_cases(counts, mask, expected):
    swaps, new = pol.plan_swaps(counts, mask, 1.05)
    assert swaps == expected
    want = list(map(bool, mask))
    for h, c in expected:
        want[h], want[c] = True, False
    assert new == want


def test_algorithm1_invariants_random():
    rng = np.random.default_rng(0)
    for _ in range(300):
        E = int(rng.integers(2, 17))
        counts = rng.integers(0, 50, size=E)
        mask = rng.random(E) < rng.random()
        swaps, new = pol.plan_swaps(counts, mask, 1.05)
        assert sum(new) == int(mask.sum())                 # cache size never changes
        assert len(swaps) <= E // 2
        ins = [h for h, _ in swaps]
        outs = [c for _, c in swaps]
        assert len(set(ins)) == len(ins) and len(set(outs)) == len(outs)
        for h, c in swaps:
            assert not mask[h] and mask[c]
            assert counts[h] > 0 and counts[h] >= 1.05 * counts[c]
        # every swapped-in expert is at least as active as every CPU expert that stayed out of the hot list
        if swaps:
            assert min(counts[h] for h in ins) >= 0
        # an infinite threshold freezes the cache; a zero threshold swaps every pair with a non-idle hot expert
        assert pol.plan_swaps(counts, mask, float("inf"))[0] == []
        n_pairs = min(E // 2, int((~mask).sum()), int(mask.sum()))
        hot_sorted = sorted((int(counts[e]) for e in range(E) if not mask[e]), reverse=True)[:n_pairs]
        assert len(pol.plan_swaps(counts, mask, 0.0)[0]) == sum(1 for v in hot_sorted if v > 0)


def test_algorithm1_total_gpu_activity_never_decreases():
    """Each swap brings in an expert with more tokens than the one it evicts (threshold > 1)."""
    rng = np.random.default_rng(1)
    for _ in range(200):
        E = 8
        counts = rng.integers(0, 100, size=E)
        mask = np.zeros(E, bool)
        mask[rng.permutation(E)[: int(rng.integers(0, E + 1))]] = True
        _, new = pol.plan_swaps(counts, mask, 1.05)
        assert counts[np.array(new)].sum() >= counts[mask].sum()


def test_similarity_closed_forms():
    rng = np.random.default_rng(2)
    P = rng.integers(1, 100, size=(5, 8)).astype(float)
    mean, per = pol.similarity(P, P)
    assert abs(mean - 1.0) < 1e-15 and np.allclose(per, 1.0, atol=1e-15)
    # invariant to a positive scale per row (counts vs probabilities, Eq. 1's normalisation is immaterial)
    scale = rng.random((5, 1)) * 10 + 0.1
    D = rng.integers(0, 100, size=(5, 8)).astype(float)
    assert abs(pol.similarity(P * scale, D)[0] - pol.similarity(P, D)[0]) < 1e-14
    # orthogonal rows -> 0; a 3-4-5 construction -> 0.6 and 0.8
    assert pol.similarity([[1, 0], [0, 2]], [[0, 3], [5, 0]])[0] == 0.0
    mean, per = pol.similarity([[1, 0], [0, 1]], [[3, 4], [3, 4]])
    assert abs(per[0] - 0.6) < 1e-15 and abs(per[1] - 0.8) < 1e-15 and abs(mean - 0.7) < 1e-15
    # against the library routine
    ref = [np.dot(P[l], D[l]) / (np.linalg.norm(P[l]) * np.linalg.norm(D[l])) for l in range(5)]
    assert np.allclose(pol.similarity(P, D)[1], ref, rtol=1e-13)
    # a layer that saw no tokens contributes 0
    mean, per = pol.similarity([[0, 0], [1, 1]], [[1, 2], [1, 1]])
    assert per[0] == 0.0 and abs(per[1] - 1.0) < 1e-15 and abs(mean - 0.5) < 1e-15


def test_memory_init_paper_arithmetic():
    """Sec. V-A/B: an expert cache ratio of 46.875 % of Mixtral's 32 x 8 experts is 120 slots
    = 3 per layer + 24 left over (fewer than the 32 layers)."""
    L, E = 32, 8
    slots = round(0.46875 * L * E)
    assert slots == 120 and slots // L == 3 and slots - 3 * L == 24
    rng = np.random.default_rng(3)
    calib = rng.integers(0, 1000, size=(L, E))
    mask = pol.memory_init(calib, slots)
    assert mask.sum() == 120
    per = mask.sum(1)
    assert per.min() >= 3 and (per - 3).sum() == 24     # uniform base, leftover slots spread by frequency
    # the leftover slots hold the 24 largest frequencies among the experts outside the uniform base
    share = calib / calib.sum(1, keepdims=True)
    base = np.zeros_like(mask)
    for l in range(L):
        base[l, sorted(range(E), key=lambda e: (-calib[l, e], e))[:3]] = True
    extra = mask & ~base
    assert extra.sum() == 24 and share[extra].min() >= share[~mask].max()
    # every layer's residents are its most active experts
    for l in range(L):
        order = sorted(range(E), key=lambda e: (-calib[l, e], e))
        assert set(np.flatnonzero(mask[l])) == set(order[: per[l]])


def test_memory_init_leftover_goes_to_highest_frequency():
    # two layers, 3 slots: one each, then the leftover to the larger share c / row
    calib = np.array([[50, 30, 20], [10, 9, 1]])          # shares .5 .3 .2 | .5 .45 .05
    mask = pol.memory_init(calib, 3)
    assert mask.tolist() == [[True, False, False], [True, True, False]]   # 9/20 = .45 beats 30/100 = .30
    # brute force over all masks with the same per-layer base: the leftover maximises total resident frequency
    share = calib / calib.sum(1, keepdims=True)
    best = max(((l, e) for l in range(2) for e in range(3) if not (e == 0)), key=lambda le: (share[le], -le[0], -le[1]))
    assert best == (1, 1)
    # limits
    assert pol.memory_init(calib, 0).sum() == 0 and pol.memory_init(calib, 99).all()
    assert pol.memory_init(np.zeros((2, 3), int), 1).tolist() == [[True, False, False], [False, False, False]]


def test_degrade_selection_rules():
    p = [0.05, 0.40, 0.30, 0.15, 0.10]
    # a selected expert is on the GPU: nothing changes
    idx, w = pol.degrade_selection(p, 2, [0, 1, 0, 0, 0])
    assert idx == [1, 2] and abs(w[0] - 0.4 / 0.7) < 1e-15
    # both off the GPU: the lower score (2) gives way to the best expert on the GPU (3)
    idx, w = pol.degrade_selection(p, 2, [1, 0, 0, 1, 1])
    assert idx == [1, 3] and abs(sum(w) - 1) < 1e-15 and abs(w[1] - 0.15 / 0.55) < 1e-15
    # nothing on the GPU: the original selection is kept
    assert pol.degrade_selection(p, 2, [0, 0, 0, 0, 0])[0] == [1, 2]
    # everything on the GPU, or k = E: never changes; exhaustive over all masks for a small case
    for mask in itertools.product([0, 1], repeat=5):
        idx, w = pol.degrade_selection(p, 2, mask)
        assert len(set(idx)) == 2 and abs(sum(w) - 1) < 1e-12
        assert p[idx[0]] >= p[idx[1]]
        if mask[1] or mask[2]:
            assert idx == [1, 2]
        elif any(mask):
            assert idx[0] == 1 and mask[idx[1]] and p[idx[1]] == max(p[e] for e in range(5) if mask[e])
        else:
            assert idx == [1, 2]


# ---- Sec. VI-B: variation of the activation pattern over 15-token windows of the decode phase ----

def test_window_variation_hand_worked():
    # one layer, three experts, top-1, windows of two steps: counts [2,0,0] then [1,1,0] then [0,1,1]
    idx = np.array([[[0], [0], [1], [0], [2], [1]]])
    mean, per = pol.window_variation(idx, 3, window=2)
    assert per.shape == (2,)
    assert abs(per[0] - 2 / (2 * math.sqrt(2))) < 1e-15      # (2*1) / (|[2,0,0]| |[1,1,0]|)
    assert abs(per[1] - 1 / 2) < 1e-15                       # (1*1) / (sqrt 2 * sqrt 2)
    assert abs(mean - (per[0] + per[1]) / 2) < 1e-15


def test_window_variation_limits():
    rng = np.random.default_rng(5)
    L, E, k, W = 3, 8, 2, 15
    same = np.tile(np.array([[[1, 4]]]), (L, 4 * W, 1))
    assert pol.window_variation(same, E)[0] == pytest.approx(1.0, abs=1e-15)      # the pattern never changes
    a = np.tile(np.array([[[0, 1]]]), (L, W, 1))
    b = np.tile(np.array([[[2, 3]]]), (L, W, 1))
    mean, per = pol.window_variation(np.concatenate([a, b, a], axis=1), E)         # disjoint expert sets
    assert mean == 0.0 and per.tolist() == [0.0, 0.0]
    # fewer than two whole windows: no pair
    assert pol.window_variation(same[:, : 2 * W - 1], E) [0] == 0.0 and pol.window_variation(same[:, :W], E)[1].size == 0
    # a shorter tail is left out; the order of the steps inside a window does not matter
    idx = np.stack([np.stack([rng.permutation(E)[:k] for _ in range(3 * W + 7)]) for _ in range(L)])
    full = pol.window_variation(idx, E)
    assert np.array_equal(pol.window_variation(idx[:, : 3 * W], E)[1], full[1])
    shuffled = idx.copy()
    shuffled[:, W:2 * W] = shuffled[:, W:2 * W][:, rng.permutation(W)]
    assert np.array_equal(pol.window_variation(shuffled, E)[1], full[1])
    # window = 15 is the default
    assert np.array_equal(pol.window_variation(idx, E, window=15)[1], full[1])


def test_window_variation_is_eq1_between_consecutive_window_counts():
    rng = np.random.default_rng(6)
    L, E, k, W, S = 4, 6, 2, 5, 20
    idx = np.stack([np.stack([rng.permutation(E)[:k] for _ in range(S)]) for _ in range(L)])
    mean, per = pol.window_variation(idx, E, window=W)

    def counts(v):   # library histogram of one window, per layer
        return np.stack([np.bincount(idx[l, v * W:(v + 1) * W].ravel(), minlength=E) for l in range(L)])

    want = [pol.similarity(counts(v), counts(v + 1))[0] for v in range(S // W - 1)]
    assert np.array_equal(per, np.array(want)) and mean == pytest.approx(np.mean(want), abs=1e-15)
    assert counts(0).sum() == L * W * k
