"""Pins for the oracle's routing, counts, margin and prediction.

None of these call the HIP library.  Expected values come from exact rational
arithmetic on dyadic inputs, closed forms, invariants and special cases, so a
dropped bias, a transposed gate, a wrong sort direction or a missing
renormalisation each fail at least one test.
"""
import math
from fractions import Fraction

import numpy as np
import pytest


def _dyadic(rng, shape, denom, lo, hi):
    return rng.integers(lo, hi + 1, size=shape).astype(np.float64) / denom


def _exact_logits(x, wg, bias):
    T, H = x.shape
    E = wg.shape[0]
    z = [[Fraction(0) for _ in range(E)] for _ in range(T)]
    for t in range(T):
        for e in range(E):
            s = Fraction(0)
            for h in range(H):
                s += Fraction(float(x[t, h])) * Fraction(float(wg[e, h]))
            if bias is not None:
                s += Fraction(float(bias[e]))
            z[t][e] = s
    return z


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("T,H,E,k", [(8, 16, 8, 2), (5, 7, 6, 3), (3, 4, 2, 1), (4, 9, 5, 5)])
def test_topk_bruteforce_on_dyadic_inputs(oracle, dtype, T, H, E, k):
    rng = np.random.default_rng(100 + T + H + E + k)
    x = _dyadic(rng, (T, H), 4, -8, 8)
    wg = _dyadic(rng, (E, H), 8, -8, 8)
    bias = _dyadic(rng, (E,), 16, -16, 16)
    r = oracle.route(x.astype(dtype), wg.astype(dtype), bias, k)
    z = _exact_logits(x, wg, bias)
    for t in range(T):
        order = sorted(range(E), key=lambda e: (-z[t][e], e))
        assert list(r["idx"][t]) == order[:k]
        # Softmax over all experts then renormalising the selected k equals a
        # softmax over the k selected logits alone.
        sel = [float(z[t][e]) for e in order[:k]]
        m = max(sel)
        den = sum(math.exp(v - m) for v in sel)
        for j in range(k):
            assert abs(r["w"][t, j] - math.exp(sel[j] - m) / den) < 2e-6
        # and the full probability vector is the textbook softmax
        zf = [float(v) for v in z[t]]
        den_all = sum(math.exp(v - max(zf)) for v in zf)
        for e in range(E):
            assert abs(float(r["p"][t, e]) - math.exp(zf[e] - max(zf)) / den_all) < 1e-6


def test_weight_and_index_invariants(oracle):
    rng = np.random.default_rng(1)
    T, H, E, k = 300, 32, 8, 2
    x = rng.standard_normal((T, H)).astype(np.float32)
    wg = (rng.standard_normal((E, H)) / math.sqrt(H)).astype(np.float32)
    r = oracle.route(x, wg, None, k)
    assert np.all(np.abs(r["w"].sum(axis=1) - 1.0) < 1e-12)
    assert np.all(r["w"][:, 0] >= r["w"][:, 1])
    assert np.all(r["idx"] >= 0) and np.all(r["idx"] < E)
    assert np.all(r["idx"][:, 0] != r["idx"][:, 1])
    assert np.all(np.abs(r["p"].sum(axis=1) - 1.0) < 1e-5)
    # selected probabilities are the largest ones
    top = np.sort(r["p"], axis=1)[:, ::-1][:, :k]
    got = np.take_along_axis(r["p"], r["idx"], axis=1)
    assert np.array_equal(top, got)


def test_zero_input_routes_by_bias_alone(oracle):
    E, H, k = 8, 16, 2
    x = np.zeros((3, H), dtype=np.float32)
    wg = np.ones((E, H), dtype=np.float32)
    bias = np.array([0.0, 0.5, -1.0, 2.0, 0.25, 2.0, -3.0, 1.0])
    r = oracle.route(x, wg, bias, k)
    # largest bias is 2.0 at experts 3 and 5: the tie goes to the lower index first
    assert np.all(r["idx"] == np.array([3, 5]))
    assert np.allclose(r["w"], 0.5, atol=1e-12)
    r = oracle.route(x, wg, None, k)
    assert np.all(r["idx"] == np.array([0, 1]))
    bias2 = np.array([0.0, 1.0, 3.0, -1.0, 0.0, 0.0, 0.0, 0.0])
    r = oracle.route(x, wg, bias2, k)
    assert np.all(r["idx"] == np.array([2, 1]))
    w0 = math.exp(3.0) / (math.exp(3.0) + math.exp(1.0))
    assert np.allclose(r["w"][:, 0], w0, atol=1e-6) and np.allclose(r["w"][:, 1], 1 - w0, atol=1e-6)


def test_gate_is_not_transposed_and_bias_is_added(oracle):
    # One-hot gate rows: logit e is x[:, col[e]]; a transposed or mis-strided gate picks other columns.
    H, E = 6, 4
    col = [5, 0, 3, 1]
    wg = np.zeros((E, H), dtype=np.float64)
    for e, c in enumerate(col):
        wg[e, c] = 1.0
    x = np.array([[0.0, 4.0, 9.0, 2.0, 9.0, 1.0]])  # logits: [1, 0, 2, 4]
    r = oracle.route(x, wg, None, 2)
    assert list(r["idx"][0]) == [3, 2]
    r = oracle.route(x, wg, np.array([10.0, 0.0, 0.0, 0.0]), 2)  # logits: [11, 0, 2, 4]
    assert list(r["idx"][0]) == [0, 3]


def test_expert_permutation_equivariance(oracle):
    rng = np.random.default_rng(2)
    T, H, E, k = 64, 24, 8, 2
    x = rng.standard_normal((T, H))
    wg = rng.standard_normal((E, H)) / math.sqrt(H)
    bias = rng.standard_normal(E)
    perm = rng.permutation(E)  # new expert i is old expert perm[i]
    a = oracle.route(x, wg, bias, k)
    b = oracle.route(x, wg[perm], bias[perm], k)
    assert np.array_equal(perm[b["idx"]], a["idx"])
    assert np.array_equal(b["counts"], a["counts"][perm])
    assert np.array_equal(a["w"], b["w"])


def test_counts_invariants(oracle):
    rng = np.random.default_rng(3)
    T, H, E, k = 257, 16, 8, 2
    x = rng.standard_normal((T, H)).astype(np.float32)
    wg = rng.standard_normal((E, H)).astype(np.float32)
    r = oracle.route(x, wg, None, k)
    assert r["counts"].sum() == T * k
    assert np.all(r["counts"] <= T)
    assert np.array_equal(r["counts"], np.bincount(r["idx"].ravel(), minlength=E))
    shuffled = oracle.route(x[rng.permutation(T)], wg, None, k)
    assert np.array_equal(shuffled["counts"], r["counts"])
    acc = r["counts"].copy()
    oracle.route(x, wg, None, k, counts=acc)
    assert np.array_equal(acc, 2 * r["counts"])
    empty = oracle.route(x[:0], wg, None, k)
    assert empty["counts"].sum() == 0 and empty["idx"].shape == (0, k)


@pytest.mark.parametrize("k", [1, 2, 4, 6])
def test_margin_is_smallest_deciding_gap(oracle, k):
    rng = np.random.default_rng(4)
    T, H, E = 50, 8, 6
    x = rng.standard_normal((T, H))
    wg = rng.standard_normal((E, H))
    r = oracle.route(x, wg, None, k)
    ps = np.sort(r["p"], axis=1)[:, ::-1]
    gaps = ps[:, :-1] - ps[:, 1:]
    last = k if k < E else E - 1
    assert np.array_equal(r["margin"], gaps[:, :last].min(axis=1))


def test_prediction_is_the_next_gate_on_the_same_hidden_state(oracle):
    rng = np.random.default_rng(5)
    T, H, E, k = 20000, 32, 8, 2
    x = rng.standard_normal((T, H)).astype(np.float32)
    wg = rng.standard_normal((E, H)).astype(np.float32)
    wg_next = rng.standard_normal((E, H)).astype(np.float32)
    cur = oracle.route(x, wg, None, k)
    pred = oracle.predict_next(x, wg_next, None, k)
    assert np.array_equal(pred["idx"], oracle.route(x, wg_next, None, k)["idx"])
    same = oracle.predict_next(x, wg, None, k)
    assert np.array_equal(same["idx"], cur["idx"])
    # Independent gates: the predicted pair equals the actual pair with probability 1 / C(8,2).
    hit = np.mean(np.all(np.sort(pred["idx"], 1) == np.sort(cur["idx"], 1), axis=1))
    p0 = 1.0 / 28.0
    assert abs(hit - p0) < 5 * math.sqrt(p0 * (1 - p0) / T)


def test_zipf_bias_gives_the_documented_skew(oracle):
    import torch
    from paper_2501_10375_amd import synth

    T, H, E = 8192, 256, 8
    x = synth.to_numpy(synth.normal((T, H), 0, synth.TID_X, 1.0, torch.float32))
    wg = synth.to_numpy(synth.normal((E, H), 0, synth.TID_WG, H ** -0.5, torch.float32))
    bias = synth.zipf_gate_bias(E, 1.2).numpy()
    r = oracle.route(x, wg, bias.astype(np.float64), 2)
    share = r["counts"] / r["counts"].sum()
    want = np.array([0.40, 0.24, 0.14, 0.085, 0.056, 0.039, 0.027, 0.020])
    assert np.all(np.abs(share - want) < 0.04), share


def test_bad_arguments_are_rejected(oracle):
    x = np.zeros((2, 4), dtype=np.float32)
    wg = np.zeros((3, 4), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.route(x, wg, None, 4)  # k > E
    with pytest.raises(TypeError):
        oracle.route(x, wg.astype(np.float64), None, 1)
