"""Pins for the oracle's expert execution with pre-calculated experts (Sec. IV-C): some selections
are evaluated on an earlier hidden state.  The paper gives no worked numbers, so the function is
pinned to the already pinned plain expert function through special cases and its linearity in the
combine weights, and to a library matmul on a single dense expert."""
import math

import numpy as np

from test_oracle_ffn import _dense_swiglu, _rand_layer


def _case(rng, T=7, H=10, F=14, E=5, k=3):
    x, wg, w1, w3, w2 = _rand_layer(rng, T, H, F, E)
    x_stale = x + 0.5 * rng.standard_normal((T, H))
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    w = rng.random((T, k))
    w /= w.sum(1, keepdims=True)
    stale = rng.random((T, k)) < 0.5
    stale[0] = [True, False, True][:k]      # one token with a mixed row for sure
    return x, x_stale, stale, idx, w, w1, w3, w2


def test_identical_inputs_make_the_mask_irrelevant(oracle):
    x, x_stale, stale, idx, w, w1, w3, w2 = _case(np.random.default_rng(40))
    want = oracle.expert_ffn(x, idx, w, w1, w3, w2)
    for mask in (stale, ~stale, np.zeros_like(stale), np.ones_like(stale)):
        got = oracle.expert_ffn_precalc(x, x.copy(), mask, idx, w, w1, w3, w2)
        assert np.allclose(got, want, rtol=1e-13, atol=1e-14)


def test_all_fresh_and_all_stale_reduce_to_the_plain_expert_function(oracle):
    x, x_stale, stale, idx, w, w1, w3, w2 = _case(np.random.default_rng(41))
    fresh = oracle.expert_ffn_precalc(x, x_stale, np.zeros_like(stale), idx, w, w1, w3, w2)
    old = oracle.expert_ffn_precalc(x, x_stale, np.ones_like(stale), idx, w, w1, w3, w2)
    assert np.allclose(fresh, oracle.expert_ffn(x, idx, w, w1, w3, w2), rtol=1e-13, atol=1e-14)
    assert np.allclose(old, oracle.expert_ffn(x_stale, idx, w, w1, w3, w2), rtol=1e-13, atol=1e-14)
    assert np.abs(fresh - old).max() > 1e-3   # the two inputs do differ


def test_mixed_mask_is_the_sum_of_the_two_weight_masked_runs(oracle):
    """The output is linear in the combine weights, so a mixed call equals the plain function on the
    fresh input with the stale selections' weights zeroed plus the plain function on the stale input
    with the fresh selections' weights zeroed.  The mask acts per selection, not per token."""
    x, x_stale, stale, idx, w, w1, w3, w2 = _case(np.random.default_rng(42))
    got = oracle.expert_ffn_precalc(x, x_stale, stale, idx, w, w1, w3, w2)
    want = oracle.expert_ffn(x, idx, np.where(stale, 0.0, w), w1, w3, w2) \
        + oracle.expert_ffn(x_stale, idx, np.where(stale, w, 0.0), w1, w3, w2)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-13)
    per_token = np.repeat(stale[:, :1], stale.shape[1], axis=1)
    other = oracle.expert_ffn_precalc(x, x_stale, per_token, idx, w, w1, w3, w2)
    mixed_rows = np.where((stale != per_token).any(1))[0]
    assert mixed_rows.size > 0 and np.abs(got[mixed_rows] - other[mixed_rows]).max() > 1e-4


def test_single_dense_expert_on_the_stale_input(oracle):
    rng = np.random.default_rng(43)
    x, wg, w1, w3, w2 = _rand_layer(rng, 6, 12, 20, 1)
    x_stale = rng.standard_normal(x.shape)
    idx = np.zeros((6, 1), dtype=np.int32)
    w = np.full((6, 1), 0.75)
    stale = np.array([[1], [0], [1], [1], [0], [0]], dtype=bool)
    got = oracle.expert_ffn_precalc(x, x_stale, stale, idx, w, w1, w3, w2)
    want = 0.75 * np.where(stale, _dense_swiglu(x_stale, w1[0], w3[0], w2[0]), _dense_swiglu(x, w1[0], w3[0], w2[0]))
    assert np.allclose(got, want, rtol=1e-12, atol=1e-13)


def test_token_subset_and_bf16_storage(oracle):
    rng = np.random.default_rng(44)
    x, x_stale, stale, idx, w, w1, w3, w2 = _case(rng, T=9)

    def bf16(a):   # keep the top 16 bits: exactly representable values, stored as bit patterns
        bits = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32) >> 16
        return bits.astype(np.uint16), (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)

    (xb, xf), (sb, sf), (b1, f1), (b3, f3), (b2, f2) = bf16(x), bf16(x_stale), bf16(w1), bf16(w3), bf16(w2)
    tok = [8, 0, 3]
    got = oracle.expert_ffn_precalc(xb, sb, stale, idx, w, b1, b3, b2, tokens=tok)
    want = oracle.expert_ffn_precalc(xf, sf, stale, idx, w, f1, f3, f2)[tok]
    assert np.array_equal(got, want)
