"""Helpers that compare the HIP library with the CPU oracle on the same seeded inputs.

Rules:
  * selected experts and activation counts must match the oracle bit-exactly, leaving out only
    tokens whose oracle top-k margin (smallest deciding gap of the fp32 probabilities) is below
    1e-4; those are counted and returned;
  * gate weights within 1e-5 absolute on compared tokens;
  * layer outputs: err = max |y - yhat| / max(|yhat|, rms(yhat)) <= 2e-2 (bf16) or 1e-4 (fp32),
    on tokens where both sides selected the same expert set.
"""
import numpy as np
import torch

from paper_2501_10375_amd import moe, synth

MARGIN = 1e-4
TOL = {torch.bfloat16: 2e-2, torch.float32: 1e-4}


def host(d):
    return {k: synth.to_numpy(v) for k, v in d.items()}


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def check_routing(idx_gpu, w_gpu, counts_gpu, ref, E, label=""):
    """ref = oracle.route(...) dict.  Returns (n_excluded, keep_mask)."""
    idx_gpu = idx_gpu.cpu().numpy()
    T, k = idx_gpu.shape
    keep = ref["margin"] >= MARGIN
    n_excl = int((~keep).sum())
    assert np.array_equal(idx_gpu[keep], ref["idx"][keep]), f"{label}: selected experts differ outside the margin set"
    assert idx_gpu.min(initial=0) >= 0 and idx_gpu.max(initial=0) < E
    if k > 1 and T > 0:
        srt = np.sort(idx_gpu, axis=1)
        assert np.all(srt[:, 1:] != srt[:, :-1]), f"{label}: duplicate expert for a token"
    if w_gpu is not None:
        w = w_gpu.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(w.sum(axis=1) - 1.0) < 1e-5)
        assert np.all(np.abs(w[keep] - ref["w"][keep]) < 1e-5), f"{label}: gate weights differ"
    if counts_gpu is not None:
        c = counts_gpu.cpu().numpy()
        assert c.sum() == T * k, f"{label}: counts do not sum to tokens*k"
        assert np.array_equal(c, np.bincount(idx_gpu.ravel(), minlength=E)), f"{label}: counts != histogram of idx"
        hist_gpu = np.bincount(idx_gpu[keep].ravel(), minlength=E)
        hist_ref = np.bincount(ref["idx"][keep].ravel(), minlength=E)
        assert np.array_equal(hist_gpu, hist_ref)
        assert np.abs(c - ref["counts"]).sum() <= 2 * k * n_excl
    return n_excl, keep


def output_error(y_gpu_rows: np.ndarray, y_ref_rows: np.ndarray) -> float:
    if y_ref_rows.size == 0:
        return 0.0
    rms = np.sqrt(np.mean(y_ref_rows ** 2))
    den = np.maximum(np.abs(y_ref_rows), rms)
    return float(np.max(np.abs(y_gpu_rows - y_ref_rows) / den))


def check_layer(oracle, d_gpu, shape, out, dtype, tokens=None, label="", predict=True):
    """Compare a finished moe_layer call (out = dict from moe.run_layer) with the oracle.

    tokens: the token subset on which y is compared (None = all)."""
    torch.cuda.synchronize()
    h = host(d_gpu)
    E, k = shape.n_experts, shape.top_k
    T = d_gpu["x"].shape[0]
    ref = oracle.route(h["x"], h["wg"], h["bias"], k)
    n_excl, keep = check_routing(out["idx"], out["w"], out["counts"], ref, E, label)
    n_excl_pred = 0
    if predict and out.get("pred_idx") is not None:
        pref = oracle.predict_next(h["x"], h["wg_next"], h["bias_next"], k)
        n_excl_pred, _ = check_routing(out["pred_idx"], None, None, pref, E, label + " (prediction)")
    tok = np.arange(T) if tokens is None else np.asarray(tokens)
    idx_gpu = out["idx"].cpu().numpy()
    same_set = np.all(np.sort(idx_gpu[tok], 1) == np.sort(ref["idx"][tok], 1), axis=1)
    tok = tok[same_set]
    # tokens where the GPU legitimately picked another set (near-ties) are skipped; the rest use the oracle's routing
    y_ref = oracle.expert_ffn(h["x"], ref["idx"], ref["w"], h["w1"], h["w3"], h["w2"], tokens=tok)
    y_gpu = to_f64(out["y"])[tok]
    err = output_error(y_gpu, y_ref)
    assert np.all(np.isfinite(y_gpu))
    assert err <= TOL[dtype], f"{label}: output error {err:.3e} > {TOL[dtype]:.0e}"
    return {"excluded": n_excl, "excluded_pred": n_excl_pred, "err": err, "compared_tokens": int(tok.size)}
