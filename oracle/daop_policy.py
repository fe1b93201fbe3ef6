"""CPU oracle for the count-driven policy steps of DAOP (test infrastructure, not a product path).

Plain Python / numpy in fp64 and exact integers, written from the paper:

  * similarity        - Eq. 1 (Sec. III, observation 2): mean over layers of the cosine similarity
                        between the prefill and decode activation rows.
  * plan_swaps        - Algorithm 1 (Sec. IV-B), the expert-cache update of one block.
  * memory_init       - Sec. IV-A, the calibrated initial expert cache.
  * degrade_selection - Sec. IV-C "Graceful Degradation", index substitution given a placement.
  * window_variation  - Sec. VI-B "Limitation & Future Work": how much a sequence's activation
                        pattern changes while it is decoded, measured on 15-token windows.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.  It
shares no code with the HIP path.

Readings where the paper is silent (listed in the design notes as well):
  - Eq. 1: a row whose norm is zero in either matrix contributes cosine 0.
  - Algorithm 1: SwapNum = floor(0.5 * E); "most active" / "least active" ties go to the lower
    expert index; the hot and cold lists are paired in rank order and the shorter list decides the
    number of pairs; a pair is swapped when hot >= SwapInOut * cold AND hot > 0 (two idle experts
    are never exchanged); the comparison is made on token counts in fp64 (dividing both sides by
    the number of tokens would not change it).
  - Memory initialisation: every layer first gets floor(slots / L) experts, the ones with the most
    calibration tokens (ties: lower index); the remaining slots (fewer than L) go to the
    not-yet-resident experts with the highest activation frequency = tokens of that expert divided
    by the tokens of its layer, compared exactly as cross products (ties: lower layer, then lower
    expert).  A layer with no calibration tokens has frequency 0 for all its experts.
  - Graceful degradation (top-k, stated for k = 2 in the paper): if ALL selected experts are
    off-GPU, the selected expert with the lowest score is replaced by the best-scoring expert that
    is on the GPU (ties: lower index); with no expert on the GPU the selection is kept.  The
    weights are the selected experts' probabilities renormalised to sum to one; the list stays in
    descending probability.
  - Windowed variation (Sec. VI-B names the quantity and the window of 15 tokens, nothing more):
    the decode steps of a sequence are cut into consecutive windows of `window` tokens (a shorter
    tail is left out); each window gives an L x E matrix of activation counts, exactly like D in
    Eq. 1; the variation measure is the Eq. 1 similarity of each window with the next one, and
    their mean over the sequence.  Fewer than two whole windows: no pair, the mean is 0.
"""
from __future__ import annotations

import math

import numpy as np


def similarity(P, D):
    """Eq. 1.  P, D: [L, E] activation counts or probabilities.  Returns (mean, per_layer[L])."""
    P = np.asarray(P, dtype=np.float64)
    D = np.asarray(D, dtype=np.float64)
    assert P.shape == D.shape and P.ndim == 2
    L, E = P.shape
    per_layer = np.zeros(L, dtype=np.float64)
    for l in range(L):
        dot = 0.0
        pp = 0.0
        dd = 0.0
        for e in range(E):
            dot += P[l, e] * D[l, e]
            pp += P[l, e] * P[l, e]
            dd += D[l, e] * D[l, e]
        if pp > 0.0 and dd > 0.0:
            per_layer[l] = dot / (math.sqrt(pp) * math.sqrt(dd))
    total = 0.0
    for l in range(L):
        total += per_layer[l]
    return total / L, per_layer


def plan_swaps(counts, on_gpu, swap_in_out=1.05):
    """Algorithm 1 for one block.  counts[E] tokens per expert, on_gpu[E] booleans.
    Returns (swaps, new_on_gpu): swaps is a list of (hot_expert_in, cold_expert_out)."""
    counts = [int(c) for c in counts]
    on_gpu = [bool(b) for b in on_gpu]
    E = len(counts)
    swap_num = E // 2
    cpu = [e for e in range(E) if not on_gpu[e]]
    gpu = [e for e in range(E) if on_gpu[e]]
    hot = sorted(cpu, key=lambda e: (-counts[e], e))[:swap_num]   # most active first
    cold = sorted(gpu, key=lambda e: (counts[e], e))[:swap_num]   # least active first
    swaps = []
    new = list(on_gpu)
    for h, c in zip(hot, cold):
        if counts[h] > 0 and float(counts[h]) >= float(swap_in_out) * float(counts[c]):
            swaps.append((h, c))
            new[h] = True
            new[c] = False
    return swaps, new


def plan_swaps_all(counts, on_gpu, swap_in_out=1.05):
    """Algorithm 1 over all blocks.  counts, on_gpu: [L, E].  Returns (list of per-layer swap lists, new mask)."""
    counts = np.asarray(counts)
    on_gpu = np.asarray(on_gpu).astype(bool)
    out = np.zeros_like(on_gpu)
    swaps = []
    for l in range(counts.shape[0]):
        s, new = plan_swaps(counts[l], on_gpu[l], swap_in_out)
        swaps.append(s)
        out[l] = new
    return swaps, out


def memory_init(calib_counts, slots):
    """Sec. IV-A.  calib_counts[L, E] decode-phase calibration counts, slots = GPU expert slots in total.
    Returns on_gpu[L, E] (bool)."""
    calib = np.asarray(calib_counts).astype(np.int64)
    L, E = calib.shape
    slots = max(0, min(int(slots), L * E))
    per_layer = slots // L
    mask = np.zeros((L, E), dtype=bool)
    for l in range(L):
        order = sorted(range(E), key=lambda e: (-int(calib[l, e]), e))
        for e in order[:per_layer]:
            mask[l, e] = True
    left = slots - per_layer * L
    # frequency of (l, e) as an exact fraction num / den; a layer without tokens has frequency 0
    def freq(l, e):
        r = int(calib[l].sum())
        return (int(calib[l, e]), r) if r > 0 else (0, 1)
    for _ in range(left):
        best = None
        for l in range(L):
            for e in range(E):
                if mask[l, e]:
                    continue
                if best is None:
                    best = (l, e)
                    continue
                n1, d1 = freq(l, e)
                n2, d2 = freq(*best)
                if n1 * d2 > n2 * d1:   # strictly greater: earlier (layer, expert) wins ties
                    best = (l, e)
        if best is None:
            break
        mask[best] = True
    return mask


def degrade_selection(probs, k, on_gpu):
    """Graceful degradation for one token.  probs[E] gate probabilities, on_gpu[E].
    Returns (idx list of k experts in descending probability, weights list)."""
    probs = [float(p) for p in probs]
    on_gpu = [bool(b) for b in on_gpu]
    E = len(probs)
    order = sorted(range(E), key=lambda e: (-probs[e], e))
    sel = order[:k]
    if not any(on_gpu[e] for e in sel):
        rest = [e for e in order[k:] if on_gpu[e]]
        if rest:
            sel = sel[:-1] + [rest[0]]   # drop the lowest score, take the best expert on the GPU
            sel = sorted(sel, key=lambda e: (-probs[e], e))
    s = 0.0
    for e in sel:
        s += probs[e]
    return sel, [probs[e] / s for e in sel]


def window_variation(idx, n_experts, window=15):
    """Sec. VI-B.  idx: int [L, S, k], the experts every layer selected at each of S decode steps of
    one sequence.  Returns (mean similarity of consecutive windows, per_pair[S // window - 1])."""
    idx = np.asarray(idx)
    assert idx.ndim == 3 and window >= 1
    L, S, k = idx.shape
    n_windows = S // window
    patterns = []
    for v in range(n_windows):
        counts = np.zeros((L, n_experts), dtype=np.int64)
        for l in range(L):
            for step in range(v * window, (v + 1) * window):
                for j in range(k):
                    counts[l, int(idx[l, step, j])] += 1
        patterns.append(counts)
    per_pair = np.zeros(max(n_windows - 1, 0), dtype=np.float64)
    for v in range(n_windows - 1):
        per_pair[v] = similarity(patterns[v], patterns[v + 1])[0]
    total = 0.0
    for v in range(per_pair.shape[0]):
        total += per_pair[v]
    return (total / per_pair.shape[0] if per_pair.shape[0] > 0 else 0.0), per_pair
