"""CPU oracle for the count-driven policy steps of DAOP (test infrastructure, not a product path).

Plain Python / numpy in fp64 and exact integers, written from the paper:

  * similarity        - Eq. 1 (Sec. III, observation 2): mean over layers of the cosine similarity
                        between the prefill and decode activation rows.
  * plan_swaps        - Algorithm 1 (Sec. IV-B), the expert-cache update of one block.
  * memory_init       - Sec. IV-A, the calibrated initial expert cache.
  * degrade_selection - Sec. IV-C "Graceful Degradation", index substitution given a placement.

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
