"""Strength of the oracle's pins: planted mistakes must not survive them.

Each case below rewrites one expression of the oracle's C source (a dropped term, a wrong sign or
index, a swapped operand, a missing normalisation), compiles the result into a temporary library
and runs the pin tests of test_oracle_route.py / test_oracle_ffn.py against it.  The unmodified
source has to pass all of them; every planted mistake has to fail at least one.  Everything here
runs on the CPU and touches only the oracle.
"""
import importlib.util
import inspect
import os

import numpy as np
import pytest

import test_oracle_ffn as pins_ffn
import test_oracle_precalc as pins_precalc
import test_oracle_route as pins_route

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "moe_oracle.c")
WRAPPER = os.path.join(ROOT, "oracle", "moe_oracle.py")

# (name, text in the source, what a mistaken author might have written instead)
MUTANTS = [
    ("gate bias dropped", "if (bias) z += bias[e];", ""),
    ("gate row of another expert", "dot_row(wg, dtype, (size_t)e * H, xt, H)", "dot_row(wg, dtype, (size_t)(E - 1 - e) * H, xt, H)"),
    ("equal probabilities go to the higher index", "p32[order[pos - 1]] < p32[e]", "p32[order[pos - 1]] <= p32[e]"),
    ("experts sorted ascending", "p32[order[pos - 1]] < p32[e]", "p32[order[pos - 1]] > p32[e]"),
    ("top-k weights not renormalised", "(double)p32[order[j]] / wsum;", "(double)p32[order[j]];"),
    ("softmax of the negated logits", "p32[e] = (float)(exp((double)z32[e] - (double)zmax) / denom);",
     "p32[e] = (float)(exp((double)zmax - (double)z32[e]) / denom);"),
    ("softmax without its denominator", "p32[e] = (float)(exp((double)z32[e] - (double)zmax) / denom);",
     "p32[e] = (float)(exp((double)z32[e] - (double)zmax));"),
    ("only the first selection counted", "counts[idx[(size_t)t * k + j]] += 1;", "counts[idx[(size_t)t * k + j]] += (j == 0);"),
    ("margin ignores the gap that decides the set", "int last = (k < E) ? k : E - 1;", "int last = k - 1;"),
    ("margin is the largest gap", "if (gap < m) m = gap;", "if (gap > m || r == 0) m = gap;"),
    ("silu with the wrong sign", "a[f] = g / (1.0 + exp(-g)) * u;", "a[f] = g / (1.0 + exp(g)) * u;"),
    ("gate and up projections swapped", "a[f] = g / (1.0 + exp(-g)) * u;", "a[f] = u / (1.0 + exp(-u)) * g;"),
    ("activation without the up projection", "a[f] = g / (1.0 + exp(-g)) * u;", "a[f] = g / (1.0 + exp(-g));"),
    ("w3 read from w1", "double u = dot_row(w3, dtype, row, xt, H);", "double u = dot_row(w1, dtype, row, xt, H);"),
    ("w2 indexed as its transpose", "size_t row = ((size_t)e * H + h) * (size_t)F;", "size_t row = (size_t)e * H * F + h;"),
    ("combine weight dropped", "+= wj * dot_row(w2, dtype, row, a, F);", "+= dot_row(w2, dtype, row, a, F);"),
    ("second selection overwrites the first", "+= wj * dot_row(w2, dtype, row, a, F);", "= wj * dot_row(w2, dtype, row, a, F);"),
    ("every selection uses the first expert", "int e = idx[(size_t)t * k + j];", "int e = idx[(size_t)t * k];"),
    ("every selection uses the first weight", "double wj = w[(size_t)t * k + j];", "double wj = w[(size_t)t * k];"),
    ("token list ignored", "int t = tokens ? tokens[i] : i;", "int t = i;"),
    ("pre-calculation: stale mask inverted", "const void *source = stale[sel] ? x_stale : x;",
     "const void *source = stale[sel] ? x : x_stale;"),
    ("pre-calculation: mask of the token's first selection used for all", "const void *source = stale[sel] ? x_stale : x;",
     "const void *source = stale[(size_t)t * k] ? x_stale : x;"),
    ("pre-calculation: stale selections dropped", "yt[h] += w[sel] * dot_row(", "yt[h] += (stale[sel] ? 0.0 : w[sel]) * dot_row("),
    ("pre-calculation: up projection read from w1", "double up = dot_row(w3, dtype, wrow, in, H);",
     "double up = dot_row(w1, dtype, wrow, in, H);"),
    ("pre-calculation: silu on the up projection", "hid[f] = gate / (1.0 + exp(-gate)) * up;", "hid[f] = up / (1.0 + exp(-up)) * gate;"),
    ("pre-calculation: combine weight of the first selection", "yt[h] += w[sel] * dot_row(", "yt[h] += w[(size_t)t * k] * dot_row("),
    ("bf16 widened with the wrong shift", "uint32_t bits = (uint32_t)r[i] << 16;", "uint32_t bits = (uint32_t)r[i] << 15;"),
    ("fp32 rows read with half the stride", "const float *r = (const float *)mat + row_offset;",
     "const float *r = (const float *)mat + row_offset / 2;"),
]


def _load_oracle(src_path, lib_path, tag):
    """The oracle's Python wrapper, bound to another C source and library file."""
    spec = importlib.util.spec_from_file_location(f"moe_oracle_{tag}", WRAPPER)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod._SRC, mod._LIB, mod._lib = src_path, lib_path, None
    mod.build(force=True)
    return mod


def _pin_calls():
    """Every pin test of the two oracle test files as a zero-argument-but-oracle callable."""
    calls = []
    for module in (pins_route, pins_ffn, pins_precalc):
        for name, fn in sorted(vars(module).items()):
            if not name.startswith("test_") or not inspect.isfunction(fn):
                continue
            if name in ("test_tiny_config_runs_in_seconds", "test_bad_arguments_are_rejected",
                        "test_zipf_bias_gives_the_documented_skew"):
                continue  # timing, argument checks and the input recipe: not about the arithmetic
            params = [n for n in inspect.signature(fn).parameters if n != "oracle"]
            if not params:
                calls.append((name, lambda o, fn=fn: fn(o)))
            elif name == "test_topk_bruteforce_on_dyadic_inputs":
                for dtype in (np.float32, np.float64):
                    for shape in ((8, 16, 8, 2), (5, 7, 6, 3), (3, 4, 2, 1), (4, 9, 5, 5)):
                        calls.append((f"{name}[{dtype.__name__}-{shape}]",
                                      lambda o, fn=fn, dtype=dtype, shape=shape: fn(o, dtype, *shape)))
            elif name == "test_margin_is_smallest_deciding_gap":
                for k in (1, 2, 4, 6):
                    calls.append((f"{name}[{k}]", lambda o, fn=fn, k=k: fn(o, k)))
            else:
                raise AssertionError(f"pin {name} takes parameters this file does not know: {params}")
    return calls


def _failing_pins(oracle_module):
    failed = []
    for name, call in _pin_calls():
        try:
            call(oracle_module)
        except AssertionError:
            failed.append(name)
        except Exception as exc:  # a planted mistake may also make a pin crash on a bad value
            failed.append(f"{name} ({type(exc).__name__})")
    return failed


def test_unmodified_source_passes_every_pin(tmp_path):
    mod = _load_oracle(SRC, str(tmp_path / "libmoe_oracle_copy.so"), "copy")
    assert _failing_pins(mod) == []


def test_every_planted_text_occurs_in_the_source():
    text = open(SRC).read()
    for name, old, _ in MUTANTS:
        assert text.count(old) >= 1, f"{name}: the source no longer contains {old!r}"


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0].replace(" ", "_") for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    text = open(SRC).read()
    assert old in text
    src = tmp_path / "moe_oracle_mutant.c"
    src.write_text(text.replace(old, new))
    mod = _load_oracle(str(src), str(tmp_path / "libmoe_oracle_mutant.so"), "mutant")
    failed = _failing_pins(mod)
    assert failed, f"planted mistake survived every pin: {name}"


# ---- the policy oracle (Python): same idea, the planted text goes through exec() ----
import types

import test_oracle_policy as pins_policy

POLICY_SRC = os.path.join(ROOT, "oracle", "daop_policy.py")

POLICY_MUTANTS = [
    # (a swap number above E / 2 can never bind: the shorter of the two lists has at most E / 2 entries)
    ("swap number is a quarter of the experts", "swap_num = E // 2", "swap_num = E // 4"),
    ("swap needs strictly more than the threshold", ">= float(swap_in_out) * float(counts[c])", "> float(swap_in_out) * float(counts[c])"),
    ("threshold ignored", ">= float(swap_in_out) * float(counts[c])", ">= float(counts[c])"),
    ("least active off-GPU experts taken as hot", "key=lambda e: (-counts[e], e))[:swap_num]", "key=lambda e: (counts[e], e))[:swap_num]"),
    ("most active on-GPU experts taken as cold", "key=lambda e: (counts[e], e))[:swap_num]", "key=lambda e: (-counts[e], e))[:swap_num]"),
    ("idle experts may be swapped in", "if counts[h] > 0 and float(counts[h])", "if float(counts[h])"),
    ("cold expert stays on the GPU", "            new[c] = False\n", ""),
    ("cosine without the square roots", "dot / (math.sqrt(pp) * math.sqrt(dd))", "dot / (pp * dd)"),
    ("similarity summed, not averaged", "return total / L, per_layer", "return total, per_layer"),
    ("similarity of a layer with itself only", "dot += P[l, e] * D[l, e]", "dot += P[l, e] * P[l, e]"),
    ("uniform share divided by the expert count", "per_layer = slots // L", "per_layer = slots // E"),
    ("leftover slots by raw count", "if n1 * d2 > n2 * d1:", "if n1 > n2:"),
    ("leftover slots: later entry wins ties", "if n1 * d2 > n2 * d1:", "if n1 * d2 >= n2 * d1:"),
    ("degradation drops the best expert", "sel = sel[:-1] + [rest[0]]", "sel = sel[1:] + [rest[0]]"),
    ("degradation whenever any expert is off the GPU", "if not any(on_gpu[e] for e in sel):", "if not all(on_gpu[e] for e in sel):"),
    ("degradation takes the worst on-GPU expert", "sel = sel[:-1] + [rest[0]]", "sel = sel[:-1] + [rest[-1]]"),
    ("windows overlap by one step", "for step in range(v * window, (v + 1) * window):", "for step in range(v * window, (v + 1) * window + 1):"),
    ("windows compared with the first one", "similarity(patterns[v], patterns[v + 1])[0]", "similarity(patterns[0], patterns[v + 1])[0]"),
    ("only the first selection of a step counted", "for j in range(k):\n                    counts[l, int(idx[l, step, j])] += 1", "for j in range(1):\n                    counts[l, int(idx[l, step, j])] += 1"),
    ("shorter tail kept as a window", "n_windows = S // window", "n_windows = -(-S // window)"),
    ("variation summed, not averaged", "(total / per_pair.shape[0] if per_pair.shape[0] > 0 else 0.0)", "total"),
    ("degraded weights not renormalised", "return sel, [probs[e] / s for e in sel]", "return sel, [probs[e] for e in sel]"),
]


def _policy_module(text, tag):
    mod = types.ModuleType(f"daop_policy_{tag}")
    exec(compile(text, f"<daop_policy {tag}>", "exec"), mod.__dict__)
    return mod


def _failing_policy_pins(mod, monkeypatch):
    monkeypatch.setattr(pins_policy, "pol", mod)
    calls = []
    for name, fn in sorted(vars(pins_policy).items()):
        if not name.startswith("test_") or not inspect.isfunction(fn):
            continue
        if name == "test_algorithm1_hand_worked_cases":
            for i, case in enumerate(pins_policy._cases()):
                args = case.values if hasattr(case, "values") else case
                calls.append((f"{name}[{i}]", lambda fn=fn, args=args: fn(*args)))
        else:
            assert not inspect.signature(fn).parameters, f"pin {name} takes parameters this file does not know"
            calls.append((name, fn))
    failed = []
    for name, call in calls:
        try:
            call()
        except AssertionError:
            failed.append(name)
        except Exception as exc:
            failed.append(f"{name} ({type(exc).__name__})")
    return failed


def test_unmodified_policy_source_passes_every_pin(monkeypatch):
    assert _failing_policy_pins(_policy_module(open(POLICY_SRC).read(), "copy"), monkeypatch) == []


@pytest.mark.parametrize("name,old,new", POLICY_MUTANTS, ids=[m[0].replace(" ", "_") for m in POLICY_MUTANTS])
def test_planted_policy_mistake_is_caught(monkeypatch, name, old, new):
    text = open(POLICY_SRC).read()
    assert old in text, f"{name}: the source no longer contains {old!r}"
    failed = _failing_policy_pins(_policy_module(text.replace(old, new), "mutant"), monkeypatch)
    assert failed, f"planted mistake survived every pin: {name}"
