#!/usr/bin/env python3
"""Benchmark of the MoE layer on one MI355X.

A "step" is one moe_layer call (routing, counts, next-layer prediction, permute, grouped SwiGLU
experts, combine) on one batch of synthetic input that is already resident in HBM.  The headline
workload is the Mixtral-8x7B-shaped layer (Table III of the DAOP paper: hidden 4096, 8 experts of
FFN width 14336, top-2) at a 4096-token prefill; the same run also times decode calls of 1, 8 and 32 tokens and
the CPU oracle on the host cores.  One JSON line is printed.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E

WORKLOADS = {
    # name: (H, F, E, k, zipf_s, prefill_T, decode_T)
    "mixtral": dict(H=4096, F=14336, E=8, k=2, zipf=1.2),
    "phi": dict(H=4096, F=6400, E=16, k=2, zipf=1.5),
    # not a model of the paper: many small experts and top-6, to exercise the wide router and the
    # permute / grouped GEMM with 64 groups
    "finegrained": dict(H=2048, F=1408, E=64, k=6, zipf=0.5),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--model", default="mixtral", choices=sorted(WORKLOADS))
    ap.add_argument("--tokens", type=int, default=4096, help="tokens of the headline (prefill) workload")
    ap.add_argument("--decode-tokens", type=int, nargs="*", default=[1, 8, 32], help="decode batch sizes also timed")
    ap.add_argument("--prefill-tokens", type=int, nargs="*", default=[512, 2048],
                    help="other prefill lengths of the same layer also timed")
    ap.add_argument("--other-model", default="phi", choices=sorted(WORKLOADS) + [""],
                    help="second model shape also timed (prefill and decode); empty string to skip")
    ap.add_argument("--other-prefill", type=int, default=2048)
    ap.add_argument("--other-decode-tokens", type=int, nargs="*", default=[1])
    ap.add_argument("--with-stack", action="store_true", default=None,
                    help="also run the resident stack of layers (default: only in a run with no workload options)")
    ap.add_argument("--no-stack", dest="with_stack", action="store_false")
    ap.add_argument("--decode-layers", type=int, default=4,
                    help="distinct weight sets the decode loop rotates over (keeps the weights cold in cache)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="only run a plain device-to-device copy of this many MiB three times (reference for "
                         "scaling the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run) and exit")
    ap.add_argument("--cpu-sample", type=int, default=0, help="tokens the oracle is timed on (0 = pick for ~15 s)")
    ap.add_argument("--workload", default="layer", choices=["layer", "stack"],
                    help="layer: the headline single-layer benchmark; stack: a resident stack of layers, "
                         "one prefill then single-token decode steps (prints its own JSON line)")
    ap.add_argument("--stack-layers", type=int, default=32)
    ap.add_argument("--stack-prefill", type=int, default=1024)
    ap.add_argument("--stack-decode-steps", type=int, default=128)
    args = ap.parse_args()
    if args.with_stack is None:   # the stack leg belongs to the default headline run
        args.with_stack = args.model == "mixtral" and args.tokens == 4096 and args.workload == "layer"
    return args


def run_stack(args, brief=False):
    """32 resident Mixtral-shaped layers: prefill of one sequence, then decode steps of one token.
    brief: leave out the graph replay and the pre-calculation study (the default run's stack leg)."""
    import torch
    from paper_2501_10375_amd import moe, policy, stack, synth

    cfg = WORKLOADS[args.model]
    H, F, E, k = cfg["H"], cfg["F"], cfg["E"], cfg["k"]
    L, T, steps = args.stack_layers, args.stack_prefill, args.stack_decode_steps
    dev = "cuda:0"
    torch.cuda.set_device(0)
    st = stack.MoeStack(L, H, F, E, k, torch.bfloat16, dev, zipf_s=cfg["zipf"], max_tokens=max(T, 1))
    torch.cuda.synchronize()

    def timed(fn, calls):
        torch.cuda.synchronize()
        moe.moe_stage_timing_begin(calls)
        t0 = time.perf_counter()
        r = fn()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        stages = moe.moe_stage_timing_end()
        gpu_ms = sum(ms * n for ms, n in stages.values())
        return r, wall, gpu_ms

    h0 = synth.normal((T, H), 999, synth.TID_X, 1.0, torch.float32, dev)
    st.forward(h0, st.new_counts())   # warm-up
    prefill = st.new_counts()
    out, p_wall, p_gpu_ms = timed(lambda: st.forward(h0, prefill), L)
    exact, overlap = stack.agreement(out["pred"].clone(), out["idx"].clone())

    hs = [synth.normal((1, H), 1000 + s, synth.TID_X, 1.0, torch.float32, dev) for s in range(steps)]
    decode = st.new_counts()
    d_exact = torch.zeros(L - 1, dtype=torch.float64, device=dev)
    selections = torch.zeros((L, steps, k), dtype=torch.int32, device=dev)   # experts of every layer at every decode step

    def decode_loop():
        for i, h in enumerate(hs):
            o = st.forward(h, decode)
            e, _ = stack.agreement(o["pred"], o["idx"])
            d_exact.add_(e)
            selections[:, i] = o["idx"][:, 0]

    st.forward(hs[0], st.new_counts())
    _, d_wall, d_gpu_ms = timed(decode_loop, L * steps)
    dec_bytes = steps * L * (2 * 3.0 * H * F * 2)   # two experts per token and layer
    graph = None
    if not brief:
        # the same steps replayed from one HIP graph per step (no per-stage events inside a graph, so wall time only)
        graph_counts = st.new_counts()
        step = stack.CapturedStep(st, 1, graph_counts)
        step.h_in.copy_(hs[0])
        step.replay()
        graph_counts.zero_()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for h in hs:
            step.h_in.copy_(h)
            step.replay()
        torch.cuda.synchronize()
        g_wall = time.perf_counter() - t0
        graph = {"wall_ms": g_wall * 1e3, "tokens_per_s_wall": steps / g_wall, "GBps_wall": dec_bytes / g_wall / 1e9,
                 "frac_of_hbm_peak_wall": dec_bytes / g_wall / 1e9 / PEAK_HBM_GBS,
                 "counts_equal_eager_run": bool(torch.equal(graph_counts, decode))}
    P, D = prefill[:, :E].contiguous(), decode[:, :E].contiguous()
    sim, per = policy.daop_similarity(P, D)
    win_mean, win_pairs = policy.daop_window_variation(selections, E, 15)   # Sec. VI-B: 15-token decode windows
    cache = policy.daop_memory_init(D, (L * E * 15) // 32)      # expert cache ratio 46.875 %
    resident_before = (P * cache.int()).sum().item() / P.sum().item()
    _, n_swaps = policy.daop_plan_swaps(P, cache)
    resident_after = (P * cache.int()).sum().item() / P.sum().item()
    # what DAOP's decode approximation (predicted experts, stale inputs for experts outside the cache) does to the
    # output of the synthetic stack, by expert cache ratio: cache from the decode counts, then Algorithm 1 on the
    # prefill counts
    hq = torch.cat(hs[:8], dim=0)
    exact_h = st.forward(hq, st.new_counts())["h"].clone()
    precalc = []
    for ecr in (() if brief else (0.25, 0.46875, 0.75, 1.0)):
        c = policy.daop_memory_init(D, int(round(ecr * L * E)))
        policy.daop_plan_swaps(P, c)
        r = stack.forward_precalc(st, hq, c, first_predicted_layer=5)
        precalc.append({"expert_cache_ratio": ecr, "stale_selections": r["stale_selections"],
                        "rel_err_final_hidden": ((r["h"] - exact_h).norm() / exact_h.norm()).item()})
    gave_up = moe.moe_decode_status(st.workspace)
    result = {
        "metric": "moe_stack_decode_tokens_per_s", "value": steps / (d_gpu_ms * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.model}_stack_{L}_layers_prefill_T{T}_then_{steps}_decode_steps", "layers": L,
                   "hidden": H, "ffn": F, "n_experts": E, "top_k": k, "weights_GB": st.weight_bytes() / 1e9,
                   "glue": "parameter-free RMS norm + residual in torch between the layers (stand-in for attention)"},
        "prefill": {"tokens": T, "moe_gpu_ms": p_gpu_ms, "wall_ms": p_wall * 1e3, "tokens_per_s_moe_gpu_time": T / (p_gpu_ms * 1e-3),
                    "tflops_moe_gpu_time": L * T * 12.0 * H * F / (p_gpu_ms * 1e-3) / 1e12},
        "decode": {"steps": steps, "moe_gpu_ms": d_gpu_ms, "wall_ms": d_wall * 1e3,
                   "tokens_per_s_moe_gpu_time": steps / (d_gpu_ms * 1e-3), "tokens_per_s_wall": steps / d_wall,
                   "graph_replay": graph, "rendezvous_gave_up": gave_up,
                   "GBps_moe_gpu_time": dec_bytes / (d_gpu_ms * 1e-3) / 1e9,
                   "frac_of_hbm_peak_moe_gpu_time": dec_bytes / (d_gpu_ms * 1e-3) / 1e9 / PEAK_HBM_GBS},
        "prediction_agreement": {"prefill_exact_set_mean": exact.mean().item(), "prefill_overlap_mean": overlap.mean().item(),
                                 "prefill_exact_set_layers_ge_4": exact[3:].mean().item() if L > 4 else None,
                                 "decode_exact_set_mean": (d_exact / steps).mean().item()},
        "eq1_similarity_prefill_vs_decode": sim.item(),
        "decode_window_variation": {"window_tokens": 15, "window_pairs": int(win_pairs.numel()),
                                    "mean_similarity_of_consecutive_windows": win_mean.item(),
                                    "min_pair": win_pairs.min().item() if win_pairs.numel() else None},
        "algorithm1": {"cache_slots": int(cache.sum().item()), "swaps": int(n_swaps.sum().item()),
                       "prefill_tokens_on_resident_experts_before": resident_before,
                       "prefill_tokens_on_resident_experts_after": resident_after},
        "precalculation_error_vs_cache_ratio": precalc,
        "prefill_counts_first_layers": P[:2].cpu().tolist(),
    }
    del st
    torch.cuda.empty_cache()
    return result


def time_steps(fn, steps, warmup):
    import torch

    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def stage_times(fn, steps):
    """Mean per-launch GPU time of each stage (HIP events on the launch stream), over `steps` calls."""
    import torch
    from paper_2501_10375_amd import moe

    torch.cuda.synchronize()
    moe.moe_stage_timing_begin(steps)
    for _ in range(steps):
        fn()
    return moe.moe_stage_timing_end()


def kernel_source_digest():
    """Short hash of the kernel sources: a stored traffic figure is only quoted for the sources it was measured on."""
    import hashlib

    h = hashlib.sha256()
    base = os.path.join(ROOT, "paper_2501_10375_amd", "csrc")
    for name in sorted(os.listdir(base)):
        with open(os.path.join(base, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def read_traffic(key):
    """Per-launch HBM bytes of a kernel from the committed rocprofv3 --pmc summary.  Counters cannot be read from
    inside this process, so the figure is a stored one: it is returned together with where it comes from, and only
    if the kernel sources are still the ones it was measured on (otherwise null, with the reason)."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            t = json.load(f)
    except (OSError, ValueError):
        return None, "no profiles/traffic.json"
    if key not in t:
        return None, "no counter run stored for this kernel and workload"
    src = f"{t.get('_source', 'profiles/')} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, measured separately; not read in this run)"
    if t.get("_kernel_source_digest") != kernel_source_digest():
        return None, "stored figure is for other kernel sources: " + src
    return t[key], src


def prefill_leg(model, T, steps, warmup, d=None):
    """One prefill-size moe_layer workload (counts and prediction on): timing, per-stage kernel times, both
    roofline fractions of the layer and the roofline of its dominant kernel (the first grouped GEMM)."""
    import torch
    from paper_2501_10375_amd import moe, synth

    cfg = WORKLOADS[model]
    H, F, E, k = cfg["H"], cfg["F"], cfg["E"], cfg["k"]
    dev, dtype = "cuda:0", torch.bfloat16
    shape = moe.make_shape(H, F, E, k, dtype)
    if d is None:
        d = synth.moe_layer_inputs(T, H, F, E, dtype, dev, seed=0, zipf_s=cfg["zipf"], with_next=True)
    elif d["x"].shape[0] != T:
        d = dict(d, x=synth.normal((T, H), 0, synth.TID_X, 1.0, dtype, dev))
    out = moe.LayerOutputs(shape, T, dtype, dev, predict=True)

    def step():
        moe.run_layer(shape, d, out)

    sec = time_steps(step, steps, warmup)
    st = stage_times(step, steps)
    counts = out.counts.cpu().tolist()
    A = T * k
    active = sum(1 for c in counts if c > 0)
    flops_layer = T * (12.0 * H * F + 2 * 2.0 * H * E)
    # bytes: each active expert's weights once, x in, y out, the bf16 intermediate written and read
    bytes_layer = active * 3.0 * H * F * 2 + 2.0 * T * H * 2 + 2.0 * A * F * 2
    t_mfma, t_hbm = flops_layer / (PEAK_BF16_TFLOPS * 1e12), bytes_layer / (PEAK_HBM_GBS * 1e9)
    flops_gemm1 = 4.0 * A * H * F
    bytes_gemm1 = active * 2.0 * H * F * 2 + A * H * 2.0 + A * F * 2.0
    g1_ms = st["gemm1"][0]
    mfma_bound = flops_gemm1 / (PEAK_BF16_TFLOPS * 1e12) >= bytes_gemm1 / (PEAK_HBM_GBS * 1e9)
    key = f"{model}_prefill_T{T}_gemm1"
    traffic, traffic_source = read_traffic(key)
    if mfma_bound:
        ach = flops_gemm1 / (g1_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": "grouped_gemm_bf16<gemm1+swiglu>", "achieved": ach, "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "traffic": traffic, "traffic_source": traffic_source,
                    "kernel_ms": g1_ms, "algorithmic_flops_per_launch": flops_gemm1}
    else:
        ach = bytes_gemm1 / (g1_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "grouped_gemm_bf16<gemm1+swiglu>", "achieved": ach, "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": ach / PEAK_HBM_GBS, "traffic": traffic, "traffic_source": traffic_source,
                    "kernel_ms": g1_ms, "algorithmic_bytes_per_launch": bytes_gemm1,
                    "frac_of_mfma_peak": flops_gemm1 / (g1_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
    leg = {
        "workload": f"{model}_layer_prefill_T{T}_bf16_top{k}_with_counts_and_prediction", "tokens": T,
        "value": T / sec, "unit": "tokens/s", "ms_per_step": sec * 1e3, "steps": steps,
        "layer_tflops": flops_layer / sec / 1e12, "layer_frac_of_mfma_peak": flops_layer / sec / 1e12 / PEAK_BF16_TFLOPS,
        "layer_GBps": bytes_layer / sec / 1e9, "layer_frac_of_hbm_peak": bytes_layer / sec / 1e9 / PEAK_HBM_GBS,
        "layer_bound": "mfma" if t_mfma >= t_hbm else "hbm", "layer_frac_of_bound": max(t_mfma, t_hbm) / sec,
        "active_experts": active, "counts": counts,
        "stage_ms": {name: round(v[0], 5) for name, v in st.items() if v[1] > 0}, "roofline": roofline,
    }
    return leg, d, out


def decode_leg(model, Td, steps, warmup, layers):
    """Decode-size moe_layer calls (no prediction) rotating over distinct weight sets so the weights stay cold."""
    import torch
    from paper_2501_10375_amd import moe, synth

    cfg = WORKLOADS[model]
    H, F, E, k = cfg["H"], cfg["F"], cfg["E"], cfg["k"]
    dev, dtype = "cuda:0", torch.bfloat16
    shape = moe.make_shape(H, F, E, k, dtype)
    xs = synth.normal((Td, H), 1000, synth.TID_X, 1.0, dtype, dev)
    outs = moe.LayerOutputs(shape, Td, dtype, dev, predict=False)
    calls = [dict(L, x=xs, wg_next=None, bias_next=None) for L in layers]
    prepared = [moe.PreparedLayerCall(shape, c, outs, predict=False) for c in calls]  # arguments marshalled once
    state = {"i": 0}

    def dstep():
        prepared[state["i"] % len(prepared)]()
        state["i"] += 1

    n = max(steps, 4 * len(calls))
    dsec = time_steps(dstep, n, max(warmup, len(calls)))
    state["i"] = 0
    dst = stage_times(dstep, n)
    distinct = []   # distinct experts hit, per weight set (the routing differs per set)
    for c in calls:
        moe.run_layer(shape, c, outs, predict=False)
        distinct.append(int((outs.counts > 0).sum().item()))
    gave_up = moe.moe_decode_status(outs.workspace)
    Dm = sum(distinct) / len(distinct)
    bytes_layer = Dm * 3.0 * H * F * 2 + 2 * Td * H * 2 + E * H * 2
    bytes_kernel = Dm * 3.0 * H * F * 2  # the one kernel of a decode call streams all three matrices
    g1 = dst["fused"][0]
    traffic, traffic_source = read_traffic(f"{model}_decode_T{Td}_layer")
    return {
        "workload": f"{model}_layer_decode_T{Td}_bf16", "tokens": Td, "value": Td / dsec,
        "unit": "tokens/s", "ms_per_step": dsec * 1e3, "steps": n, "weight_sets": len(calls),
        "distinct_experts_mean": Dm, "layer_GBps": bytes_layer / dsec / 1e9,
        "layer_frac_of_hbm_peak": bytes_layer / dsec / 1e9 / PEAK_HBM_GBS, "rendezvous_gave_up": gave_up,
        "stage_ms": {name: round(v[0], 5) for name, v in dst.items() if v[1] > 0},
        "roofline": {"bound": "hbm", "kernel": "decode_layer_kernel",
                     "achieved": bytes_kernel / (g1 * 1e-3) / 1e9 if g1 > 0 else None,
                     "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": bytes_kernel / (g1 * 1e-3) / 1e9 / PEAK_HBM_GBS if g1 > 0 else None,
                     "traffic": traffic, "traffic_source": traffic_source, "kernel_ms": g1,
                     "algorithmic_bytes_per_launch": bytes_kernel},
    }


def weight_sets(model, first, n):
    import torch
    from paper_2501_10375_amd import synth

    cfg = WORKLOADS[model]
    return [first] + [synth.moe_layer_inputs(1, cfg["H"], cfg["F"], cfg["E"], torch.bfloat16, "cuda:0", seed=s,
                                             zipf_s=cfg["zipf"], with_next=False) for s in range(1, max(1, n))]


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures ONE MI355X: this build has no multi-GPU path (no sharding, no collectives); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    if args.copy_calibration > 0:
        n = args.copy_calibration << 20
        src = torch.full((n,), 7, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": n, "copy_calibration_bytes_written": n, "copies": 3}))
        return
    from paper_2501_10375_amd import moe, synth

    moe.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.workload == "stack":
        print(json.dumps(run_stack(args)))
        return
    torch.cuda.set_device(0)
    cfg = WORKLOADS[args.model]
    H, F, E, k = cfg["H"], cfg["F"], cfg["E"], cfg["k"]
    T = args.tokens

    # ---- headline: prefill of one sequence, with counts and next-layer prediction ----------------
    head, d, out = prefill_leg(args.model, T, args.steps, args.warmup)
    result = {
        "metric": "moe_layer_tokens_per_s", "value": head["value"], "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": head["workload"], "hidden": H, "ffn": F, "n_experts": E, "top_k": k, "tokens": T,
                   "gate_bias": f"zipf({cfg['zipf']})", "counts": head["counts"]},
        "layer_tflops": head["layer_tflops"], "layer_frac_of_mfma_peak": head["layer_frac_of_mfma_peak"],
        "stage_ms": head["stage_ms"], "roofline": head["roofline"],
    }

    # ---- context for the MFMA roofline: what a register-only MFMA loop reaches on this board, with
    # operands that never change (full clock) and with random ones (power-limited clock).  The
    # roofline's `peak` stays the published 2.5 PFLOP/s; these two are measured, a few ms each.
    probe = {name: moe.moe_calibrate_mfma(rnd) for name, rnd in (("constant_operands", False), ("random_operands", True))}
    result["mfma_probe"] = {"unit": "TFLOP/s", **{name: round(v["tflops"], 1) for name, v in probe.items()},
                            "shader_clock_GHz": {name: round(v["ghz"], 3) for name, v in probe.items()}}
    if head["roofline"]["bound"] == "mfma":
        result["mfma_probe"]["gemm1_frac_of_random_operand_rate"] = head["roofline"]["achieved"] / probe["random_operands"]["tflops"]

    # ---- the other prefill lengths of the same layer (shorter ones move from the MFMA bound to the HBM bound)
    result["prefill"] = []
    for Tp in args.prefill_tokens:
        if Tp != T:
            result["prefill"].append(prefill_leg(args.model, Tp, args.steps, args.warmup, d)[0])

    # ---- decode: a few tokens per call, weights cold (rotate over distinct weight sets) -----------
    decode = []
    if args.decode_tokens:
        layers = weight_sets(args.model, d, args.decode_layers)
        for Td in args.decode_tokens:
            decode.append(decode_leg(args.model, Td, args.steps, args.warmup, layers))
        del layers
    result["decode"] = decode
    # ---- context for the HBM roofline: a plain read stream over one weight tensor of the layer (0.94 GB for the
    # Mixtral shape).  The roofline's `peak` stays the published 8 TB/s; this one is measured.
    stream_probe = moe.moe_calibrate_read_stream(d["w1"])
    result["hbm_probe"] = {"unit": "GB/s", "read_stream": round(stream_probe["GBps"], 1), "bytes": stream_probe["bytes"]}
    if decode:
        result["hbm_probe"]["decode_frac_of_read_stream"] = decode[0]["roofline"]["achieved"] / stream_probe["GBps"]

    # ---- the CPU oracle on this machine's host cores, on a bounded sample of the headline workload ----
    if not args.no_cpu_baseline:
        from oracle import moe_oracle

        h = {key: synth.to_numpy(v) for key, v in d.items()}
        threads = moe_oracle.num_threads()
        t0 = time.perf_counter()
        ref = moe_oracle.route(h["x"], h["wg"], h["bias"], k)
        moe_oracle.predict_next(h["x"], h["wg_next"], h["bias_next"], k)
        t_route = time.perf_counter() - t0  # all T tokens, both gates
        n = args.cpu_sample
        if n <= 0:
            probe = list(range(0, T, max(1, T // threads)))[:threads]
            t0 = time.perf_counter()
            moe_oracle.expert_ffn(h["x"], ref["idx"], ref["w"], h["w1"], h["w3"], h["w2"], tokens=probe)
            per_batch = time.perf_counter() - t0
            n = int(max(threads, min(T, threads * round(15.0 / max(per_batch, 1e-3)))))
        sample = [int(i * T / n) for i in range(n)]
        t0 = time.perf_counter()
        moe_oracle.expert_ffn(h["x"], ref["idx"], ref["w"], h["w1"], h["w3"], h["w2"], tokens=sample)
        t_ffn = time.perf_counter() - t0
        per_token = t_route / T + t_ffn / n
        result["cpu_baseline"] = {
            "value": 1.0 / per_token, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"routing + prediction on all {T} tokens ({t_route:.2f} s), expert FFN + combine on {n} evenly "
                      f"spaced tokens ({t_ffn:.2f} s); fp64 C oracle, OpenMP over tokens",
        }
        del h, ref
    del d, out
    torch.cuda.empty_cache()

    # ---- the second model shape of the paper (Table III): Phi-3.5-MoE-shaped, 16 experts, stronger skew
    if args.other_model and args.other_model != args.model:
        om = args.other_model
        leg, od, oout = prefill_leg(om, args.other_prefill, args.steps, args.warmup)
        other = {"model": om, "prefill": [leg], "decode": []}
        layers = weight_sets(om, od, args.decode_layers)
        for Td in args.other_decode_tokens:
            other["decode"].append(decode_leg(om, Td, args.steps, args.warmup, layers))
        del layers, od, oout
        torch.cuda.empty_cache()
        result["other_model"] = other

    # ---- the resident stack of layers (one prefill, then single-token decode steps)
    if args.with_stack:
        free, _ = torch.cuda.mem_get_info()
        need = args.stack_layers * E * 3 * H * F * 2 + (6 << 30)
        if free >= need:
            result["stack"] = run_stack(args, brief=True)
        else:
            result["stack"] = {"skipped": f"needs {need >> 30} GiB of free device memory, {free >> 30} GiB available"}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
