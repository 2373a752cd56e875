#!/usr/bin/env python3
"""Benchmark: forward + backward of one transformer layer over a packed multimodal microbatch.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--seed 0] [--no-cpu-baseline]

One step = mmtrain_layer_fwd + mmtrain_layer_bwd (all weight gradients) on one synthetic pack that is
already resident in HBM.  Prints ONE JSON line: throughput in model TFLOP/s (GEMMs 2*T*K*N forward and
twice that backward; attention 4*d per unmasked (query, key) pair per head forward, 8*d backward), the
fraction of the MI355X dense bf16 MFMA peak, a roofline object for the dominant kernel (durations from
HIP events recorded inside the timed region on the launch stream, around that kernel class only; the other
classes' durations in "kernels" come from a short untimed pass in front of it, with events around every
class), and the fp64 oracle timed on the host cores on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak (published)
PEAK_F32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E peak (published)
PAPER_CONTEXT = "paper: 54.7% MFU, 72B MLLM on 1172 GPUs (abstract; Section 7.1) -- other hardware, whole system"
# HBM-side traffic of the GEMM classes on workload 3 is a hardware-counter figure (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE,
# KiB per dispatch, scaled by what the same counters read for a plain copy).  A counter cannot be read from inside this
# process, so the figure is carried over from the committed summary of those runs and labelled as such.
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "layer_config3_hbm_traffic.txt")


def read_traffic_profile(path=TRAFFIC_PROFILE):
    """Mean bytes per launch of each GEMM class (4 launches per step) from the counter summary's table: per kernel
    FETCH_SIZE x 2 (the counter reads half the bytes fetched, per the copy calibration in the file) + WRITE_SIZE, in
    KiB per dispatch, times its dispatches; the K-cut tail kernel and its reduction belong to the weight-gradient
    class.  None if the file is missing or has no table."""
    import re
    try:
        lines = open(path).read().splitlines()
    except OSError:
        return None
    rows = {}
    for ln in lines:
        m = re.match(r"^(\S.*?)\s{2,}([0-9.]+)\s+([0-9.]+)\s+(\d+)\b", ln)
        if m:
            rows[m.group(1).strip()] = (float(m.group(2)), float(m.group(3)), int(m.group(4)))
    steps = next((n for k, (_, _, n) in rows.items() if k.startswith("attn_fwd")), 0)
    if not steps:
        return None
    cls = {"gemm_nt": 0.0, "gemm_nn": 0.0, "gemm_tn": 0.0}
    for k, (fetch, write, n) in rows.items():
        kib = (2.0 * fetch + write) * n
        if k.startswith("gemm_mfma_kernel<true, true"):
            cls["gemm_nt"] += kib
        elif k.startswith("gemm_mfma_kernel<true, false"):
            cls["gemm_nn"] += kib
        elif k.startswith("gemm_mfma_kernel<false, false") or k.startswith("tail_reduce_kernel"):
            cls["gemm_tn"] += kib
    return {k: v * 1024.0 / (4 * steps) for k, v in cls.items()}


def gemm_flops_by_layout(shape, T):
    """Model FLOPs of the layer's GEMMs per launch class (forward = NT, input grads = NN, weight grads = TN)."""
    per = 2.0 * T * (shape.nqkv * shape.hidden + shape.hidden * shape.nq + shape.fc1_rows * shape.hidden
                     + shape.hidden * shape.ffn_hidden)
    return {"NT": per, "NN": per, "TN": per}


def gemm_bytes_by_layout(shape, T):
    """Algorithmic bytes of one launch class: every operand read once, every output written once (bf16),
    plus the residual the forward projections add.  The three classes touch the same tensors in different
    roles, so the sum is the same for each up to the residual reads."""
    H, F = shape.hidden, shape.ffn_hidden
    weights = shape.nqkv * H + H * shape.nq + shape.fc1_rows * H + H * F
    acts = T * (H + shape.nqkv) + T * (shape.nq + H) + T * (H + shape.fc1_rows) + T * (F + H)
    return 2.0 * (weights + acts)


def cpu_baseline(shape, cu, modes, W, seed, target_tokens):
    """Time the fp64 oracle (forward + backward) on the leading segments of the pack, about `target_tokens` tokens."""
    from oracle import layer_oracle as orc
    from paper_2408_04275_amd import workloads as wl
    n = 1
    while n < len(cu) - 1 and cu[n] < target_tokens:
        n += 1
    sub_cu, sub_modes = cu[:n + 1].copy(), modes[:n]
    Ts = int(sub_cu[-1])
    x, dy = wl.make_activations(shape, Ts, seed)
    threads = os.cpu_count()
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        pass
    t0 = time.perf_counter()
    y, cache = orc.layer_fwd(shape.kind, shape.n_heads, shape.n_kv_heads, shape.head_dim, sub_cu, sub_modes, W, x,
                             eps=shape.norm_eps, rope_base=shape.rope_base)
    orc.layer_bwd(W, cache, dy)
    dt = time.perf_counter() - t0
    fl = wl.model_flops(shape, sub_cu, sub_modes)["fwd_bwd"]
    model, physical = cpu_identity()
    return {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "implementation": "fp64 numpy; matrix products through numpy's BLAS, everything else plain numpy",
            "cpu_model": model, "physical_cores": physical, "logical_cpus": os.cpu_count(),
            "sample": f"first {n} segments ({Ts} of {int(cu[-1])} tokens) of the same pack, forward + backward, {dt:.1f} s"}


def cpu_identity():
    """(model name, number of physical cores) from /proc/cpuinfo; (None, None) where it cannot be read."""
    try:
        text = open("/proc/cpuinfo").read()
    except OSError:
        return None, None
    model, cores = None, set()
    phys = core = None
    for ln in text.splitlines() + [""]:
        key, _, val = ln.partition(":")
        key, val = key.strip(), val.strip()
        if key == "model name" and model is None:
            model = val
        elif key == "physical id":
            phys = val
        elif key == "core id":
            core = val
        elif not ln.strip():
            if core is not None:
                cores.add((phys, core))
            phys = core = None
    return model, (len(cores) or None)


def hbm_kernel_bytes(shape, T):
    """Algorithmic bytes per step of the memory-bound kernel classes (every tensor a kernel has to read or write, once;
    bf16 activations, fp32 statistics): the figures the achieved GB/s of those kernels are quoted on."""
    H, F, F1 = shape.hidden, shape.ffn_hidden, shape.fc1_rows
    e = 2 if shape.dtype == 1 else 4
    A = T * H * e
    enc = shape.kind == 1
    rope_cols = (shape.n_heads + shape.n_kv_heads) * shape.head_dim
    return {
        "norm_fwd": 2 * (2 * A + 2 * T * 4),                                 # two launches: read x, write h, statistics
        "norm_bwd": 2 * (4 * A + 2 * T * 4),                                 # two launches: read d_out, x, d_res, write d_in
        "rope": 0 if enc else 2 * T * rope_cols * e + T * shape.head_dim * 4,   # q and k in place + the (cos, sin) table
        "act_fwd": T * (F1 + F) * e,                                         # read the pre-activation, write m
        "act_bwd": T * (F + 2 * F1) * e,                                     # read d_m and the pre-activation, write its gradient
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5, 6])
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of a HIP graph that holds one forward + backward (no per-kernel figures)")
    ap.add_argument("--cpu-sample-tokens", type=int, default=8192,
                    help="the oracle is timed on the leading segments of the pack up to about this many tokens (default: the whole 8192-token pack, 10-15 s)")
    ap.add_argument("--layers", type=int, default=1,
                    help="more than 1: time a stack of that many layers through mmtrain_stack_fwd / mmtrain_stack_bwd")
    ap.add_argument("--group", choices=["span", "sample"], default="span",
                    help="decoder workloads: 'span' = every text run / image span is a document of its own (default); 'sample' = "
                         "the whole 8192-token sequence is one causal document")
    ap.add_argument("--seed-sweep", type=int, default=None,
                    help="also time the layer on the packs of seeds 0 .. N-1 of the workload's generator (20 steps each) and report "
                         "median and range over the packs; default 5 for workload 3, 0 otherwise")
    ap.add_argument("--recompute", action="store_true",
                    help="with --layers: keep only layer inputs in forward and recompute each layer in backward")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU (one GPU's share of the training step); run with --gpus 1")

    import torch
    from paper_2408_04275_amd import binding as mm
    from paper_2408_04275_amd import workloads as wl
    from paper_2408_04275_amd.harness import LayerRunner, StackRunner, check

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    mm.load_library()                                   # fails loudly if the HIP library is missing

    shape = wl.SHAPES[args.config]
    seed = args.seed if args.seed is not None else (wl.longtail_seed() if args.config == 4 else 0)
    cu, modes, kinds = wl.make_segments(args.config, seed, group=args.group)
    T = int(cu[-1])
    W = wl.make_weights(shape, seed)
    x, dy = wl.make_activations(shape, T, seed)
    flops = wl.model_flops(shape, cu, modes)
    if args.layers > 1:
        # a stack: model FLOP = layers x one layer's; recomputation runs every layer's forward but the last twice,
        # which the model FLOP count (and so the reported rate) does not credit
        stack = StackRunner(shape, [W] + [wl.make_weights(shape, seed + 100 * l) for l in range(1, args.layers)], cu, modes,
                            recompute=args.recompute)
        stack.set_inputs(x, dy)
        for _ in range(args.warmup):
            stack.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            stack.step()
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
        print(json.dumps({"metric": "layer-stack fwd+bwd TFLOP/s (model FLOP)",
                          "value": args.layers * flops["fwd_bwd"] / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1,
                          "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
                          "dtype": "bf16" if shape.dtype == wl.BF16 else "f32", "data": "synthetic",
                          "config": {"workload": f"config {args.config}: {shape.name}", "layers": args.layers,
                                     "recompute": bool(args.recompute), "ctx_bytes": stack.ctx_bytes,
                                     "workspace_bytes": stack.ws_bytes}}))
        return
    runner = LayerRunner(shape, W, cu, modes)
    runner.set_inputs(x, dy)

    for _ in range(args.warmup):
        runner.step()
    torch.cuda.synchronize()
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            st = torch.cuda.current_stream().cuda_stream
            check(runner.forward(st), "mmtrain_layer_fwd")
            check(runner.backward(0, st), "mmtrain_layer_bwd")
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        ms_per_step = dt * 1e3 / args.steps
        print(json.dumps({"metric": "layer fwd+bwd TFLOP/s (HIP graph replay)", "value": flops["fwd_bwd"] / (ms_per_step * 1e-3) / 1e12,
                          "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
                          "higher_is_better": True, "dtype": "bf16" if shape.dtype == wl.BF16 else "f32", "data": "synthetic",
                          "config": {"workload": f"config {args.config}: {shape.name}", "graph": True}}))
        return
    names = ["gemm_nt", "gemm_nn", "gemm_tn", "attn_fwd", "attn_bwd", "norm_fwd", "norm_bwd", "rope", "act_fwd", "act_bwd"]
    # shader-clock and 100 MHz counters at the start and end of the first workgroup of the last bf16 GEMM launch
    clock_probe = torch.zeros(4, dtype=torch.int64, device="cuda")

    def timed_pass(steps, class_mask):
        """`steps` steps with HIP events around the launches of the classes in class_mask and one event at every
        step's start, between its forward and backward call and at its end (on the stream the library launches on).
        Returns wall time per step, the event-timed duration per step of each class, and per step (forward ms,
        backward ms)."""
        for k in range(len(names)):
            mm.mmtrain_profile_read(k, reset=True)
        mm.mmtrain_profile_enable(class_mask)
        mm.mmtrain_profile_gemm_clock(clock_probe)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(2 * steps + 1)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        marks[0].record()
        for i in range(steps):
            check(runner.forward(), "mmtrain_layer_fwd")
            marks[2 * i + 1].record()
            check(runner.backward(), "mmtrain_layer_bwd")
            marks[2 * i + 2].record()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        mm.mmtrain_profile_enable(0)
        mm.mmtrain_profile_gemm_clock(None)
        res = {}
        for k, name in enumerate(names):
            ms, n = mm.mmtrain_profile_read(k, reset=True)
            res[name] = {"ms_per_step": ms / steps, "launches_per_step": n / steps}
        per_step = [(marks[2 * i].elapsed_time(marks[2 * i + 1]), marks[2 * i + 1].elapsed_time(marks[2 * i + 2]))
                    for i in range(steps)]
        return dt * 1e3 / steps, res, per_step

    # Breakdown pass (untimed for the headline): every class bracketed by events.  It names the dominant GEMM class;
    # the timed region then carries events around that class only (an event pair costs a few microseconds on the stream).
    # It also keeps the matrix cores busy for tens of milliseconds right in front of the timed region, so that the timed
    # steps run at the clock the chip sustains rather than on its way there.
    n_breakdown = max(3, min(args.steps, 10))
    breakdown_ms, prof, _ = timed_pass(n_breakdown, mm.PROF_ALL)
    dom = max(("gemm_nt", "gemm_nn", "gemm_tn"), key=lambda n: prof[n]["ms_per_step"])
    ms_per_step, timed, per_step = timed_pass(args.steps, 1 << names.index(dom))
    prof[dom] = timed[dom]                       # the dominant class's figures come from the timed region itself
    tflops = flops["fwd_bwd"] / (ms_per_step * 1e-3) / 1e12
    step_ms = np.array([f + b for f, b in per_step])
    fwd_ms = np.array([f for f, _ in per_step])
    bwd_ms = np.array([b for _, b in per_step])

    gf = gemm_flops_by_layout(shape, T)
    peak = PEAK_BF16_TFLOPS if shape.dtype == wl.BF16 else PEAK_F32_TFLOPS
    kernels = {}
    for name, key in (("gemm_nt", "NT"), ("gemm_nn", "NN"), ("gemm_tn", "TN")):
        ms = prof[name]["ms_per_step"]
        kernels[name] = {"tflops": gf[key] / (ms * 1e-3) / 1e12 if ms > 0 else None, "ms_per_step": ms,
                         "launches_per_step": prof[name]["launches_per_step"]}
    af, ab = prof["attn_fwd"]["ms_per_step"], prof["attn_bwd"]["ms_per_step"]
    kernels["attn_fwd"] = {"tflops": flops["attn_fwd"] / (af * 1e-3) / 1e12 if af > 0 else None, "ms_per_step": af}
    kernels["attn_bwd"] = {"tflops": 2 * flops["attn_fwd"] / (ab * 1e-3) / 1e12 if ab > 0 else None, "ms_per_step": ab}
    # the memory-bound kernels: algorithmic bytes over event-timed duration, against the 8 TB/s HBM peak
    hb = hbm_kernel_bytes(shape, T)
    for name in ("norm_fwd", "norm_bwd", "rope", "act_fwd", "act_bwd"):
        ms, n = prof[name]["ms_per_step"], prof[name]["launches_per_step"]
        if n > 0 and ms > 0:
            gbs = hb[name] / (ms * 1e-3) / 1e9
            kernels[name] = {"gb_per_s": gbs, "frac_of_hbm_peak": gbs / PEAK_HBM_GBS, "ms_per_step": ms,
                             "launches_per_step": n, "algorithmic_bytes_per_step": hb[name]}
    dom_launches = max(prof[dom]["launches_per_step"], 1)
    traffic = read_traffic_profile() if args.config == 3 and args.group == "span" else None
    roofline = {"bound": "mfma", "kernel": dom, "achieved": kernels[dom]["tflops"], "peak": peak, "unit": "TFLOP/s",
                "frac": (kernels[dom]["tflops"] or 0.0) / peak,
                "avg_launch_ms": kernels[dom]["ms_per_step"] / dom_launches,
                "flops_per_launch": gf[{"gemm_nt": "NT", "gemm_nn": "NN", "gemm_tn": "TN"}[dom]] / dom_launches,
                "traffic": traffic[dom] if traffic else None,
                "traffic_unit": "bytes per launch (L2 <-> fabric, rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated)",
                "traffic_source": "carried over from profiles/layer_config3_hbm_traffic.txt (separate rocprofv3 --pmc runs of "
                                  "this script), not measured in this run" if traffic else None,
                "algorithmic_bytes_per_launch": gemm_bytes_by_layout(shape, T) / dom_launches}
    hw = wl.hardware_flops(shape, cu, modes) if shape.dtype == wl.BF16 else None

    out = {
        "metric": "layer fwd+bwd TFLOP/s and % bf16 MFMA peak on packed multimodal microbatch",
        "value": tflops, "unit": "TFLOP/s", "pct_of_peak": 100.0 * tflops / peak, "peak_tflops": peak,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        # per-step figures from events on the launch stream inside the timed region (ms_per_step is wall time / steps)
        "median_ms": float(np.median(step_ms)), "min_ms": float(step_ms.min()), "max_ms": float(step_ms.max()),
        "fwd_ms": {"median": float(np.median(fwd_ms)), "min": float(fwd_ms.min())},
        "bwd_ms": {"median": float(np.median(bwd_ms)), "min": float(bwd_ms.min())},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if shape.dtype == wl.BF16 else "f32", "data": "synthetic",
        "config": {"workload": f"config {args.config}: {shape.name}", "seed": int(seed), "total_tokens": T,
                   "n_segments": int(len(cu) - 1), "max_segment": int(np.diff(cu).max()), "document": args.group,
                   "hidden": shape.hidden, "heads": f"{shape.n_heads}/{shape.n_kv_heads}x{shape.head_dim}",
                   "ffn_hidden": shape.ffn_hidden, "model_tflop_per_step": flops["fwd_bwd"] / 1e12,
                   # what the matrix cores execute: + score recomputation in backward, masked parts of diagonal and
                   # boundary blocks, head-dimension padding (never credited in `value`)
                   "hardware_tflop_per_step": hw["fwd_bwd"] / 1e12 if hw else None,
                   "attention_share": 3 * flops["attn_fwd"] / flops["fwd_bwd"]},
        "roofline": roofline, "kernels": kernels,
        "kernels_note": f"{dom}: events inside the timed region; the others: untimed breakdown pass of {n_breakdown} steps "
                        f"({breakdown_ms:.3f} ms per step with all events) right before it",
        # the clock a compute unit sustained during the last GEMM launch of the timed region (the published peak is quoted at 2400 MHz)
        "gemm_shader_clock_mhz": mm.gemm_clock_mhz(clock_probe),
        "context": PAPER_CONTEXT,
    }
    # The same layer on other packs of the workload's generator: the step time depends on the pack through attention.
    n_sweep = args.seed_sweep if args.seed_sweep is not None else (5 if args.config == 3 and args.seed is None else 0)
    if n_sweep > 0 and args.config != 4:
        del runner
        torch.cuda.empty_cache()
        pcts, mss = [], []
        for sd in range(n_sweep):
            cu_s, modes_s, _ = wl.make_segments(args.config, sd, group=args.group)
            r = LayerRunner(shape, W, cu_s, modes_s)
            r.set_inputs(*wl.make_activations(shape, int(cu_s[-1]), sd))
            for _ in range(3):
                r.step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(20):
                r.step()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / 20
            mss.append(ms)
            pcts.append(100.0 * wl.model_flops(shape, cu_s, modes_s)["fwd_bwd"] / (ms * 1e-3) / 1e12 / peak)
            del r
        out["seed_sweep"] = {"seeds": list(range(n_sweep)), "steps_each": 20, "ms_per_step": mss, "pct_of_peak": pcts,
                             "median_pct": float(np.median(pcts)), "min_pct": float(min(pcts)), "max_pct": float(max(pcts))}
        runner = None
    if not args.no_cpu_baseline:
        del runner
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(shape, cu, modes, W, seed, args.cpu_sample_tokens)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
