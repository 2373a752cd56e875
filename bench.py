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
# HBM-side traffic per launch of each GEMM class on workload 3, in bytes, mean over the class's 4 launches per
# step: rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE runs of this script (KiB per dispatch), each scaled by
# what the same counter reads for a plain 512 MiB device copy (FETCH_SIZE reads half the bytes copied: x2;
# WRITE_SIZE reads them all: x1).  FETCH_SIZE counts what the eight L2s request from the fabric, whether it
# is then served by the memory-side cache or by HBM.  A hardware counter cannot be read from inside this
# process, so the figures are carried here and re-measured whenever the GEMM kernel changes.
MEASURED_TRAFFIC_CONFIG3 = {
    "gemm_nt": (2 * (836756.3 + 395602.7) / 2 + (274581.4 + 65570.4) / 2) * 1024,
    "gemm_nn": (2 * 610691.7 + 93211.0) * 1024,
    # four full-round kernels per step, plus the K-cut last round of the 22016 x 4096 gradient and its reduction
    "gemm_tn": (2 * (4 * 594075.2 + 82077.6 + 24590.7) + 4 * 95750.2 + 77382.6 + 12288.0) / 4 * 1024,
}
PAPER_CONTEXT = "paper: 54.7% MFU, 72B MLLM on 1172 GPUs (abstract; Section 7.1) -- other hardware, whole system"


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
    return {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": f"first {n} segments ({Ts} of {int(cu[-1])} tokens) of the same pack, fp64 numpy, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
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
    cu, modes, kinds = wl.make_segments(args.config, seed)
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
    names = ["gemm_nt", "gemm_nn", "gemm_tn", "attn_fwd", "attn_bwd"]
    # shader-clock and 100 MHz counters at the start and end of the first workgroup of the last bf16 GEMM launch
    clock_probe = torch.zeros(4, dtype=torch.int64, device="cuda")

    def timed_pass(steps, class_mask):
        """`steps` steps with HIP events around the launches of the classes in class_mask; wall time per step and the
        event-timed duration per step of each class."""
        for k in range(5):
            mm.mmtrain_profile_read(k, reset=True)
        mm.mmtrain_profile_enable(class_mask)
        mm.mmtrain_profile_gemm_clock(clock_probe)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            check(runner.forward(), "mmtrain_layer_fwd")
            check(runner.backward(), "mmtrain_layer_bwd")
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        mm.mmtrain_profile_enable(0)
        mm.mmtrain_profile_gemm_clock(None)
        res = {}
        for k, name in enumerate(names):
            ms, n = mm.mmtrain_profile_read(k, reset=True)
            res[name] = {"ms_per_step": ms / steps, "launches_per_step": n / steps}
        return dt * 1e3 / steps, res

    # Breakdown pass (untimed for the headline): every class bracketed by events.  It names the dominant GEMM class;
    # the timed region then carries events around that class only (36 event pairs per step cost about 1 % of the step).
    _, prof = timed_pass(max(3, min(args.steps, 10)), mm.PROF_ALL)
    dom = max(("gemm_nt", "gemm_nn", "gemm_tn"), key=lambda n: prof[n]["ms_per_step"])
    ms_per_step, timed = timed_pass(args.steps, 1 << names.index(dom))
    prof[dom] = timed[dom]                       # the dominant class's figures come from the timed region itself
    tflops = flops["fwd_bwd"] / (ms_per_step * 1e-3) / 1e12

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
    dom_launches = max(prof[dom]["launches_per_step"], 1)
    roofline = {"bound": "mfma", "kernel": dom, "achieved": kernels[dom]["tflops"], "peak": peak, "unit": "TFLOP/s",
                "frac": (kernels[dom]["tflops"] or 0.0) / peak,
                "avg_launch_ms": kernels[dom]["ms_per_step"] / dom_launches,
                "flops_per_launch": gf[{"gemm_nt": "NT", "gemm_nn": "NN", "gemm_tn": "TN"}[dom]] / dom_launches,
                "traffic": MEASURED_TRAFFIC_CONFIG3[dom] if args.config == 3 else None,
                "traffic_unit": "bytes per launch (L2 <-> fabric, rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated)",
                "algorithmic_bytes_per_launch": gemm_bytes_by_layout(shape, T) / dom_launches}

    out = {
        "metric": "layer fwd+bwd TFLOP/s and % bf16 MFMA peak on packed multimodal microbatch",
        "value": tflops, "unit": "TFLOP/s", "pct_of_peak": 100.0 * tflops / peak, "peak_tflops": peak,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if shape.dtype == wl.BF16 else "f32", "data": "synthetic",
        "config": {"workload": f"config {args.config}: {shape.name}", "seed": int(seed), "total_tokens": T,
                   "n_segments": int(len(cu) - 1), "max_segment": int(np.diff(cu).max()),
                   "hidden": shape.hidden, "heads": f"{shape.n_heads}/{shape.n_kv_heads}x{shape.head_dim}",
                   "ffn_hidden": shape.ffn_hidden, "model_tflop_per_step": flops["fwd_bwd"] / 1e12,
                   "attention_share": 3 * flops["attn_fwd"] / flops["fwd_bwd"]},
        "roofline": roofline, "kernels": kernels,
        "kernels_note": f"{dom}: events inside the timed region; the others: untimed breakdown pass before it",
        # the clock a compute unit sustained during the last GEMM launch of the timed region (the published peak is quoted at 2400 MHz)
        "gemm_shader_clock_mhz": mm.gemm_clock_mhz(clock_probe),
        "context": PAPER_CONTEXT,
    }
    if not args.no_cpu_baseline:
        del runner
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(shape, cu, modes, W, seed, args.cpu_sample_tokens)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
