"""Operator microbenchmarks through the C-ABI: time one GEMM or one attention call in isolation.

    python -m paper_2408_04275_amd.opbench gemm --layout nt --m 8192 --n 22016 --k 4096 [--iters 20]
    python -m paper_2408_04275_amd.opbench attn --config 3 [--iters 20]
    python -m paper_2408_04275_amd.opbench copy --mb 512          (a plain copy kernel, for counter calibration)

Prints one JSON line per run.  Meant to be run alone or under rocprofv3 (kernel trace or --pmc).
"""
import argparse
import json
import sys
import time

import numpy as np
import torch

from . import binding as mm
from . import workloads as wl
from .harness import check


def _time(fn, iters, warmup=3):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def bench_gemm(a):
    layout = {"nt": mm.GEMM_NT, "nn": mm.GEMM_NN, "tn": mm.GEMM_TN}[a.layout]
    M, N, K = a.m, a.n, a.k
    shp_a = (K, M) if layout == mm.GEMM_TN else (M, K)
    shp_b = (N, K) if layout == mm.GEMM_NT else (K, N)
    g = torch.Generator(device="cuda").manual_seed(0)
    A = torch.randn(shp_a, device="cuda", generator=g).to(torch.bfloat16)
    B = (torch.randn(shp_b, device="cuda", generator=g) * 0.02).to(torch.bfloat16)
    Cm = torch.empty((M, N), device="cuda", dtype=torch.bfloat16)
    R = torch.randn((M, N), device="cuda", generator=g).to(torch.bfloat16) if a.residual else None

    wsb = 0 if a.no_workspace or a.residual else mm.mmtrain_gemm_workspace_bytes(layout, M, N)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda") if wsb else None

    def run():
        check(mm.mmtrain_gemm(mm.BF16, layout, M, N, K, A, shp_a[1], B, shp_b[1], Cm, N, None, R, 0, ws, wsb), "mmtrain_gemm")

    ms = _time(run, a.iters)
    print(json.dumps({"op": "gemm", "layout": a.layout, "M": M, "N": N, "K": K, "workspace_bytes": wsb, "ms": ms,
                      "tflops": 2.0 * M * N * K / ms / 1e9}))


def bench_attn(a):
    shape = wl.SHAPES[a.config]
    seed = wl.longtail_seed() if a.config == 4 else 0
    cu, modes, _ = wl.make_segments(a.config, seed)
    T = int(cu[-1])
    desc = mm.make_desc(shape.kind, mm.BF16, shape.hidden, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.ffn_hidden)
    batch = mm.PackedBatch.on_device(cu, modes)
    g = torch.Generator(device="cuda").manual_seed(0)
    qkv = torch.randn((T, shape.nqkv), device="cuda", generator=g).to(torch.bfloat16)
    d_o = torch.randn((T, shape.nq), device="cuda", generator=g).to(torch.bfloat16)
    o = torch.empty((T, shape.nq), device="cuda", dtype=torch.bfloat16)
    d_qkv = torch.empty_like(qkv)
    lse = torch.empty((shape.n_heads, T), device="cuda", dtype=torch.float32)
    wsb = mm.mmtrain_attn_workspace_bytes(T, len(cu) - 1, shape.n_heads)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    fl = wl.model_flops(shape, cu, modes)["attn_fwd"]
    ms_f = _time(lambda: check(mm.mmtrain_attn_fwd(desc, batch, qkv, o, lse, ws, wsb), "attn_fwd"), a.iters)
    ms_b = _time(lambda: check(mm.mmtrain_attn_bwd(desc, batch, qkv, o, lse, d_o, d_qkv, ws, wsb), "attn_bwd"), a.iters)
    out = {"op": "attn", "config": a.config, "T": T, "segments": len(cu) - 1, "fwd_ms": ms_f, "bwd_ms": ms_b,
           "fwd_tflops": fl / ms_f / 1e9, "bwd_tflops": 2 * fl / ms_b / 1e9}
    if a.cu_busy:
        # one forward + backward with the per-compute-unit busy counters on: max / mean over the units that ran work
        busy = torch.zeros((3, 1024), dtype=torch.int64, device="cuda")
        mm.mmtrain_profile_attn_busy(busy)
        check(mm.mmtrain_attn_fwd(desc, batch, qkv, o, lse, ws, wsb), "attn_fwd")
        check(mm.mmtrain_attn_bwd(desc, batch, qkv, o, lse, d_o, d_qkv, ws, wsb), "attn_bwd")
        torch.cuda.synchronize()
        mm.mmtrain_profile_attn_busy(None)
        rows = busy.cpu().numpy()
        for name, r in zip(("fwd", "dq", "dkv"), rows):
            used = r[r > 0].astype(np.float64) / 100.0            # 100 MHz ticks -> microseconds
            out["cu_busy_" + name] = {"units": int(used.size), "mean_us": float(used.mean()), "max_us": float(used.max()),
                                      "max_over_mean": float(used.max() / used.mean())}
    print(json.dumps(out))


def bench_adam(a):
    """One AdamW step over n fp32 master weights (+ bf16 working copy, gradient cleared): bytes moved per second."""
    n = a.mparams * 1_000_000
    g = torch.Generator(device="cuda").manual_seed(0)
    w = torch.randn(n, device="cuda", generator=g)
    gr = torch.randn(n, device="cuda", generator=g)
    m = torch.zeros(n, device="cuda")
    v = torch.zeros(n, device="cuda")
    out = torch.empty(n, device="cuda", dtype=torch.bfloat16)
    desc = mm.make_adam_desc(1e-4, 0.9, 0.95, 1e-8, 0.1, 1.0, 1, zero_grad=True)
    ms = _time(lambda: check(mm.mmtrain_adam_step(desc, n, w, gr, m, v, out, mm.BF16), "adam"), a.iters)
    nbytes = n * (16 + 12 + 2 + 4)
    print(json.dumps({"op": "adam", "n": n, "ms": ms, "GB_per_s": nbytes / ms / 1e6, "bytes_per_element": 34,
                      "frac_of_8TBps": nbytes / ms / 1e6 / 8000.0}))


def bench_copy(a):
    n = a.mb * (1 << 20)
    src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    ms = _time(lambda: dst.copy_(src), a.iters)
    print(json.dumps({"op": "copy", "bytes_read": n, "bytes_written": n, "ms": ms, "GBps": 2 * n / ms / 1e6}))


def main(argv=None):
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="op", required=True)
    g = sub.add_parser("gemm")
    g.add_argument("--layout", default="nt", choices=["nt", "nn", "tn"])
    g.add_argument("--m", type=int, default=8192)
    g.add_argument("--n", type=int, default=22016)
    g.add_argument("--k", type=int, default=4096)
    g.add_argument("--residual", action="store_true")
    g.add_argument("--no-workspace", action="store_true", help="no scratch: the product is never cut along K")
    g.add_argument("--iters", type=int, default=20)
    t = sub.add_parser("attn")
    t.add_argument("--config", type=int, default=3)
    t.add_argument("--iters", type=int, default=20)
    t.add_argument("--cu-busy", action="store_true", help="also report the attention kernels' load balance over the compute units")
    ad = sub.add_parser("adam")
    ad.add_argument("--mparams", type=int, default=202, help="millions of parameters (202 = one 7B layer)")
    ad.add_argument("--iters", type=int, default=20)
    c = sub.add_parser("copy")
    c.add_argument("--mb", type=int, default=512)
    c.add_argument("--iters", type=int, default=10)
    a = ap.parse_args(argv)
    mm.load_library()
    {"gemm": bench_gemm, "attn": bench_attn, "copy": bench_copy, "adam": bench_adam}[a.op](a)


if __name__ == "__main__":
    main()
