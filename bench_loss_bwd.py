#!/usr/bin/env python3
"""Benchmark of the in-place log-softmax-loss backward (Sec. 4.2.2, Alg. 3) on one MI355X.

Workload: the logits of one training batch of the draft model over all TTT steps: 4096 tokens x 7
steps = 28672 rows of a 32000-entry draft vocabulary, fp32 logits and targets resident in HBM
(synthetic: seeded Gaussians / normalised random targets).  A step = one call over all rows.
One JSON line: rows/s, the HBM roofline of the kernel (algorithmic bytes = read logits + read
target + write gradient = 3 * V * element size per row, plus 4 bytes of g), and the numpy fp64
oracle timed on a bounded sample of rows.

    python bench_loss_bwd.py [--rows 28672] [--vocab 32000] [--dtype f32|bf16] [--steps 20] [--warmup 3]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
PEAK_HBM_GBS = 8000.0


def recorded_traffic(summary_name):
    """HBM bytes per launch of this script's kernel as the committed rocprofv3 summary of its default
    command states them ("... MB read ... MB written"); (bytes or None, source file)."""
    import re
    path = os.path.join(ROOT, "profiles", summary_name)
    if not os.path.exists(path):
        return None, None
    text = open(path).read()
    rd, wr = re.search(r"([\d.]+) MB read", text), re.search(r"([\d.]+) MB written", text)
    if not rd or not wr:
        return None, os.path.relpath(path, ROOT)
    return (float(rd.group(1)) + float(wr.group(1))) * 1e6, os.path.relpath(path, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--rows", type=int, default=28672)
    ap.add_argument("--vocab", type=int, default=32000)
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    import numpy as np
    import torch
    from paper_2603_18567_amd import binding as B
    assert torch.cuda.is_available(), "needs the GPU (there is no CPU path)"
    dev = torch.device("cuda:0")
    dt = {"f32": torch.float32, "bf16": torch.bfloat16}[args.dtype]
    gen = torch.Generator(device=dev).manual_seed(99)
    z0 = (torch.randn(args.rows, args.vocab, generator=gen, device=dev) * 3).to(dt)
    p = torch.rand(args.rows, args.vocab, generator=gen, device=dev) ** 6
    p = (p / p.sum(1, keepdim=True)).to(dt)
    g = torch.randn(args.rows, generator=gen, device=dev)
    z = z0.clone()

    for _ in range(args.warmup):
        B.ttt_loss_bwd_inplace(z, p, g)
    torch.cuda.synchronize()
    B.ttt_attn_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        B.ttt_loss_bwd_inplace(z, p, g)      # the buffer holds gradients after the first call: same traffic
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    k_ms = B.ttt_attn_profile_totals().get("ttt_loss_bwd_kernel", 0.0) / args.steps
    B.ttt_attn_profile_enable(False)
    ms = wall * 1e3 / args.steps
    esz = z.element_size()
    alg_bytes = args.rows * (3 * args.vocab * esz + 4)
    ach = alg_bytes / (k_ms * 1e-3) / 1e9 if k_ms else None
    traffic, traffic_source = recorded_traffic("loss_bwd_28672x32000_kernel_stats.txt")
    out = {"metric": "loss_bwd_inplace_rows_per_s", "value": args.rows / (ms * 1e-3), "unit": "rows/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
           "config": {"workload": f"draft_logits_{args.rows}x{args.vocab}", "rows": args.rows, "vocab": args.vocab},
           "roofline": {"kernel": "ttt_loss_bwd_kernel", "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": ach / PEAK_HBM_GBS if ach else None,
                        # parsed from the committed rocprofv3 summary of the default command, never typed in here
                        "traffic": traffic if (args.rows, args.vocab, args.dtype) == (28672, 32000, "f32") else None, "traffic_source": traffic_source, "avg_ms": k_ms,
                        "algorithmic_bytes_per_launch": alg_bytes}}
    if not args.no_cpu_baseline:
        from oracle.loss_oracle import logsoftmax_loss_bwd
        n = min(args.rows, 2048)
        zs, ps, gs = z0[:n].float().cpu().numpy(), p[:n].float().cpu().numpy(), g[:n].cpu().numpy()
        t0 = time.perf_counter()
        ref = logsoftmax_loss_bwd(zs, ps, gs)
        dt_cpu = time.perf_counter() - t0
        zc = z0[:n].clone()
        B.ttt_loss_bwd_inplace(zc, p[:n], g[:n])
        err = float(np.abs(zc.float().cpu().numpy() - ref).max() / np.abs(ref).max())
        out["cpu_baseline"] = {"value": n / dt_cpu, "unit": "rows/s", "cores": 1, "kind": "oracle",
                               "sample": f"first {n} rows of the workload in {dt_cpu:.2f} s (numpy fp64); GPU result of those rows "
                                         f"differs by {err:.1e} of the largest reference value"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
