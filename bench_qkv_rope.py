#!/usr/bin/env python3
"""Benchmark of the producer of Q_j, K_j, V_j (QKV projection + rotary embedding) on one MI355X.

Workload: one TTT step of a Llama-3.1-8B-shaped draft layer: 4096 tokens, hidden_in = 8192 (token
embedding and target hidden state side by side), 32 query + 8 key + 8 value heads of 128, bf16
operands resident in HBM (synthetic: seeded Gaussians).  A step = one call.  One JSON line: dense
TFLOP/s (2 * tokens * hidden_in * features per call), the bf16 MFMA roofline of the kernel, beside
it the same result made the unfused way (torch.matmul, i.e. the vendor GEMM, then a rotation written
with plain tensor ops: comparison only, nothing in the library uses it), and the numpy fp64 oracle
timed on a bounded sample of tokens.

    python bench_qkv_rope.py [--tokens 4096] [--hidden-in 8192] [--hq 32] [--hkv 8] [--steps 20] [--warmup 3]
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
PEAK_TFLOPS = 2500.0


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
    ap.add_argument("--tokens", type=int, default=4096)
    ap.add_argument("--hidden-in", type=int, default=8192)
    ap.add_argument("--hq", type=int, default=32)
    ap.add_argument("--hkv", type=int, default=8)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    import numpy as np
    import torch
    from paper_2603_18567_amd import binding as B
    assert torch.cuda.is_available(), "needs the GPU (there is no CPU path)"
    dev = torch.device("cuda:0")
    T, hin, hq, hkv, d = args.tokens, args.hidden_in, args.hq, args.hkv, 128
    nf = (hq + 2 * hkv) * d
    gen = torch.Generator(device=dev).manual_seed(2024)
    x = torch.randn(T, hin, generator=gen, device=dev).to(torch.bfloat16)
    w = (torch.randn(nf, hin, generator=gen, device=dev) / math.sqrt(hin)).to(torch.bfloat16)
    pos = torch.arange(T, dtype=torch.int32, device=dev)
    inv = 10000.0 ** (-torch.arange(0, d, 2, dtype=torch.float64) / d)
    ang = torch.arange(T, dtype=torch.float64)[:, None] * inv[None, :]
    cos_t, sin_t = torch.cos(ang).float().to(dev), torch.sin(ang).float().to(dev)
    q = torch.empty(T, hq, d, dtype=torch.bfloat16, device=dev)
    k = torch.empty(T, hkv, d, dtype=torch.bfloat16, device=dev)
    v = torch.empty(T, hkv, d, dtype=torch.bfloat16, device=dev)

    def ours():
        B.ttt_qkv_rope_fwd(x, w, cos_t, sin_t, pos, q, k, v)

    for _ in range(args.warmup):
        ours()
    torch.cuda.synchronize()
    B.ttt_attn_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ours()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    k_ms = B.ttt_attn_profile_totals().get("ttt_qkv_rope_kernel", 0.0) / args.steps
    B.ttt_attn_profile_enable(False)
    ms = wall * 1e3 / args.steps
    flops = 2.0 * T * hin * nf
    ach = flops / (k_ms * 1e-3) / 1e12 if k_ms else None

    # the unfused way: vendor GEMM, then rotation and split as separate passes over the result
    def unfused():
        y = torch.matmul(x, w.t()).view(T, hq + 2 * hkv, d)
        c, s = cos_t[:, None, :], sin_t[:, None, :]
        yr = y[:, :hq + hkv].float()
        lo, hi = yr[..., :d // 2], yr[..., d // 2:]
        rot = torch.cat([lo * c - hi * s, hi * c + lo * s], -1).to(torch.bfloat16)
        return rot[:, :hq].contiguous(), rot[:, hq:].contiguous(), y[:, hq + hkv:].contiguous()

    def gemm_only():
        return torch.matmul(x, w.t())

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    unf_ms, gemm_ms = timed(unfused), timed(gemm_only)
    uq, uk, uv = unfused()
    diff = max(float((uq.float() - q.float()).abs().max()), float((uk.float() - k.float()).abs().max()),
               float((uv.float() - v.float()).abs().max()))
    traffic, traffic_source = recorded_traffic("qkv_rope_4096x8192x6144_kernel_stats.txt")
    out = {"metric": "qkv_rope_dense_tflops", "value": flops / (ms * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"draft_qkv_{T}x{hin}x{nf}", "tokens": T, "hidden_in": hin, "hq": hq, "hkv": hkv, "head_dim": d},
           "roofline": {"kernel": "ttt_qkv_rope_kernel", "bound": "mfma", "achieved": ach, "peak": PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": ach / PEAK_TFLOPS if ach else None,
                        # parsed from the committed rocprofv3 summary of the default command, never typed in here
                        "traffic": traffic if (T, hin, hq, hkv) == (4096, 8192, 32, 8) else None, "traffic_source": traffic_source, "avg_ms": k_ms,
                        "algorithmic_flops_per_launch": flops},
           "unfused_comparison": {"vendor_gemm_plus_rotation_ms": unf_ms, "vendor_gemm_alone_ms": gemm_ms,
                                  "vendor_gemm_alone_tflops": flops / (gemm_ms * 1e-3) / 1e12,
                                  "max_abs_diff_to_ours": diff}}
    # the consumer: output projection reading O_j ([T, hq * d] -> hidden = hq * d), same kernel, no rotation
    wo = (torch.randn(hq * d, hq * d, generator=gen, device=dev) / math.sqrt(hq * d)).to(torch.bfloat16)
    proj = torch.empty(T, hq * d, dtype=torch.bfloat16, device=dev)
    o_ms = timed(lambda: B.ttt_o_proj_fwd(q, wo, proj))
    out["o_projection"] = {"ms": o_ms, "tflops": 2.0 * T * (hq * d) ** 2 / (o_ms * 1e-3) / 1e12,
                           "vendor_gemm_ms": timed(lambda: torch.matmul(q.view(T, -1), wo.t()))}
    if not args.no_cpu_baseline:
        from oracle.qkv_oracle import qkv_rope
        n = min(T, 256)
        rows = np.linspace(0, T - 1, n).astype(np.int64)
        xs, ws = x[rows].float().cpu().numpy(), w.float().cpu().numpy()
        cs, ss, ps = cos_t.cpu().numpy(), sin_t.cpu().numpy(), pos[rows].cpu().numpy()
        t0 = time.perf_counter()
        rq, rk, rv = qkv_rope(xs, ws, cs, ss, ps, hq, hkv, d)
        dt_cpu = time.perf_counter() - t0
        err = max(np.abs(q[rows].float().cpu().numpy() - rq).max(), np.abs(k[rows].float().cpu().numpy() - rk).max(),
                  np.abs(v[rows].float().cpu().numpy() - rv).max())
        out["cpu_baseline"] = {"value": 2.0 * n * hin * nf / dt_cpu / 1e12, "unit": "TFLOP/s",
                               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), "kind": "oracle",
                               "sample": f"{n} evenly spaced tokens of the workload (all {hq + 2 * hkv} heads), {dt_cpu:.2f} s; "
                                         f"max abs difference of the GPU result on them {err:.3e}"}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
