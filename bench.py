#!/usr/bin/env python3
"""Benchmark of the TTT attention hot path on one MI355X.

One "step" = one all-steps forward call + one all-steps backward call (every kernel of the path)
on one batch of seeded synthetic inputs already resident in HBM.  Prints ONE JSON line:
useful masked TFLOP/s (14*d*pairs per step; hidden pairs not counted, recomputation counted once),
the roofline of the dominant kernel from per-kernel HIP-event times taken inside the timed region,
and the fp64 oracle timed on the host cores on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload headline_4k] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3       # MI355X fp32 MFMA/vector
# HBM bytes per launch of the dominant kernel from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this
# command (profiles/headline_4k_hbm_traffic.txt: fetch scaled by the copy calibration, plus write);
# a counter cannot be read from inside this process, so the recorded figure is reported.
RECORDED_TRAFFIC = {("headline_4k", "ttt_bwd_dkv_kernel"): 912.6e6 + 302.0e6}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="headline_4k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=0, help="rows of the oracle sample (0 = sized for ~15 s)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for the FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def cpu_baseline(wl, inp, rows_override=0, target_s=15.0):
    """The fp64 oracle, as it stands, on a seeded sample of query rows of this workload
    (forward + backward restricted to those rows = a row-sparse cotangent).  A short pilot sizes
    the sample for about `target_s` seconds on this host."""
    import numpy as np
    import torch
    import oracle
    oracle.build_oracle()
    cores = int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)
    rng = np.random.default_rng(wl.seed)
    f32 = lambda ts: np.stack([t.to(torch.float32).numpy() for t in ts])
    Q, K, V = f32(inp.q), f32(inp.k), f32(inp.v)
    cu = np.asarray(wl.cu_seqlens)

    def run(n_rows):
        rs = rng.integers(0, wl.k, n_rows).astype(np.int32)
        rt = rng.integers(0, wl.T, n_rows).astype(np.int32)
        dO_rows = np.stack([inp.d_o[j][i].to(torch.float32).numpy() for j, i in zip(rs, rt)])
        starts = cu[np.searchsorted(cu, rt, side="right") - 1]
        pairs = int(((rt - starts + 1) + rs).sum()) * wl.hq
        t0 = time.perf_counter()
        oracle.oracle_run(Q, K, V, wl.cu_seqlens, wl.scale, rs, rt, dO_rows)
        return pairs, time.perf_counter() - t0

    if rows_override:
        n_rows = rows_override
    else:
        p_pairs, p_dt = run(4 * cores)                      # pilot
        rows_per_s = 4 * cores / max(p_dt, 1e-3)
        n_rows = int(max(4 * cores, min(wl.k * wl.T, rows_per_s * target_s)))
    pairs, dt = run(n_rows)
    flops = 14 * wl.d * pairs
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"{n_rows} seeded query rows (all {wl.hq} heads) of {wl.name}: fwd+bwd of those rows, "
                      f"{pairs:.3e} visible pairs in {dt:.1f} s; the full workload would take ~{wl.pairs() / pairs * dt:.0f} s (extrapolated)"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path needs no collective: documents, heads "
              "and steps are independent). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2603_18567_amd import TttAttnRunner, binding
    from paper_2603_18567_amd.workloads import WORKLOADS, make_inputs

    wl = WORKLOADS[args.workload]
    assert torch.cuda.is_available(), "bench.py needs the GPU (there is no CPU path)"
    dev = torch.device("cuda:0")
    inp = make_inputs(wl)
    q = [x.to(dev) for x in inp.q]
    k = [x.to(dev) for x in inp.k]
    v = [x.to(dev) for x in inp.v]
    d_o = [x.to(dev) for x in inp.d_o]
    run = TttAttnRunner(q, k, v, wl.cu_seqlens, wl.scale, dev)
    run.alloc_grads()

    def step():
        run.forward()
        run.backward(d_o)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.copy_calibration:
        src = torch.full((256 << 20,), 7, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)            # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # timed region: K steps between two synchronisations; per-call events for the fwd/bwd split and
    # per-kernel events (library diagnostics) for the roofline of the dominant kernel
    binding.ttt_attn_profile_enable(True)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    kernel_ms = {}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        ev[s][0].record()
        run.forward()
        ev[s][1].record()
        run.backward(d_o)
        ev[s][2].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    for name, ms in binding.ttt_attn_profile_totals().items():
        kernel_ms[name] = ms / args.steps
    binding.ttt_attn_profile_enable(False)

    fwd_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / args.steps
    bwd_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / args.steps
    ms_per_step = wall * 1e3 / args.steps
    fl = wl.useful_flops()
    peak = PEAK_BF16_TFLOPS if wl.dtype == "bf16" else PEAK_F32_TFLOPS
    value = fl["fwd_bwd"] / (ms_per_step * 1e-3) / 1e12

    # dominant kernel: key-stationary dK/dV kernel: S, dP, dV, dK on the block-0 (causal) pairs
    causal_pairs = wl.hq * sum(wl.k * L * (L + 1) // 2 for L in wl.doc_lens)
    alg = {
        "ttt_fwd_kernel": 4 * wl.d * wl.pairs(),
        "ttt_bwd_dkv_kernel": 8 * wl.d * causal_pairs,
        "ttt_bwd_dq_kernel": 2 * wl.d * wl.pairs(),
    }
    dom = max((n for n in kernel_ms if n in alg), key=lambda n: kernel_ms[n], default=None)
    roofline = None
    if dom is not None:
        ach = alg[dom] / (kernel_ms[dom] * 1e-3) / 1e12
        roofline = {"kernel": dom, "bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s",
                    "frac": ach / peak, "traffic": RECORDED_TRAFFIC.get((wl.name, dom)), "avg_ms": kernel_ms[dom],
                    "algorithmic_flops_per_launch": alg[dom]}

    out = {
        "metric": "ttt_attn_fwd_bwd_useful_tflops", "value": value, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "tokens": wl.T, "docs": len(wl.doc_lens), "hq": wl.hq, "hkv": wl.hkv,
                   "head_dim": wl.d, "k_steps": wl.k, "mode": "all-steps (one fwd call + one bwd call)"},
        "pct_of_peak": 100.0 * value / peak, "peak_tflops": peak,
        "fwd_ms": fwd_ms, "bwd_ms": bwd_ms,
        "fwd_tflops": fl["fwd"] / (fwd_ms * 1e-3) / 1e12, "bwd_tflops": fl["bwd"] / (bwd_ms * 1e-3) / 1e12,
        "useful_tflop_per_step": fl["fwd_bwd"] / 1e12,
        "kernel_ms": kernel_ms,
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, inp, args.cpu_rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
