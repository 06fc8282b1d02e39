#!/usr/bin/env python3
"""Benchmark of the TTT attention hot path on one MI355X.

One "step" = one all-steps forward call + one all-steps backward call (every kernel of the path)
on one batch of seeded synthetic inputs already resident in HBM.  Prints ONE JSON line:

  value / ms_per_step   useful masked TFLOP/s (14*d*pairs per step; hidden pairs not counted,
                        recomputation counted once) from the wall time between two synchronisations
                        around exactly --steps steps, with no diagnostics running;
  median_ms / min_ms    over the per-step HIP-event spans of the same timed steps;
  bwd_8dP_tflops        the backward under the no-recompute convention (8*d*pairs);
  pct_of_measured_clock_peak   against CU count x 4096 flop/clk x the shader clock the driver
                        reports while the same steps run back to back (a separate, untimed leg);
  sustained_power_w / power_cap_w / energy_per_step_j   board power over that leg, the board's cap;
  step_at_a_time        the training order (Sec. 2.4: step j's input depends on step j-1): k forward
                        calls, then k backward calls in descending order with the fp32 carry; also the
                        same calls replayed from one captured HIP graph;
  roofline              of the dominant kernel, from per-kernel HIP-event times (library
                        diagnostics) taken in a separate, untimed pass over the same steps;
  configs               ms / TFLOP/s / % of peak of the five configurations beside the headline one;
  cpu_baseline          the fp64 oracle timed on the host cores on a bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload headline_4k]
                    [--no-cpu-baseline] [--no-configs] [--no-stepwise]
"""
import argparse
import glob
import json
import os
import statistics
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3       # MI355X fp32 MFMA/vector
MFMA_FLOP_PER_CLK_CU = 4096   # dense bf16: 4 SIMDs x 1024 flop per clock
OTHER_CONFIGS = ("tiny_f32", "llama8b_2k", "varlen_16k", "qwen235b_8k", "long_32k")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="headline_4k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the five other configurations")
    ap.add_argument("--no-stepwise", action="store_true", help="skip the step-at-a-time leg and the clock leg")
    ap.add_argument("--cpu-rows", type=int, default=0, help="rows of the oracle sample (0 = sized for ~15 s)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for the FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def recorded_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` as the committed rocprofv3 summary of this command records
    them (profiles/<workload>_hbm_traffic.txt: FETCH_SIZE scaled by the copy calibration, plus
    WRITE_SIZE).  A counter cannot be read from inside this process; the figure is parsed from the
    summary, never typed in here.  Returns (bytes or None, source)."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None, None
    with open(path) as f:
        for line in f:
            cols = line.split()
            if len(cols) == 5 and kernel in cols[0]:
                try:
                    return (float(cols[3]) + float(cols[4])) * 1e6, os.path.relpath(path, ROOT)
                except ValueError:
                    pass
    return None, os.path.relpath(path, ROOT)


class ClockSampler(threading.Thread):
    """Polls the shader clock the driver publishes (pp_dpm_sclk: the line marked '*')."""

    def __init__(self, period=0.004):
        super().__init__(daemon=True)
        files = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        self.path = files[0] if files else None
        power = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"))
        self.power_path = power[0] if power else None          # board power, microwatts
        self.period = period
        self.samples = []
        self.power_samples = []
        self.stop_flag = False

    @staticmethod
    def read_number(path):
        try:
            with open(path) as f:
                return float(f.read().strip())
        except (OSError, ValueError, TypeError):
            return None

    def power_cap_w(self):
        if not self.power_path:
            return None
        v = self.read_number(self.power_path.replace("power1_input", "power1_cap"))
        return v / 1e6 if v else None

    def read_once(self):
        try:
            with open(self.path) as f:
                for line in f:
                    if "*" in line:
                        return float(line.split(":")[1].lower().replace("mhz", "").replace("*", "").strip())
        except (OSError, ValueError, IndexError, TypeError):
            return None
        return None

    def run(self):
        while not self.stop_flag and self.path:
            v = self.read_once()
            if v:
                self.samples.append(v)
            if self.power_path:
                w = self.read_number(self.power_path)
                if w:
                    self.power_samples.append(w / 1e6)
            time.sleep(self.period)


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


class Bench:
    """One workload resident on the GPU with its runner."""

    def __init__(self, wl, dev, inp=None):
        import torch
        from paper_2603_18567_amd import TttAttnRunner
        from paper_2603_18567_amd.workloads import make_inputs
        self.torch = torch
        self.wl = wl
        self.inp = make_inputs(wl) if inp is None else inp
        self.d_o = [x.to(dev) for x in self.inp.d_o]
        self.run = TttAttnRunner([x.to(dev) for x in self.inp.q], [x.to(dev) for x in self.inp.k],
                                 [x.to(dev) for x in self.inp.v], wl.cu_seqlens, wl.scale, dev)
        self.run.alloc_grads()

    def all_steps(self):
        self.run.forward()
        self.run.backward(self.d_o)

    def stepwise(self):
        k = self.wl.k
        for j in range(k):
            self.run.forward(j, j + 1)
        for j in reversed(range(k)):
            self.run.backward(self.d_o, j, j + 1, accumulate=True)

    def timed(self, fn, steps, warmup):
        """(wall ms per step, [per-step event spans in ms]) of `steps` calls of fn after `warmup`."""
        torch = self.torch
        for _ in range(warmup):
            fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev[0].record()
        for s in range(steps):
            fn()
            ev[s + 1].record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return wall * 1e3 / steps, [ev[s].elapsed_time(ev[s + 1]) for s in range(steps)]


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path needs no collective: documents, heads "
              "and steps are independent). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2603_18567_amd import binding
    from paper_2603_18567_amd.workloads import WORKLOADS

    wl = WORKLOADS[args.workload]
    assert torch.cuda.is_available(), "bench.py needs the GPU (there is no CPU path)"
    dev = torch.device("cuda:0")
    b = Bench(wl, dev)
    run, d_o = b.run, b.d_o
    fl = wl.useful_flops()
    peak = PEAK_BF16_TFLOPS if wl.dtype == "bf16" else PEAK_F32_TFLOPS

    # ---- the timed region: warm-up, then K all-steps fwd+bwd between two synchronisations, no diagnostics
    for _ in range(args.warmup):
        b.all_steps()
    torch.cuda.synchronize()
    if args.copy_calibration:
        src = torch.full((256 << 20,), 7, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)            # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
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
    ms_per_step = wall * 1e3 / args.steps
    fwd_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / args.steps
    bwd_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / args.steps
    spans = [e[0].elapsed_time(e[2]) for e in ev]
    value = fl["fwd_bwd"] / (ms_per_step * 1e-3) / 1e12

    # ---- per-kernel durations: the same steps again, untimed, with the library's event diagnostics on
    binding.ttt_attn_profile_enable(True)
    for _ in range(args.steps):
        b.all_steps()
    torch.cuda.synchronize()
    kernel_ms = {name: ms / args.steps for name, ms in binding.ttt_attn_profile_totals().items()}
    binding.ttt_attn_profile_enable(False)

    # dominant kernel: the key-stationary dK/dV kernel does S, dP, dV, dK on the block-0 (causal) pairs
    causal_pairs = wl.hq * sum(wl.k * L * (L + 1) // 2 for L in wl.doc_lens)
    alg = {
        "ttt_fwd_kernel": 4 * wl.d * wl.pairs(),
        "ttt_bwd_dkv_kernel": 8 * wl.d * causal_pairs,
        "ttt_bwd_dkv_p8_kernel": 8 * wl.d * causal_pairs,
        "ttt_bwd_dq_kernel": 2 * wl.d * wl.pairs(),
        "ttt_bwd_dq_pipe_kernel": 2 * wl.d * wl.pairs(),
    }
    dom = max((n for n in kernel_ms if n in alg), key=lambda n: kernel_ms[n], default=None)
    roofline = None
    if dom is not None:
        ach = alg[dom] / (kernel_ms[dom] * 1e-3) / 1e12
        traffic, source = recorded_traffic(wl.name, dom)
        roofline = {"kernel": dom, "bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s",
                    "frac": ach / peak, "traffic": traffic, "traffic_source": source, "avg_ms": kernel_ms[dom],
                    "algorithmic_flops_per_launch": alg[dom]}

    out = {
        "metric": "ttt_attn_fwd_bwd_useful_tflops", "value": value, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "tokens": wl.T, "docs": len(wl.doc_lens), "hq": wl.hq, "hkv": wl.hkv,
                   "head_dim": wl.d, "k_steps": wl.k, "mode": "all-steps (one fwd call + one bwd call)"},
        "pct_of_peak": 100.0 * value / peak, "peak_tflops": peak,
        "median_ms": statistics.median(spans), "min_ms": min(spans),
        "fwd_ms": fwd_ms, "bwd_ms": bwd_ms,
        "fwd_tflops": fl["fwd"] / (fwd_ms * 1e-3) / 1e12, "bwd_tflops": fl["bwd"] / (bwd_ms * 1e-3) / 1e12,
        "bwd_8dP_tflops": 0.8 * fl["bwd"] / (bwd_ms * 1e-3) / 1e12,
        "useful_tflop_per_step": fl["fwd_bwd"] / 1e12,
        "kernel_ms": kernel_ms,
        "roofline": roofline,
    }

    if not args.no_stepwise:
        # ---- sustained shader clock while the same steps run back to back (untimed leg)
        sampler = ClockSampler()
        n_clock_steps = max(args.steps, int(600.0 / max(ms_per_step, 0.05)))
        for _ in range(3):
            b.all_steps()
        torch.cuda.synchronize()
        sampler.start()
        for _ in range(min(n_clock_steps, 2000)):
            b.all_steps()
        torch.cuda.synchronize()
        sampler.stop_flag = True
        sampler.join()
        half = sampler.samples[len(sampler.samples) // 2:]       # the second half: the clock has settled
        if half:
            clk = statistics.median(half)
            n_cu = torch.cuda.get_device_properties(0).multi_processor_count
            clock_peak = n_cu * MFMA_FLOP_PER_CLK_CU * clk * 1e6 / 1e12
            out["sustained_clock_mhz"] = clk
            out["clock_samples"] = len(half)
            out["compute_units"] = n_cu
            out["pct_of_measured_clock_peak"] = 100.0 * value / clock_peak if wl.dtype == "bf16" else None
        else:
            out["sustained_clock_mhz"] = None
            out["pct_of_measured_clock_peak"] = None
        # board power over the same leg (the driver's hwmon reading) beside the board's cap: these
        # kernels run against the cap, so a step's time is its energy divided by the cap
        phalf = sampler.power_samples[len(sampler.power_samples) // 2:]
        out["sustained_power_w"] = statistics.median(phalf) if phalf else None
        out["power_cap_w"] = sampler.power_cap_w()
        out["energy_per_step_j"] = out["sustained_power_w"] * ms_per_step * 1e-3 if phalf else None

        # ---- the training order: k forward calls, then k backward calls (descending, fp32 carry)
        sw_ms, sw_spans = b.timed(b.stepwise, args.steps, max(2, args.warmup // 2))
        sw_val = fl["fwd_bwd"] / (sw_ms * 1e-3) / 1e12
        out["step_at_a_time"] = {"ms": sw_ms, "median_ms": statistics.median(sw_spans), "min_ms": min(sw_spans),
                                 "tflops": sw_val, "pct_of_peak": 100.0 * sw_val / peak,
                                 "calls": f"{wl.k} forward + {wl.k} backward (accumulate_dkv=1, descending steps)"}
        # the same 2k calls recorded once in a HIP graph and replayed (the library allocates nothing and
        # never synchronises, so its calls can be captured): what the host-side launches cost
        try:
            graph = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.graph(graph, stream=side):
                b.stepwise()
            torch.cuda.synchronize()
            g_ms, g_spans = b.timed(graph.replay, args.steps, 2)
            out["step_at_a_time"]["graph_replay_ms"] = g_ms
            out["step_at_a_time"]["graph_replay_median_ms"] = statistics.median(g_spans)
        except RuntimeError as err:       # capture refused by the runtime: reported, not fatal
            out["step_at_a_time"]["graph_replay_ms"] = None
            out["step_at_a_time"]["graph_replay_error"] = str(err)[:200]

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, b.inp, args.cpu_rows)

    if not args.no_configs:
        # ---- the other configurations, same kernels, few steps each (the long ones take 0.07-0.25 s a step)
        del b, run, d_o
        torch.cuda.empty_cache()
        cfgs = []
        for name in OTHER_CONFIGS:
            if name == wl.name:
                continue
            w = WORKLOADS[name]
            bb = Bench(w, dev)
            est_ms, _ = bb.timed(bb.all_steps, 1, 1)
            steps = max(3, min(args.steps, int(300.0 / max(est_ms, 0.01))))
            ms, sp = bb.timed(bb.all_steps, steps, 1)
            f = w.useful_flops()["fwd_bwd"]
            pk = PEAK_BF16_TFLOPS if w.dtype == "bf16" else PEAK_F32_TFLOPS
            cfgs.append({"workload": name, "dtype": w.dtype, "tokens": w.T, "docs": len(w.doc_lens), "steps": steps,
                         "ms": ms, "median_ms": statistics.median(sp), "min_ms": min(sp),
                         "tflops": f / (ms * 1e-3) / 1e12, "pct_of_peak": 100.0 * f / (ms * 1e-3) / 1e12 / pk})
            del bb
            torch.cuda.empty_cache()
        out["configs"] = cfgs
    print(json.dumps(out))


if __name__ == "__main__":
    main()
