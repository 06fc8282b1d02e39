#!/usr/bin/env python3
"""The paper's own attention micro-benchmark, in kind (Sec. 5.4): the FINAL training-time-test step
only (step k-1 of k = 7 attends to the causal prefix plus k-1 diagonal keys), forward + backward,
time and peak device memory over a sweep of sequence lengths, beside two baselines that
materialise the mask / the logits the way an unfused implementation does:

  naive : one GEMM for the [hq, S, k*S] logits over the concatenated cache, the mask of Alg. 2 as a
          boolean tensor, softmax, a second GEMM; backward by autograd (plain PyTorch ops).
  sdpa  : torch.nn.functional.scaled_dot_product_attention with that mask as attn_mask (whatever
          backend this PyTorch build selects for an arbitrary mask).

Both baselines are comparison points only; nothing in the library uses them.  They are skipped at
lengths where their logits would not fit the device.  One JSON line per sequence length.

    python bench_final_step.py [--seqs 1024 2048 4096 8192 16384 32768] [--ks 7] [--steps 5] [--warmup 2]

--ks sweeps the TTT length as well (the paper's Training Insights study lengths up to 17):
    python bench_final_step.py --seqs 4096 --ks 1 3 5 7 9 13 17
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--seqs", type=int, nargs="+", default=[1024, 2048, 4096, 8192, 16384, 32768])
    ap.add_argument("--k", type=int, default=7, help="TTT length (used when --ks is not given)")
    ap.add_argument("--ks", type=int, nargs="+", default=None, help="TTT lengths to sweep")
    ap.add_argument("--hq", type=int, default=32)
    ap.add_argument("--hkv", type=int, default=8)
    ap.add_argument("--d", type=int, default=128)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--baseline-mem-gib", type=float, default=40.0,
                    help="skip a baseline whose logits alone would exceed this many GiB")
    return ap.parse_args()


def timed(fn, steps, warmup, torch):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps, torch.cuda.max_memory_allocated()


def alg2_mask(S, k, j, dev, torch):
    """[S, k*S] boolean mask of query step j (Alg. 2): block 0 causal, blocks 1..j their own token."""
    i = torch.arange(S, device=dev)[:, None]
    col = torch.arange(k * S, device=dev)[None, :]
    blk, m = col // S, col % S
    return ((blk == 0) & (m <= i)) | ((blk >= 1) & (blk <= j) & (m == i))


def main():
    args = parse()
    import torch
    assert torch.cuda.is_available(), "needs the GPU"
    for k in (args.ks or [args.k]):
        for S in args.seqs:
            one_point(args, k, S)


def one_point(args, k, S):
    import torch
    import torch.nn.functional as F
    from paper_2603_18567_amd import TttAttnRunner, binding
    from paper_2603_18567_amd.workloads import custom_workload, make_inputs
    dev = torch.device("cuda:0")
    j = k - 1
    G = args.hq // args.hkv
    wl = custom_workload(f"final_step_{S}", "bf16", (S,), args.hq, args.hkv, args.d, k, seed=4242 + S)
    inp = make_inputs(wl)
    q = [x.to(dev) for x in inp.q]
    kk = [x.to(dev) for x in inp.k]
    v = [x.to(dev) for x in inp.v]
    d_o = [x.to(dev) for x in inp.d_o]

    # ---- this library: forward and backward of step j alone.  Everything the two calls need beyond the
    # inputs they are handed -- O_j, LSE_j, dQ_j, dK_l and dV_l of the blocks l <= j, the two workspaces --
    # is allocated inside the measured region, and the figure is the allocator's peak, like the baselines'.
    run = TttAttnRunner(q, kk, v, wl.cu_seqlens, wl.scale, dev, allocate_outputs=False)
    p1 = run.params(j, j + 1)
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    before = torch.cuda.memory_allocated()
    run.o = [torch.empty_like(q[j]) if s == j else None for s in range(k)]
    run.lse = [torch.empty((args.hq, S), dtype=torch.float32, device=dev) if s == j else None for s in range(k)]
    run.dq = [torch.empty_like(q[j]) if s == j else None for s in range(k)]
    run.dk = [torch.empty_like(kk[l]) if l <= j else None for l in range(k)]
    run.dv = [torch.empty_like(v[l]) if l <= j else None for l in range(k)]
    for which in (binding.TTT_PASS_FWD, binding.TTT_PASS_BWD):
        run._ws[which] = torch.empty(binding.ttt_attn_workspace_bytes(p1, which), dtype=torch.uint8, device=dev)

    def ours():
        run.forward(j, j + 1)
        run.backward(d_o, j, j + 1)

    ours()
    torch.cuda.synchronize()
    ours_extra = torch.cuda.max_memory_allocated() - before
    ours_ms, _ = timed(ours, args.steps, args.warmup, torch)
    pairs = args.hq * (S * (S + 1) // 2 + S * j)
    flops = 14 * args.d * pairs
    out = {"bench": "final_ttt_step_fwd_bwd", "seq_len": S, "k": k, "step": j, "dtype": "bf16",
           "hq": args.hq, "hkv": args.hkv, "head_dim": args.d,
           "ours_ms": ours_ms, "ours_useful_tflops": flops / (ours_ms * 1e-3) / 1e12,
           "ours_pct_of_bf16_peak": 100 * flops / (ours_ms * 1e-3) / 2.5e15,
           "ours_mem_beyond_inputs_MiB": ours_extra / 2**20}
    # the same two calls replayed from a captured HIP graph (nothing in them allocates or synchronises):
    # what the host side of the launches costs at short sequences
    try:
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.graph(graph, stream=side):
            ours()
        torch.cuda.synchronize()
        out["ours_graph_replay_ms"], _ = timed(graph.replay, args.steps, args.warmup, torch)
    except RuntimeError as err:
        out["ours_graph_replay_ms"] = None
        out["ours_graph_replay_error"] = str(err)[:200]

    # ---- baselines
    logits_gib = args.hq * S * k * S * 2 / 2**30
    Qh = q[j].transpose(0, 1).contiguous().requires_grad_(True)                       # [hq, S, d]
    Kc = torch.cat(kk, 0).transpose(0, 1).contiguous().requires_grad_(True)            # [hkv, kS, d]
    Vc = torch.cat(v, 0).transpose(0, 1).contiguous().requires_grad_(True)
    dOh = d_o[j].transpose(0, 1).contiguous()
    mask = alg2_mask(S, k, j, dev, torch)
    ref_o = run.o[j].transpose(0, 1).float()

    def naive():
        Ke = Kc.repeat_interleave(G, 0)
        Ve = Vc.repeat_interleave(G, 0)
        s = torch.matmul(Qh, Ke.transpose(1, 2)) * wl.scale
        s = s.masked_fill(~mask, float("-inf"))
        p = torch.softmax(s.float(), -1).to(Qh.dtype)
        o = torch.matmul(p, Ve)
        o.backward(dOh)
        Qh.grad = Kc.grad = Vc.grad = None
        return o

    def sdpa():
        o = F.scaled_dot_product_attention(Qh[None], Kc[None], Vc[None], attn_mask=mask, scale=wl.scale,
                                           enable_gqa=True)[0]
        o.backward(dOh)
        Qh.grad = Kc.grad = Vc.grad = None
        return o

    for name, fn in (("naive", naive), ("sdpa", sdpa)):
        if logits_gib > args.baseline_mem_gib:
            out[name] = f"skipped: [hq, S, k*S] bf16 logits alone are {logits_gib:.0f} GiB"
            continue
        try:
            err = float((fn().detach().float() - ref_o).abs().max())
            torch.cuda.synchronize()
            before = torch.cuda.memory_allocated()
            ms, peak = timed(fn, args.steps, args.warmup, torch)
            out[name + "_ms"] = ms
            out[name + "_mem_beyond_inputs_MiB"] = (peak - before) / 2**20 + mask.numel() / 2**20
            out[name + "_max_abs_diff_O"] = err
            out["time_vs_" + name] = ours_ms / ms - 1.0
            out["mem_vs_" + name] = ours_extra / max(peak - before + mask.numel(), 1) - 1.0
        except Exception as e:   # out of memory, or a backend without support for this call
            out[name] = f"failed: {type(e).__name__}: {str(e)[:120]}"
            torch.cuda.empty_cache()
    print(json.dumps(out), flush=True)
    del run, q, kk, v, d_o, Qh, Kc, Vc, dOh, mask, ref_o
    torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
