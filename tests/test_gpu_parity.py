"""GPU parity: the HIP library, called through its C ABI, against the fp64 oracle on the same seeded
inputs.  Small and mid-size cases are compared element by element on every output; the full-size
workloads are compared on sampled rows, with a row-sparse cotangent that lets every dK/dV entry be
checked, and through the gradient invariants, in the launch configuration bench.py times."""
import numpy as np
import pytest
import torch

import oracle as O
from paper_2603_18567_amd.workloads import WORKLOADS, custom_workload
from ttt_testlib import WORST_ROW_RATIO, Case, check, compare_full, dq_row_slack, to_np32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _built():
    O.build_oracle()


def run_all_steps(case):
    case.run.forward()
    case.run.backward(case.d_o)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ element-by-element cases
SMALL = [
    WORKLOADS["tiny_f32"],                                                         # config 1
    custom_workload("bf16_varlen_3docs", "bf16", [130, 1, 169], 4, 2, 128, 3, 7),  # ragged, doc of length 1
    custom_workload("bf16_one_doc_333", "bf16", [333], 8, 2, 128, 4, 8),           # ragged tail, GQA 4
    custom_workload("bf16_tiles_span", "bf16", [257, 300, 64, 191], 8, 8, 128, 2, 9),   # tile/doc boundaries interleave
    custom_workload("bf16_d64", "bf16", [150, 90], 4, 1, 64, 3, 10),
    custom_workload("f32_d128", "f32", [97, 140], 2, 2, 128, 2, 11),
    custom_workload("f32_gqa_ragged", "f32", [70, 3, 200], 6, 3, 64, 4, 12),       # hkv=3: no XCD remap path
    custom_workload("bf16_k1", "bf16", [260], 4, 4, 128, 1, 13),                   # k = 1: plain causal attention
    custom_workload("bf16_len1_docs", "bf16", [1] * 70, 4, 2, 128, 5, 14),         # only diagonal structure
    custom_workload("bf16_empty_docs", "bf16", [0, 40, 0, 0, 90, 0], 2, 1, 128, 3, 15),
    custom_workload("bf16_T1", "bf16", [1], 2, 2, 128, 7, 16),
    custom_workload("bf16_k17", "bf16", [140], 2, 1, 128, 17, 17),                 # longest TTT length the paper studies
    custom_workload("bf16_sharp", "bf16", [400], 4, 2, 128, 3, 18, qk_mult=2.0),   # sharp softmax (long-context recipe)
    custom_workload("bf16_1100", "bf16", [700, 400], 16, 2, 128, 7, 19),           # several tiles in every kernel, G=8
    custom_workload("bf16_k32_max", "bf16", [40], 2, 2, 128, 32, 20),              # the largest step count the ABI takes
    custom_workload("bf16_hkv16", "bf16", [200, 120], 32, 16, 128, 2, 22),         # two kv heads per XCD in the block map
    custom_workload("bf16_d64_multi", "bf16", [500, 333, 100], 8, 2, 64, 4, 23),   # head_dim 64 over several tiles
    custom_workload("f32_multi_tile", "f32", [450, 310], 4, 2, 128, 3, 24),        # fp32 kernels over several tiles
    custom_workload("bf16_gqa3", "bf16", [300, 45, 600], 6, 2, 128, 3, 25),        # 3 query heads per kv head: no head packing
    custom_workload("bf16_hkv3", "bf16", [420, 130], 6, 3, 128, 3, 26),            # hkv neither divides nor is divided by 8
    custom_workload("bf16_hkv5", "bf16", [777], 10, 5, 128, 4, 27),                # the same with an odd head count, 7 key tiles
    custom_workload("bf16_g16", "bf16", [390, 260], 64, 4, 128, 3, 28),            # 16 query heads per kv head (the 235B shape's grouping)
]


@pytest.mark.parametrize("wl", SMALL, ids=lambda w: w.name)
def test_all_outputs_match_oracle(wl):
    print(f"case {wl.name} {wl.dtype} docs={wl.doc_lens} hq={wl.hq} hkv={wl.hkv} d={wl.d} k={wl.k}", flush=True)
    case = Case(wl)
    run_all_steps(case)
    compare_full(case)


def test_outputs_are_fully_overwritten_and_others_untouched():
    wl = custom_workload("overwrite", "bf16", [300], 4, 2, 128, 3, 21)
    case = Case(wl)
    run = case.run
    run.alloc_grads()
    for ts in (run.o, run.dq, run.dk, run.dv):
        for t in ts:
            t.fill_(float("nan"))
    for t in run.lse:
        t.fill_(float("nan"))
    run.forward(0, 2)
    torch.cuda.synchronize()
    assert torch.isnan(run.o[2]).all() and torch.isnan(run.lse[2]).all()
    assert not torch.isnan(run.o[0]).any() and not torch.isnan(run.o[1]).any()
    run.forward(2, 3)
    run.backward(case.d_o, 0, 2)
    torch.cuda.synchronize()
    assert torch.isnan(run.dq[2]).all() and torch.isnan(run.dk[2]).all() and torch.isnan(run.dv[2]).all()
    for l in (0, 1):
        assert not torch.isnan(run.dq[l]).any() and not torch.isnan(run.dk[l]).any() and not torch.isnan(run.dv[l]).any()
    compare_full(case, 0, 2)


# ------------------------------------------------------------------ calling patterns
@pytest.mark.parametrize("wl", [
    custom_workload("steps_bf16", "bf16", [210, 90], 8, 2, 128, 4, 31),
    custom_workload("steps_f32", "f32", [150], 4, 4, 64, 3, 32),
    # k > 8: the sweep's calls for steps >= 8 and < 8 take different preprocess kernels over one carry
    custom_workload("steps_bf16_k12", "bf16", [300, 77], 4, 2, 128, 12, 35),
], ids=lambda w: w.name)
def test_step_at_a_time_equals_all_steps(wl):
    """Training order: k forward calls j = 0..k-1, then k backward calls j = k-1..0 with the fp32
    carry; results must match the oracle like the all-steps call does."""
    case = Case(wl)
    run = case.run
    for j in range(wl.k):
        run.forward(j, j + 1)
    for j in reversed(range(wl.k)):
        run.backward(case.d_o, j, j + 1, accumulate=True)
    torch.cuda.synchronize()
    compare_full(case)
    stepwise = [to_np32(t) for t in run.dk + run.dv + run.dq + run.o]
    run_all_steps(case)
    allsteps = [to_np32(t) for t in run.dk + run.dv + run.dq + run.o]
    scale = max(np.abs(x).max() for x in allsteps)
    for a, b in zip(stepwise, allsteps):
        assert np.abs(a - b).max() <= (1e-5 if wl.dtype == "f32" else 2e-2) * scale


def test_run_twice_is_deterministic_where_no_atomics_meet():
    """Two runs on the same inputs: O, LSE, dQ and the dK_l, dV_l of the blocks l >= 1 have one owner
    each and must come out bit-identical; dK_0, dV_0 are sums of fp32 atomics whose order is not
    fixed, so they may differ in the last bits only."""
    wl = custom_workload("twice", "bf16", [900, 333, 40], 8, 2, 128, 5, 37)
    case = Case(wl)
    run = case.run
    snaps = []
    for _ in range(2):
        for t in run.o + run.lse:
            t.fill_(float("nan"))
        run_all_steps(case)
        snaps.append([t.clone() for t in run.o + run.lse + run.dq + run.dk[1:] + run.dv[1:]] + [run.dk[0].clone(), run.dv[0].clone()])
    for a, b in zip(snaps[0][:-2], snaps[1][:-2]):
        assert torch.equal(a, b)
    for a, b in zip(snaps[0][-2:], snaps[1][-2:]):
        scale = float(b.float().abs().max())
        assert float((a.float() - b.float()).abs().max()) <= 2.0 ** -7 * scale   # one bf16 rounding step of the largest value


def test_final_step_alone_matches_oracle():
    """The call the paper's micro-benchmark times (Sec. 5.4): forward and backward of the LAST step
    only, no carry, TTT length 7 -- every output against the oracle."""
    wl = custom_workload("final_step_1280", "bf16", [1280], 8, 2, 128, 7, 36)
    case = Case(wl)
    case.run.forward(wl.k - 1, wl.k)
    case.run.backward(case.d_o, wl.k - 1, wl.k)
    torch.cuda.synchronize()
    compare_full(case, wl.k - 1, wl.k)


def test_partial_range_without_carry_is_the_sum_over_the_range():
    wl = custom_workload("range", "bf16", [180, 77], 4, 2, 128, 4, 33)
    case = Case(wl)
    case.run.forward()
    case.run.backward(case.d_o, 1, 3)
    torch.cuda.synchronize()
    Q, K, V, dO = case.oracle_inputs()
    _, _, dQo, dKo, dVo = O.oracle_full(Q, K, V, wl.cu_seqlens, wl.scale, dO, 1, 3)
    for n, j in enumerate((1, 2)):
        check(f"dQ[{j}]", to_np32(case.run.dq[j]), dQo[n], wl.dtype)
    for l in range(3):
        check(f"dK[{l}]", to_np32(case.run.dk[l]), dKo[l], wl.dtype)
        check(f"dV[{l}]", to_np32(case.run.dv[l]), dVo[l], wl.dtype)


def test_strided_inputs_and_side_stream():
    """Tensors that are views into larger buffers (non-dense strides), launched on a non-default stream."""
    wl = custom_workload("strided", "bf16", [200, 120], 4, 2, 128, 3, 34)
    dense = Case(wl)
    run_all_steps(dense)
    dev = dense.q[0].device
    T = wl.T

    def widen(ts, heads):
        out = []
        for t in ts:
            buf = torch.zeros((T, heads + 1, wl.d + 8), dtype=t.dtype, device=dev)
            view = buf[:, :heads, :wl.d]
            view.copy_(t)
            out.append(view)
        return out

    from paper_2603_18567_amd import TttAttnRunner
    q, k, v = widen(dense.q, wl.hq), widen(dense.k, wl.hkv), widen(dense.v, wl.hkv)
    run = TttAttnRunner(q, k, v, wl.cu_seqlens, wl.scale, dev)
    run.o = widen(dense.q, wl.hq)            # strided outputs too (same strides as q)
    d_o = widen(dense.d_o, wl.hq)
    run.dq = widen(dense.q, wl.hq); run.dk = widen(dense.k, wl.hkv); run.dv = widen(dense.v, wl.hkv)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        run.forward(stream=s)
        run.backward(d_o, stream=s)
    s.synchronize()
    for a, b in zip(run.o + run.dq + run.dk[1:] + run.dv[1:], dense.run.o + dense.run.dq + dense.run.dk[1:] + dense.run.dv[1:]):
        assert torch.equal(a.contiguous(), b)          # same kernels, same order: bit-identical
    for a, b in zip(run.dk[:1] + run.dv[:1], dense.run.dk[:1] + dense.run.dv[:1]):
        assert (a.float() - b.float()).abs().max() <= 2e-2 * b.float().abs().max()   # fp32 atomics order


# ------------------------------------------------------------------ full-size workloads
def sample_rows(wl, n, seed):
    """Seeded rows that include, for every document, its first and last token and the tokens next to
    the 64/128/256 tile edges, for every step; the rest uniform."""
    rng = np.random.default_rng(seed)
    cu = wl.cu_seqlens
    must = set()
    for a, b in zip(cu[:-1], cu[1:]):
        if b == a:
            continue
        for t in (a, b - 1, a + 1, b - 2):
            if a <= t < b:
                must.add(t)
    for edge in range(64, wl.T, 64):
        if len(must) < n // 2:
            must.update(t for t in (edge - 1, edge) if 0 <= t < wl.T)
    toks = sorted(must)
    rng.shuffle(toks)
    toks = toks[: n // 2]
    rows = [(int(rng.integers(0, wl.k)), t) for t in toks]
    rows += [(wl.k - 1, wl.T - 1), (0, 0)]
    while len(rows) < n:
        rows.append((int(rng.integers(0, wl.k)), int(rng.integers(0, wl.T))))
    rows = sorted(set(rows))
    return np.array([r[0] for r in rows], dtype=np.int32), np.array([r[1] for r in rows], dtype=np.int32)


def device_invariants(case):
    """Shift / scale / mass invariants of the gradients, evaluated in fp64 on the device outputs."""
    wl, run = case.wl, case.run
    G = wl.hq // wl.hkv
    f64 = lambda t: t.to(torch.float64)
    for a, b in zip(wl.cu_seqlens[:-1], wl.cu_seqlens[1:]):
        if b == a:
            continue
        sum_dk = sum(f64(run.dk[l][a:b]).sum(0) for l in range(wl.k))                  # [hkv,d]
        abs_dk = sum(f64(run.dk[l][a:b]).abs().sum(0) for l in range(wl.k))
        sum_dv = sum(f64(run.dv[l][a:b]).sum(0) for l in range(wl.k))
        sum_do = sum(f64(case.d_o[j][a:b]).sum(0) for j in range(wl.k)).view(wl.hkv, G, wl.d).sum(1)
        abs_do = sum(f64(case.d_o[j][a:b]).abs().sum(0) for j in range(wl.k)).view(wl.hkv, G, wl.d).sum(1)
        qdq = sum((f64(case.q[j][a:b]) * f64(run.dq[j][a:b])).sum((0, 2)) for j in range(wl.k)).view(wl.hkv, G).sum(1)
        kdk = sum((f64(case.k[l][a:b]) * f64(run.dk[l][a:b])).sum((0, 2)) for l in range(wl.k))
        abs_qdq = sum((f64(case.q[j][a:b]) * f64(run.dq[j][a:b])).abs().sum((0, 2)) for j in range(wl.k)).view(wl.hkv, G).sum(1)
        # outputs are rounded to bf16 (rel 2^-9 each, independent), sums of n terms: allow a few 1e-3 of the abs mass
        assert (sum_dk.abs() <= 4e-3 * abs_dk + 1e-6).all(), "shift invariant (sum of dK over a document)"
        assert ((sum_dv - sum_do).abs() <= 4e-3 * abs_do + 1e-6).all(), "mass invariant (sum dV = sum dO)"
        assert ((qdq - kdk).abs() <= 4e-3 * abs_qdq + 1e-6).all(), "scale invariant (<Q,dQ> = <K,dK>)"


BIG = {"llama8b_2k": 1600, "headline_4k": 1600, "varlen_16k": 480, "qwen235b_8k": 416, "long_32k": 400}


@pytest.mark.parametrize("name", list(BIG), ids=str)
def test_full_size_workload_sampled_rows_and_invariants(name):
    wl = WORKLOADS[name]
    print(f"workload {name}: T={wl.T} docs={len(wl.doc_lens)} hq={wl.hq} hkv={wl.hkv} k={wl.k}", flush=True)
    case = Case(wl)
    run = case.run
    run_all_steps(case)                                  # dense cotangent, bench.py's launch configuration
    print("  dense run done", flush=True)
    device_invariants(case)
    print("  invariants ok", flush=True)
    rs, rt = sample_rows(wl, BIG[name], wl.seed)
    Q, K, V, _ = case.oracle_inputs()
    dO_rows = np.stack([case.inp.d_o[j][i].to(torch.float32).numpy() for j, i in zip(rs, rt)])
    ref = O.oracle_run(Q, K, V, wl.cu_seqlens, wl.scale, rs, rt, dO_rows)
    slack = dq_row_slack(dO_rows, ref.O, O.oracle_run(Q, K, K, wl.cu_seqlens, wl.scale, rs, rt).O, wl.scale)
    print(f"  oracle on {len(rs)} rows done", flush=True)
    got_O = np.stack([to_np32(run.o[j][i]) for j, i in zip(rs, rt)])
    got_L = np.stack([to_np32(run.lse[j][:, i]) for j, i in zip(rs, rt)])
    got_dQ = np.stack([to_np32(run.dq[j][i]) for j, i in zip(rs, rt)])
    WORST_ROW_RATIO.clear()
    check("O rows", got_O, ref.O, wl.dtype, rows=True)
    check("LSE rows", got_L, ref.LSE, wl.dtype, lse=True)
    check("dQ rows", got_dQ, ref.dQ, wl.dtype, rows=True, row_slack=slack)
    print(f"  worst per-row error / per-row bound: {WORST_ROW_RATIO}", flush=True)
    # second backward with a cotangent that is zero off the sampled rows: linear in dO, same kernel
    # work, and the oracle's sums over the listed rows are then the complete dK, dV
    sparse = [torch.zeros_like(t) for t in case.d_o]
    for j, i in zip(rs, rt):
        sparse[j][i] = case.d_o[j][i]
    run.backward(sparse)
    torch.cuda.synchronize()
    for l in range(wl.k):
        check(f"dK[{l}] (row-sparse dO)", to_np32(run.dk[l]), ref.dK[l], wl.dtype)
        check(f"dV[{l}] (row-sparse dO)", to_np32(run.dv[l]), ref.dV[l], wl.dtype)
    keep = torch.zeros((wl.k, wl.T), dtype=torch.bool)
    keep[torch.as_tensor(rs, dtype=torch.long), torch.as_tensor(rt, dtype=torch.long)] = True
    for j in range(wl.k):
        off = run.dq[j][~keep[j].to(run.dq[j].device)]
        assert (off == 0).all(), "dQ must vanish where the cotangent row is zero"
    got_dQ2 = np.stack([to_np32(run.dq[j][i]) for j, i in zip(rs, rt)])
    check("dQ rows (row-sparse dO)", got_dQ2, ref.dQ, wl.dtype, rows=True, row_slack=slack)
