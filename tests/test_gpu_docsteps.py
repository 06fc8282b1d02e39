"""Per-document TTT step counts: the docsteps entry points against the fp64 oracle restricted to
the active (step, token) rows -- which is exactly the method with a row-sparse cotangent -- and the
promise that inactive (step, document) combinations are neither read nor written."""
import numpy as np
import pytest
import torch

import oracle as O
from paper_2603_18567_amd.workloads import custom_workload
from ttt_testlib import Case, check, dq_row_slack, to_np32

pytestmark = pytest.mark.gpu

CASES = [
    # (workload, steps per document)
    (custom_workload("ds_bf16_mixed", "bf16", [150, 40, 1, 260, 90], 8, 2, 128, 5, 31), [5, 2, 2, 0, 3]),
    (custom_workload("ds_bf16_all_equal", "bf16", [130, 200], 4, 2, 128, 3, 32), [3, 3]),
    (custom_workload("ds_f32_mixed", "f32", [70, 33, 120], 4, 4, 64, 4, 33), [1, 4, 2]),
    (custom_workload("ds_bf16_empty_docs", "bf16", [0, 64, 0, 100], 2, 1, 128, 4, 34), [4, 1, 0, 4]),
]


@pytest.mark.parametrize("wl,steps", CASES, ids=[c[0].name for c in CASES])
def test_docsteps_match_oracle_and_leave_the_rest_alone(wl, steps):
    print(f"case {wl.name}: docs={wl.doc_lens} steps={steps} k={wl.k}", flush=True)
    O.build_oracle()
    case = Case(wl)
    run = case.run
    run.alloc_grads()
    SENT = 7.5   # representable in bf16
    for ts in (run.o, run.dq, run.dk, run.dv, run.lse):
        for t in ts:
            t.fill_(SENT)
    run.forward_docsteps(steps)
    run.backward_docsteps(case.d_o, steps)
    torch.cuda.synchronize()

    cu = wl.cu_seqlens
    tok_steps = np.zeros(wl.T, dtype=np.int32)
    for r, kr in enumerate(steps):
        tok_steps[cu[r]:cu[r + 1]] = kr
    rows = [(j, i) for j in range(wl.k) for i in range(wl.T) if j < tok_steps[i]]
    row_step = np.array([r[0] for r in rows], dtype=np.int32)
    row_tok = np.array([r[1] for r in rows], dtype=np.int32)
    Q, K, V, dO = case.oracle_inputs()
    res = O.oracle_run(Q, K, V, cu, wl.scale, row_step, row_tok, dO[row_step, row_tok])

    o = np.stack([to_np32(t) for t in run.o])          # [k, T, hq, d]
    dq = np.stack([to_np32(t) for t in run.dq])
    lse = np.stack([to_np32(t) for t in run.lse])      # [k, hq, T]
    dk = np.stack([to_np32(t) for t in run.dk])
    dv = np.stack([to_np32(t) for t in run.dv])
    act = np.zeros((wl.k, wl.T), dtype=bool)
    act[row_step, row_tok] = True
    if len(rows):
        check("O (active rows)", o[row_step, row_tok], res.O, wl.dtype)
        check("LSE (active rows)", lse[row_step, :, row_tok], res.LSE, wl.dtype, lse=True)
        check("dQ (active rows)", dq[row_step, row_tok], res.dQ, wl.dtype)
        check("dK (existing keys)", dk[act], res.dK[act], wl.dtype)
        check("dV (existing keys)", dv[act], res.dV[act], wl.dtype)
    # nothing else was written
    assert np.all(o[~act] == SENT) and np.all(dq[~act] == SENT)
    assert np.all(dk[~act] == SENT) and np.all(dv[~act] == SENT)
    assert np.all(np.transpose(lse, (0, 2, 1))[~act] == SENT)


def test_docsteps_argument_errors():
    from paper_2603_18567_amd import binding as B
    wl = custom_workload("ds_err", "bf16", [40, 40], 2, 1, 128, 3, 35)
    case = Case(wl)
    with pytest.raises(B.TttAttnError):
        case.run.forward_docsteps([4, 1])          # more steps than k
    with pytest.raises(B.TttAttnError):
        case.run.forward_docsteps([-1, 1])


def test_docsteps_on_the_packed_varlen_workload():
    """Per-document step counts at full size (the 16384-token packed batch, 9 documents): sampled
    active rows against the oracle, every dK/dV entry through a row-sparse cotangent, and the
    inactive (step, document) combinations untouched."""
    from paper_2603_18567_amd.workloads import WORKLOADS
    wl = WORKLOADS["varlen_16k"]
    n_docs = len(wl.doc_lens)
    steps = [(7, 3, 5, 7, 1, 0, 4, 7, 2)[r % 9] for r in range(n_docs)]
    print(f"workload {wl.name}: docs={wl.doc_lens} steps={steps}", flush=True)
    O.build_oracle()
    case = Case(wl)
    run = case.run
    run.alloc_grads()
    SENT = 7.5
    for ts in (run.o, run.dq, run.dk, run.dv, run.lse):
        for t in ts:
            t.fill_(SENT)
    run.forward_docsteps(steps)
    run.backward_docsteps(case.d_o, steps)
    torch.cuda.synchronize()
    print("  dense run done", flush=True)

    cu = wl.cu_seqlens
    tok_steps = np.zeros(wl.T, dtype=np.int64)
    for r, kr in enumerate(steps):
        tok_steps[cu[r]:cu[r + 1]] = kr
    act = torch.from_numpy(np.arange(wl.k)[:, None] < tok_steps[None, :])     # [k, T]
    rng = np.random.default_rng(wl.seed + 1)
    rows = set()
    for r, kr in enumerate(steps):                       # first / last token of every active document, every step
        if kr == 0 or cu[r + 1] == cu[r]:
            continue
        for j in range(kr):
            rows.add((j, cu[r]))
            rows.add((j, cu[r + 1] - 1))
    while len(rows) < 320:
        i = int(rng.integers(0, wl.T))
        if tok_steps[i] > 0:
            rows.add((int(rng.integers(0, tok_steps[i])), i))
    rows = sorted(rows)
    rs = np.array([r[0] for r in rows], dtype=np.int32)
    rt = np.array([r[1] for r in rows], dtype=np.int32)
    Q, K, V, _ = case.oracle_inputs()
    dO_rows = np.stack([case.inp.d_o[j][i].to(torch.float32).numpy() for j, i in zip(rs, rt)])
    ref = O.oracle_run(Q, K, V, cu, wl.scale, rs, rt, dO_rows)
    print(f"  oracle on {len(rows)} rows done", flush=True)
    check("O rows", np.stack([to_np32(run.o[j][i]) for j, i in zip(rs, rt)]), ref.O, wl.dtype, rows=True)
    check("LSE rows", np.stack([to_np32(run.lse[j][:, i]) for j, i in zip(rs, rt)]), ref.LSE, wl.dtype, lse=True)
    slack = dq_row_slack(dO_rows, ref.O, O.oracle_run(Q, K, K, cu, wl.scale, rs, rt).O, wl.scale)
    check("dQ rows", np.stack([to_np32(run.dq[j][i]) for j, i in zip(rs, rt)]), ref.dQ, wl.dtype, rows=True, row_slack=slack)
    dev = run.o[0].device
    for j in range(wl.k):
        off = ~act[j].to(dev)
        assert (run.o[j][off] == SENT).all() and (run.dq[j][off] == SENT).all() and (run.lse[j][:, off] == SENT).all()
        assert (run.dk[j][off] == SENT).all() and (run.dv[j][off] == SENT).all()

    sparse = [torch.zeros_like(t) for t in case.d_o]
    for j, i in zip(rs, rt):
        sparse[j][i] = case.d_o[j][i]
    run.backward_docsteps(sparse, steps)
    torch.cuda.synchronize()
    for l in range(wl.k):
        on = act[l].to(dev)
        check(f"dK[{l}] (row-sparse dO)", to_np32(run.dk[l][on]), ref.dK[l][act[l].numpy()], wl.dtype)
        check(f"dV[{l}] (row-sparse dO)", to_np32(run.dv[l][on]), ref.dV[l][act[l].numpy()], wl.dtype)
        assert (run.dk[l][~on] == SENT).all() and (run.dv[l][~on] == SENT).all()
