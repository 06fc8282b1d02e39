"""Per-document TTT step counts: the docsteps entry points against the fp64 oracle restricted to
the active (step, token) rows -- which is exactly the method with a row-sparse cotangent -- and the
promise that inactive (step, document) combinations are neither read nor written."""
import numpy as np
import pytest
import torch

import oracle as O
from paper_2603_18567_amd.workloads import custom_workload
from ttt_testlib import Case, check, to_np32

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
