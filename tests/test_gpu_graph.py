"""The library's calls inside a captured HIP graph: they allocate nothing, never synchronise and clear
their accumulators with a fill kernel (no memset node), so the training-order pattern of Sec. 2.4
(k forward calls, then k backward calls in descending order with the fp32 carry) can be recorded
once and replayed.  Every replay is checked against the oracle and against the eager result, with
eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2603_18567_amd.workloads import custom_workload
from ttt_testlib import Case, compare_full, to_np32

pytestmark = pytest.mark.gpu


def _stepwise(case, stream=None):
    wl, run = case.wl, case.run
    for j in range(wl.k):
        run.forward(j, j + 1, stream=stream)
    for j in reversed(range(wl.k)):
        run.backward(case.d_o, j, j + 1, accumulate=True, stream=stream)


def test_training_order_replayed_from_a_graph():
    wl = custom_workload("graph_bf16", "bf16", [300, 45, 131], 8, 2, 128, 4, 41)
    case = Case(wl)
    run = case.run
    _stepwise(case)                      # eager: allocates outputs and workspaces, sets kernel attributes
    torch.cuda.synchronize()
    compare_full(case)
    outs = lambda: run.o + run.lse + run.dq + run.dk + run.dv
    eager = [t.clone() for t in outs()]

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        _stepwise(case)                  # the binding takes torch's current stream: the capturing one
    torch.cuda.synchronize()

    n_exact = len(run.o) + len(run.lse) + len(run.dq)
    for replay in range(3):
        for t in outs():                 # eager work between the replays: poison every output
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        compare_full(case)
        got = outs()
        for a, b in zip(got[:n_exact], eager[:n_exact]):
            assert torch.equal(a, b), f"replay {replay}: O / LSE / dQ differ from the eager call"
        for a, b in zip(got[n_exact:], eager[n_exact:]):       # dK, dV: fp32 atomics in any order
            scale = float(b.float().abs().max())
            assert float((a.float() - b.float()).abs().max()) <= 2e-2 * scale + 1e-5
        if replay == 1:                  # an eager call between two replays must not disturb the next one
            run.forward()
            run.backward(case.d_o)
            torch.cuda.synchronize()
