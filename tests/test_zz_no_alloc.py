"""The workspace-free forward entry point (for callers that cannot allocate device memory) against
the ordinary forward, through the C ABI: two calls in a row on the shared built-in scratch, the
second with a smaller input."""
import pytest
import torch

from paper_2603_18567_amd import binding as B
from paper_2603_18567_amd.workloads import custom_workload
from ttt_testlib import Case, check, to_np32

pytestmark = pytest.mark.gpu


def _both_ways(wl):
    case = Case(wl)
    run = case.run
    run.forward()                                     # existing entry point, caller-owned workspace
    torch.cuda.synchronize()
    ref_o = [t.clone() for t in run.o]
    ref_lse = [t.clone() for t in run.lse]
    for t in run.o + run.lse:
        t.fill_(float("nan"))
    B.ttt_attn_fwd_static(run.params(), run.q, run.k, run.v, run.cu_dev, run.cu_host, run.o, run.lse)
    torch.cuda.synchronize()
    for j in range(wl.k):
        check(f"O[{j}]", to_np32(run.o[j]), to_np32(ref_o[j]).astype("float64"), wl.dtype, rows=True)
        check(f"LSE[{j}]", to_np32(run.lse[j]), to_np32(ref_lse[j]).astype("float64"), wl.dtype, lse=True)
        # the same kernels on the same inputs, no atomics in the forward: the results are identical
        assert torch.equal(run.o[j], ref_o[j]) and torch.equal(run.lse[j], ref_lse[j])


def test_static_scratch_forward_twice_second_call_smaller():
    print("case static_large: 3 documents, 1500 tokens", flush=True)
    _both_ways(custom_workload("static_large", "bf16", [700, 1, 799], 8, 2, 128, 4, 41))
    print("case static_small: 2 documents, 190 tokens", flush=True)
    _both_ways(custom_workload("static_small", "bf16", [130, 60], 4, 2, 128, 3, 42))


def test_static_scratch_forward_rejects_more_tokens_than_the_scratch_holds():
    wl = custom_workload("static_reject", "bf16", [64], 2, 1, 128, 2, 43)
    case = Case(wl)
    run = case.run
    p = run.params()
    p.total_tokens = B.TTT_STATIC_MAX_TOKENS + 1
    cu_host = [0, B.TTT_STATIC_MAX_TOKENS + 1]
    with pytest.raises(B.TttAttnError) as ei:
        B.ttt_attn_fwd_static(p, run.q, run.k, run.v, run.cu_dev, cu_host, run.o, run.lse)
    assert ei.value.code == B.TTT_ERR_WORKSPACE and "TTT_STATIC_MAX_TOKENS" in str(ei.value)
