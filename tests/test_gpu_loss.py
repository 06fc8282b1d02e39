"""GPU parity of the in-place log-softmax-loss backward (Alg. 3) against the fp64 oracle, element by
element, through the C ABI: vectorised and element-wise paths, register-cached and streamed rows,
ragged vocabulary sizes, strided rows, masked rows (g = 0)."""
import os
import sys

import numpy as np
import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
from oracle.loss_oracle import logsoftmax_loss_bwd   # noqa: E402

# fp32: the result is O(|g|); exp2 and the V-term sums carry a few fp32 ulps each.
# bf16: one rounding of the output (2^-9 relative) plus the rounding of nothing else (inputs are
# given rounded); elements where p*g and pi*s cancel are bounded relative to the row maximum.
TOL = {torch.float32: 2e-5, torch.bfloat16: 2e-2}


def make(n, v, dtype, seed, stride_pad=0):
    gen = torch.Generator().manual_seed(seed)
    z = (torch.randn(n, v + stride_pad, generator=gen) * 3).to(dtype)
    p = torch.rand(n, v + stride_pad, generator=gen) ** 6
    p = (p / p[:, :v].sum(1, keepdim=True)).to(dtype)
    g = torch.randn(n, generator=gen)
    if n > 2:
        g[1] = 0.0                     # a masked position
    return z, p, g


CASES = [   # name, rows, vocabulary, dtype, stride padding; the position in this list + 500 is the seed
    ("f32_small", 7, 1000, torch.float32, 0),
    ("f32_draft_vocab", 5, 32000, torch.float32, 0),
    ("bf16_draft_vocab", 5, 32000, torch.bfloat16, 0),
    ("f32_ragged_unaligned", 4, 4099, torch.float32, 0),        # vocab not a multiple of the vector width
    ("bf16_ragged", 4, 50257, torch.bfloat16, 0),
    ("f32_strided_rows", 6, 2048, torch.float32, 64),
    ("f32_odd_stride_elementwise", 3, 777, torch.float32, 3),   # stride not 16-byte aligned: element path
    ("f32_streamed_long_row", 3, 70001, torch.float32, 0),      # beyond the register cache
    ("bf16_streamed_long_row", 2, 151936, torch.bfloat16, 0),
    ("f32_vocab_1", 3, 1, torch.float32, 0),
]


@pytest.mark.gpu
@pytest.mark.parametrize("seed,name,n,v,dtype,pad", [(500 + i, *c) for i, c in enumerate(CASES)], ids=[c[0] for c in CASES])
def test_loss_backward_matches_oracle(seed, name, n, v, dtype, pad):
    from paper_2603_18567_amd import binding as B
    print(f"case {name}: rows={n} vocab={v} dtype={dtype} stride_pad={pad} seed={seed}", flush=True)
    z, p, g = make(n, v, dtype, seed=seed, stride_pad=pad)
    ref = logsoftmax_loss_bwd(z[:, :v].float().numpy(), p[:, :v].float().numpy(), g.numpy())
    dev = torch.device("cuda:0")
    zd, pd, gd = z.to(dev), p.to(dev), g.to(dev)
    p_before = pd.clone()
    B.ttt_loss_bwd_inplace(zd[:, :v], pd[:, :v], gd)
    torch.cuda.synchronize()
    got = zd[:, :v].float().cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    err = np.abs(got - ref).max()
    # every element is the difference of the two terms p*g and pi*s: the error is relative to them
    # (a one-entry vocabulary makes them cancel exactly: the reference is identically zero)
    terms = np.abs(p[:, :v].double().numpy() * g.double().numpy()[:, None]).max()
    bound = TOL[dtype] * max(np.abs(ref).max(), terms, 1e-30)
    assert err <= bound, f"max abs err {err:.3e} > {bound:.3e}"
    if n > 2:
        assert np.all(got[1] == 0.0), "a row with g = 0 must become exactly zero"
    assert torch.equal(pd, p_before), "the target must not be written"
    if pad:
        assert torch.equal(zd[:, v:].cpu(), z[:, v:]), "columns past the vocabulary must not be touched"


@pytest.mark.gpu
def test_loss_backward_no_rows_and_bad_arguments():
    from paper_2603_18567_amd import binding as B
    dev = torch.device("cuda:0")
    z = torch.zeros(0, 16, device=dev)
    B.ttt_loss_bwd_inplace(z, z.clone(), torch.zeros(0, device=dev))      # no-op
    lib = B.load_library()
    assert lib.ttt_loss_bwd_inplace(None, None, None, 4, 0, 16, 16, B.TTT_F32, None) == B.TTT_ERR_INVALID_ARG
    assert lib.ttt_loss_bwd_inplace(None, None, None, 4, 16, 8, 16, B.TTT_F32, None) == B.TTT_ERR_INVALID_ARG
    assert lib.ttt_loss_bwd_inplace(None, None, None, 4, 16, 16, 16, 7, None) == B.TTT_ERR_UNSUPPORTED
    assert lib.ttt_loss_bwd_inplace(None, None, None, 4, 16, 16, 16, B.TTT_F32, None) == B.TTT_ERR_INVALID_ARG
