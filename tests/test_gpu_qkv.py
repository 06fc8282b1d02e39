"""GPU parity of the QKV projection + rotary embedding producer against its fp64 oracle, element by
element, through the C ABI: ragged token and head tiles, an odd number of contraction slices,
strided operand rows, positions out of range, and sampled rows at the draft-layer shape."""
import math
import os
import sys

import numpy as np
import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
from oracle.qkv_oracle import qkv_rope, rope_tables   # noqa: E402

pytestmark = pytest.mark.gpu

# The operands are given in bf16 and taken exactly by both sides; products are exact in fp32 and
# their fp32 accumulation over hidden_in terms errs by ~sqrt(hidden_in) * 2^-24 relative, far below
# the single rounding of the result to bf16: 2^-9 relative to a value no larger than max|ref|
# (a rotation does not lengthen a pair).  2^-8 * max|ref| leaves a factor two.
TOL = 2.0 ** -8


def make(T, hin, hq, hkv, d, seed, n_pos=4096, x_pad=0, w_pad=0):
    gen = torch.Generator().manual_seed(seed)
    x = torch.randn(T, hin + x_pad, generator=gen).to(torch.bfloat16)
    w = (torch.randn((hq + 2 * hkv) * d, hin + w_pad, generator=gen) / math.sqrt(hin)).to(torch.bfloat16)
    pos = torch.randint(0, n_pos, (T,), generator=gen, dtype=torch.int32)
    cos64, sin64 = rope_tables(n_pos, d)
    cos_t = torch.from_numpy(cos64).to(torch.float32)
    sin_t = torch.from_numpy(sin64).to(torch.float32)
    return x, w, pos, cos_t, sin_t


def run_gpu(x, w, pos, cos_t, sin_t, hq, hkv, d, hin):
    from paper_2603_18567_amd import binding
    dev = torch.device("cuda:0")
    T = x.shape[0]
    xd, wd = x.to(dev)[:, :hin], w.to(dev)[:, :hin]
    q = torch.full((T, hq, d), float("nan"), dtype=torch.bfloat16, device=dev)
    k = torch.full((T, hkv, d), float("nan"), dtype=torch.bfloat16, device=dev)
    v = torch.full((T, hkv, d), float("nan"), dtype=torch.bfloat16, device=dev)
    binding.ttt_qkv_rope_fwd(xd, wd, cos_t.to(dev), sin_t.to(dev), pos.to(dev), q, k, v)
    torch.cuda.synchronize()
    return q.float().cpu().numpy(), k.float().cpu().numpy(), v.float().cpu().numpy()


def check(got, ref, name):
    assert np.isfinite(got).all(), f"{name}: non-finite or unwritten values"
    bound = TOL * np.abs(ref).max()
    err = np.abs(got - ref).max()
    assert err <= bound, f"{name}: max abs err {err:.3e} > bound {bound:.3e}"


CASES = [
    # name, T, hidden_in, hq, hkv, x_pad, w_pad
    ("one_tile_ragged", 300, 128, 3, 1, 0, 0),            # 5 heads: the last feature tile holds one head
    ("several_tiles_odd_slices", 700, 320, 4, 2, 0, 0),   # 3 token tiles (ragged), 4 feature tiles, 5 slices
    ("strided_rows", 257, 192, 2, 2, 64, 8),
    ("single_token", 1, 64, 1, 1, 0, 0),
    ("gqa_draft_heads_short", 512, 256, 32, 8, 0, 0),     # 48 heads = 24 feature tiles
    ("large_token_tiles_ragged", 4000, 64, 24, 4, 0, 0),  # 16 x 16 tiles of 256 tokens fill the device in one
                                                          # round: the 256-token variant, last tile ragged
]


@pytest.mark.parametrize("name,T,hin,hq,hkv,x_pad,w_pad", CASES, ids=[c[0] for c in CASES])
def test_producer_matches_oracle(name, T, hin, hq, hkv, x_pad, w_pad):
    d = 128
    print(f"case {name} T={T} hidden_in={hin} hq={hq} hkv={hkv}", flush=True)
    x, w, pos, cos_t, sin_t = make(T, hin, hq, hkv, d, seed=100 + T, x_pad=x_pad, w_pad=w_pad)
    q, k, v = run_gpu(x, w, pos, cos_t, sin_t, hq, hkv, d, hin)
    rq, rk, rv = qkv_rope(x[:, :hin].float().numpy(), w[:, :hin].float().numpy(), cos_t.numpy(), sin_t.numpy(),
                          pos.numpy(), hq, hkv, d)
    check(q, rq, "Q")
    check(k, rk, "K")
    check(v, rv, "V")


def test_positions_out_of_range_are_clamped_and_no_tokens_is_a_noop():
    from paper_2603_18567_amd import binding
    d, hq, hkv, hin, T = 128, 2, 1, 64, 40
    x, w, pos, cos_t, sin_t = make(T, hin, hq, hkv, d, seed=9, n_pos=16)
    pos[3] = -5
    pos[7] = 1000
    q, k, v = run_gpu(x, w, pos, cos_t, sin_t, hq, hkv, d, hin)
    rq, rk, rv = qkv_rope(x.float().numpy(), w.float().numpy(), cos_t.numpy(), sin_t.numpy(),
                          np.clip(pos.numpy(), 0, 15), hq, hkv, d)
    check(q, rq, "Q")
    check(k, rk, "K")
    dev = torch.device("cuda:0")
    e = torch.empty(0, hin, dtype=torch.bfloat16, device=dev)
    binding.ttt_qkv_rope_fwd(e, w.to(dev), cos_t.to(dev), sin_t.to(dev), torch.empty(0, dtype=torch.int32, device=dev),
                             torch.empty(0, hq, d, dtype=torch.bfloat16, device=dev),
                             torch.empty(0, hkv, d, dtype=torch.bfloat16, device=dev),
                             torch.empty(0, hkv, d, dtype=torch.bfloat16, device=dev))


def test_argument_errors():
    from paper_2603_18567_amd import binding
    dev = torch.device("cuda:0")
    bf = dict(dtype=torch.bfloat16, device=dev)
    cos_t = torch.ones(4, 64, device=dev)
    pos = torch.zeros(8, dtype=torch.int32, device=dev)
    with pytest.raises(binding.TttAttnError):      # hidden_in not a multiple of 64
        binding.ttt_qkv_rope_fwd(torch.zeros(8, 96, **bf), torch.zeros(3 * 128, 96, **bf), cos_t, cos_t, pos,
                                 torch.zeros(8, 1, 128, **bf), torch.zeros(8, 1, 128, **bf), torch.zeros(8, 1, 128, **bf))
    with pytest.raises(binding.TttAttnError):      # head_dim 64 is not built
        binding.ttt_qkv_rope_fwd(torch.zeros(8, 64, **bf), torch.zeros(3 * 64, 64, **bf), torch.ones(4, 32, device=dev),
                                 torch.ones(4, 32, device=dev), pos, torch.zeros(8, 1, 64, **bf), torch.zeros(8, 1, 64, **bf),
                                 torch.zeros(8, 1, 64, **bf))


def test_draft_layer_shape_sampled_tokens():
    """T = 4096 tokens, hidden_in = 8192 (token embedding and target hidden state side by side), 32 + 8 + 8
    heads of 128: the launch bench_qkv_rope.py times.  The oracle computes 48 sampled tokens."""
    d, hq, hkv, hin, T = 128, 32, 8, 8192, 4096
    x, w, pos, cos_t, sin_t = make(T, hin, hq, hkv, d, seed=77)
    q, k, v = run_gpu(x, w, pos, cos_t, sin_t, hq, hkv, d, hin)
    rows = np.random.default_rng(3).choice(T, 48, replace=False)
    rows[:4] = [0, 255, 256, T - 1]
    rq, rk, rv = qkv_rope(x[rows].float().numpy(), w.float().numpy(), cos_t.numpy(), sin_t.numpy(), pos[rows].numpy(),
                          hq, hkv, d)
    check(q[rows], rq, "Q")
    check(k[rows], rk, "K")
    check(v[rows], rv, "V")
    assert np.isfinite(q).all() and np.isfinite(k).all() and np.isfinite(v).all()


O_CASES = [
    # name, T, hq, out_features, o_pad, w_pad
    ("o_small_ragged", 300, 2, 384, 0, 0),          # 3 half-tiles of features: the last feature tile holds one
    ("o_strided", 520, 4, 256, 128, 8),
    ("o_draft_layer_rows", 4096, 32, 4096, 0, 0),   # the draft layer's shape (sampled tokens below)
]


@pytest.mark.parametrize("name,T,hq,nout,o_pad,w_pad", O_CASES, ids=[c[0] for c in O_CASES])
def test_output_projection_matches_oracle(name, T, hq, nout, o_pad, w_pad):
    from oracle.qkv_oracle import o_proj
    from paper_2603_18567_amd import binding
    d = 128
    fin = hq * d
    print(f"case {name} T={T} in={fin} out={nout}", flush=True)
    gen = torch.Generator().manual_seed(500 + T)
    o = torch.randn(T, fin + o_pad, generator=gen).to(torch.bfloat16)
    w = (torch.randn(nout, fin + w_pad, generator=gen) / math.sqrt(fin)).to(torch.bfloat16)
    dev = torch.device("cuda:0")
    out = torch.full((T, nout), float("nan"), dtype=torch.bfloat16, device=dev)
    binding.ttt_o_proj_fwd(o.to(dev)[:, :fin], w.to(dev)[:, :fin], out)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    rows = np.arange(T) if T <= 1024 else np.concatenate([[0, 255, 256, T - 1], np.random.default_rng(4).choice(T, 60, replace=False)])
    ref = o_proj(o[rows, :fin].float().numpy(), w[:, :fin].float().numpy())
    check(got[rows], ref, "out")
    assert np.isfinite(got).all()


def test_output_projection_argument_errors():
    from paper_2603_18567_amd import binding
    dev = torch.device("cuda:0")
    bf = dict(dtype=torch.bfloat16, device=dev)
    with pytest.raises(binding.TttAttnError):      # out_features not a multiple of 128
        binding.ttt_o_proj_fwd(torch.zeros(8, 128, **bf), torch.zeros(100, 128, **bf), torch.zeros(8, 100, **bf))
    with pytest.raises(binding.TttAttnError):      # in_features not a multiple of 64
        binding.ttt_o_proj_fwd(torch.zeros(8, 96, **bf), torch.zeros(128, 96, **bf), torch.zeros(8, 128, **bf))
