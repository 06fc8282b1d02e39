"""Seeded synthetic workloads for TTT attention.

Shapes, document structure and value distributions only: this module holds none of the method's
arithmetic and is the one piece shared by the GPU tests/benchmark and the CPU oracle's tests.
The attention operator never sees the content of the paper's chat corpora (Sec. 6), only sequence
lengths and head geometry, so seeded Gaussian tensors of the stated shapes stand in for them.

Every tensor is drawn on the CPU with torch.Generator(seed) as fp32 N(0,1) (times `qk_mult` for
Q and K), then rounded once to the workload dtype; both sides receive the rounded values.
"""
from __future__ import annotations

import math
import random
from dataclasses import dataclass, field

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                 # "f32" | "bf16"
    doc_lens: tuple            # document lengths, packed in this order
    hq: int
    hkv: int
    d: int
    k: int
    seed: int
    qk_mult: float = 1.0       # Q and K are N(0,1) * qk_mult
    note: str = ""

    @property
    def T(self) -> int:
        return int(sum(self.doc_lens))

    @property
    def cu_seqlens(self) -> list:
        cu = [0]
        for L in self.doc_lens:
            cu.append(cu[-1] + int(L))
        return cu

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d)

    @property
    def torch_dtype(self):
        return {"f32": torch.float32, "bf16": torch.bfloat16}[self.dtype]

    @property
    def elem_bytes(self) -> int:
        return {"f32": 4, "bf16": 2}[self.dtype]

    def pairs(self) -> int:
        """Visible (query, key) pairs times query heads: causal prefix plus j diagonal keys."""
        k = self.k
        return self.hq * sum(k * L * (L + 1) // 2 + L * k * (k - 1) // 2 for L in self.doc_lens)

    def useful_flops(self) -> dict:
        p = self.pairs()
        return {"fwd": 4 * self.d * p, "bwd": 10 * self.d * p, "fwd_bwd": 14 * self.d * p}


def varlen_doc_lens(total: int, lo: int, hi: int, seed: int) -> tuple:
    """Lengths iid uniform in [lo,hi] until the sum reaches `total`; the last is clipped to fit and
    the whole list is redrawn if the clipped last one is shorter than `lo`."""
    rng = random.Random(seed)
    while True:
        lens, s = [], 0
        while s < total:
            L = rng.randint(lo, hi)
            L = min(L, total - s)
            lens.append(L)
            s += L
        if lens[-1] >= lo:
            return tuple(lens)


WORKLOADS = {w.name: w for w in [
    Workload("tiny_f32", "f32", (128,), 4, 4, 64, 3, seed=1235,
             note="tiny fp32 case: S=128, Hq=Hkv=4, d=64, k=3, one document"),
    Workload("llama8b_2k", "bf16", (2048,), 32, 8, 128, 7, seed=1236,
             note="Llama-3.1-8B-shaped draft layer, S=2048"),
    Workload("varlen_16k", "bf16", varlen_doc_lens(16384, 256, 4096, 1237), 32, 8, 128, 7, seed=1237,
             note="packed varlen batch, 16384 tokens, lengths uniform in [256,4096]"),
    Workload("qwen235b_8k", "bf16", (8192, 8192), 64, 4, 128, 7, seed=1238,
             note="Qwen3-235B-A22B-shaped draft layer, B=2, S=8192"),
    Workload("long_32k", "bf16", (32768,), 32, 8, 128, 7, seed=1239, qk_mult=2.0,
             note="long context S=32768, Q/K scaled by 2 to sharpen the softmax"),
    Workload("headline_4k", "bf16", (4096,), 32, 8, 128, 7, seed=1234,
             note="headline shape: Llama-3.1-8B geometry at S=4096, k=7 (the paper's micro-benchmark length, Sec. 5.4)"),
]}


@dataclass
class Inputs:
    wl: Workload
    cu_seqlens: torch.Tensor                    # int32 [n_docs+1], CPU
    q: list = field(default_factory=list)       # k tensors [T,hq,d]
    k: list = field(default_factory=list)       # k tensors [T,hkv,d]
    v: list = field(default_factory=list)
    d_o: list = field(default_factory=list)     # k tensors [T,hq,d]


def make_inputs(wl: Workload, with_grad: bool = True) -> Inputs:
    """CPU tensors in the workload dtype, one per step."""
    g = torch.Generator(device="cpu")
    g.manual_seed(wl.seed)
    inp = Inputs(wl, torch.tensor(wl.cu_seqlens, dtype=torch.int32))
    T = wl.T

    def draw(heads, mult):
        x = torch.randn((T, heads, wl.d), generator=g, dtype=torch.float32)
        if mult != 1.0:
            x *= mult
        return x.to(wl.torch_dtype)

    for _ in range(wl.k):
        inp.q.append(draw(wl.hq, wl.qk_mult))
        inp.k.append(draw(wl.hkv, wl.qk_mult))
        inp.v.append(draw(wl.hkv, 1.0))
        if with_grad:
            inp.d_o.append(draw(wl.hq, 1.0))
    return inp


def custom_workload(name, dtype, doc_lens, hq, hkv, d, k, seed, qk_mult=1.0) -> Workload:
    return Workload(name, dtype, tuple(int(x) for x in doc_lens), hq, hkv, d, k, seed, qk_mult)
