"""Convenience holder used by the tests, the smoke check and the benchmark: allocates outputs and
workspace with PyTorch for one workload and calls the C-ABI entry points.  No arithmetic here."""
from __future__ import annotations

import torch

from . import binding as B


class TttAttnRunner:
    def __init__(self, q, k, v, cu_seqlens, softmax_scale, device="cuda:0", allocate_outputs=True):
        """q: list of k [T,hq,d] tensors; k,v: lists of k [T,hkv,d] tensors (device); cu_seqlens: ints.
        allocate_outputs=False leaves o / lse to the caller (lists of k entries, None where not needed)."""
        self.dev = torch.device(device)
        self.q, self.k, self.v = q, k, v
        self.K = len(q)
        self.cu_host = [int(x) for x in cu_seqlens]
        self.cu_dev = torch.tensor(self.cu_host, dtype=torch.int32, device=self.dev)
        self.scale = float(softmax_scale)
        T, hq, d = q[0].shape
        self.T, self.hq, self.d = T, hq, d
        self.o = [torch.empty_like(x) for x in q] if allocate_outputs else None
        self.lse = [torch.empty((hq, T), dtype=torch.float32, device=self.dev) for _ in q] if allocate_outputs else None
        self.dq = self.dk = self.dv = None
        self._ws = {}

    def params(self, step_begin=0, step_end=None):
        step_end = self.K if step_end is None else step_end
        return B.make_params(self.q[0], self.k[0], self.K, step_begin, step_end, self.cu_host, self.scale)

    def workspace(self, which_pass):
        if which_pass not in self._ws:
            n = B.ttt_attn_workspace_bytes(self.params(), which_pass)
            self._ws[which_pass] = torch.empty(n, dtype=torch.uint8, device=self.dev)
        return self._ws[which_pass]

    def forward(self, step_begin=0, step_end=None, stream=None):
        p = self.params(step_begin, step_end)
        B.ttt_attn_fwd(p, self.q, self.k, self.v, self.cu_dev, self.cu_host, self.o, self.lse,
                       self.workspace(B.TTT_PASS_FWD), stream)

    def forward_docsteps(self, doc_steps, stream=None):
        B.ttt_attn_fwd_docsteps(self.params(), doc_steps, self.q, self.k, self.v, self.cu_dev, self.cu_host, self.o,
                                self.lse, self.workspace(B.TTT_PASS_FWD), stream)

    def backward_docsteps(self, d_o, doc_steps, stream=None):
        self.alloc_grads()
        B.ttt_attn_bwd_docsteps(self.params(), doc_steps, self.q, self.k, self.v, self.o, self.lse, d_o, self.cu_dev,
                                self.cu_host, self.dq, self.dk, self.dv, self.workspace(B.TTT_PASS_BWD), stream)

    def alloc_grads(self):
        if self.dq is None:
            self.dq = [torch.empty_like(x) for x in self.q]
            self.dk = [torch.empty_like(x) for x in self.k]
            self.dv = [torch.empty_like(x) for x in self.v]

    def backward(self, d_o, step_begin=0, step_end=None, accumulate=False, stream=None):
        self.alloc_grads()
        p = self.params(step_begin, step_end)
        ws = self.workspace(B.TTT_PASS_BWD_ACCUM if accumulate else B.TTT_PASS_BWD)
        B.ttt_attn_bwd(p, self.q, self.k, self.v, self.o, self.lse, d_o, self.cu_dev, self.cu_host,
                       self.dq, self.dk, self.dv, int(accumulate), ws, stream)
