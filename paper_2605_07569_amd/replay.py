"""Ring replay on one GPU: iterate the KV chunk list through the C-ABI calls.

The CP ring of HexiSeq (App. A.4: K steps, one source KV block per step) is replayed by a host loop
over the chunk list: forward = fwd_chunk (+ LSE merge) per chunk; backward = Delta once, then
bwd_chunk per chunk.  Nothing is skipped by hand: chunks in the shard's future are passed to the
library like any other.  This module only owns device buffers and the loop; all arithmetic is in
the library's kernels.
"""
import torch

from . import hexi
from .workloads import Workload, gather_rows


class ShardRun:
    """Device buffers of one workload plus the forward / backward replay loops."""

    def __init__(self, w: Workload, inputs, device="cuda:0", fused_merge=True, keep_partials=False):
        self.w = w
        self.dev = torch.device(device)
        self.fused = fused_merge
        self.q = inputs["q"].to(self.dev)
        self.d_o = inputs["d_o"].to(self.dev)
        self.k = [gather_rows(inputs["k"], ch).to(self.dev) for ch in w.chunks]
        self.v = [gather_rows(inputs["v"], ch).to(self.dev) for ch in w.chunks]
        nq, nkv, d, lq = w.n_q_heads, w.n_kv_heads, w.head_dim, w.lq
        f32 = dict(dtype=torch.float32, device=self.dev)
        self.o = torch.zeros((lq, nq, d), **f32)
        self.lse = torch.full((nq, lq), float("-inf"), **f32)
        self.delta = torch.empty((nq, lq), **f32)
        self.dq = torch.zeros((lq, nq, d), **f32)
        self.dk = [torch.empty((kc.shape[0], nkv, d), **f32) for kc in self.k]
        self.dv = [torch.empty((kc.shape[0], nkv, d), **f32) for kc in self.k]
        if not fused_merge:
            self.o_part = torch.empty_like(self.o)
            self.lse_part = torch.empty_like(self.lse)
        self.partials = [] if keep_partials else None
        self.desc = [hexi.desc_for(self.q, kc, w.scale, w.kv_of_q) for kc in self.k]

    def forward(self):
        w = self.w
        self.o.zero_()
        self.lse.fill_(float("-inf"))
        for j, ch in enumerate(w.chunks):
            if self.fused:
                hexi.hexi_attn_fwd_chunk(self.desc[j], w.q_segs, ch, self.q, self.k[j], self.v[j], self.o, self.lse,
                                         flags=hexi.HEXI_ACCUMULATE)
            else:
                hexi.hexi_attn_fwd_chunk(self.desc[j], w.q_segs, ch, self.q, self.k[j], self.v[j], self.o_part, self.lse_part)
                if self.partials is not None:
                    self.partials.append((self.o_part.clone(), self.lse_part.clone()))
                hexi.hexi_attn_merge_lse(self.o, self.lse, self.o_part, self.lse_part)

    def backward(self):
        w = self.w
        self.dq.zero_()
        for j, ch in enumerate(w.chunks):
            flags = hexi.HEXI_COMPUTE_DELTA if j == 0 else 0
            hexi.hexi_attn_bwd_chunk(self.desc[j], w.q_segs, ch, self.q, self.k[j], self.v[j], self.o, self.d_o,
                                     self.lse, self.delta, self.dq, self.dk[j], self.dv[j], flags=flags)

    def step(self):
        self.forward()
        self.backward()
