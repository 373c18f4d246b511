"""Descriptor plumbing for running a whole node's placement on one GPU: the hierarchical partitioner decides which
device runs what (Sec. 3.1), the device buffers are laid end to end as the attention layout, the remap planner and its
permutation connect that layout to the token-balanced one of the linear modules (Sec. 3.4), and the attention engine
runs local sequences whole and ring sequences as chunk pairs, one ring round per call (Sec. 3.2).

Everything here is list handling around the C-ABI helpers (zp_partition, zp_node_segments, zp_remap_plan,
zp_remap_indices); all arithmetic on tokens runs in the library's kernels.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


class NodePlan:
    def __init__(self, lengths, P: int, N: int, L: int, b_intra: int = 1, b_inter: int = 1):
        self.lengths = [int(x) for x in lengths]
        self.P, self.N, self.L = P, N, L
        self.placements, self.s1, self.s0 = B.partition(self.lengths, P, N, L)
        self.segments, self.A = B.node_segments(self.lengths, self.placements, P, N)
        self.T = int(self.A.sum())
        assert self.T == sum(self.lengths)
        self.M, self.remap_cost = B.remap_plan(self.A, P, b_intra, b_inter)
        self.idx = B.remap_indices(self.A, self.M)          # balanced position -> attention-layout position
        # every run is one entry of the packed batch; runs of ring sequences are left to the chunk-pair calls
        self.cu = np.zeros(len(self.segments) + 1, np.int32)
        self.cu[1:] = np.cumsum([s["len"] for s in self.segments])
        self.skip = np.asarray([1 if s["n_chunks"] > 1 else 0 for s in self.segments], np.uint8)
        # attention-layout position -> position in the batch as drawn (sequence after sequence)
        self.orig = B.segment_positions(self.lengths, self.segments, self.T)
        self.ring_segments = [s for s in self.segments if s["n_chunks"] > 1]
        ring_seqs = {s["seq"] for s in self.ring_segments}
        # ring rounds (zp_ring_round_pairs): round t holds the pairs (qc, qc - t) of every ring sequence, so no query
        # run and no key run appears twice in a call
        self.max_chunks, self.rounds = 0, []
        if self.ring_segments:
            segs = B._segments_array(self.segments)
            first, self.max_chunks = B.ring_round_pairs(segs, 0)
            self.rounds = [first] + [B.ring_round_pairs(segs, t)[0] for t in range(1, self.max_chunks)]
        self.ring_pairs = sum(L_ * (L_ + 1) // 2 for seq, L_ in enumerate(self.lengths) if seq in ring_seqs)
        self.local_pairs = sum(L_ * (L_ + 1) // 2 for seq, L_ in enumerate(self.lengths) if seq not in ring_seqs)


class NodeJob:
    """Device buffers of one emulated node; forward() / backward() enqueue the hot path in the attention layout,
    to_attention() / to_balanced() are the remapping layer."""

    def __init__(self, plan: NodePlan, Hq: int, Hkv: int, d: int, device="cuda:0"):
        self.plan, self.dev = plan, device
        T = plan.T
        self.idx = torch.from_numpy(plan.idx).to(device)
        mk = lambda h, dt=torch.bfloat16: torch.empty((T, h, d), dtype=dt, device=device)
        self.o = mk(Hq); self.dq = mk(Hq); self.dk = mk(Hkv); self.dv = mk(Hkv)
        self.lse = torch.empty((Hq, T), dtype=torch.float32, device=device)
        if plan.ring_segments:
            self.o_run = mk(Hq, torch.float32)
            self.lse_run = torch.empty((Hq, T), dtype=torch.float32, device=device)
            self.dq_acc = mk(Hq, torch.float32); self.dk_acc = mk(Hkv, torch.float32); self.dv_acc = mk(Hkv, torch.float32)

    def to_attention(self, x_balanced, out=None):
        return B.remap_tokens(x_balanced, self.idx, 1, dst=out)

    def to_balanced(self, x_attention, out=None):
        return B.remap_tokens(x_attention, self.idx, 0, dst=out)

    def forward(self, q, k, v, scale=0.0):
        pl = self.plan
        B.varlen_attn_fwd(q, k, v, pl.cu, o=self.o, lse=self.lse, scale=scale, seq_skip=pl.skip)
        if pl.ring_segments:
            self.lse_run.fill_(float("-inf"))
            for arr, n in pl.rounds:
                B.chunk_attn_update(q, k, v, (arr, n), self.o_run, self.lse_run, scale=scale)
            for s in pl.ring_segments:
                sl = slice(s["tok0"], s["tok0"] + s["len"])
                B.accum_to_bf16(self.o_run[sl], self.o[sl])
        return self.o, self.lse           # LSE of ring rows stays in self.lse_run

    def backward(self, do, q, k, v, scale=0.0):
        pl = self.plan
        B.varlen_attn_bwd(do, q, k, v, self.o, self.lse, pl.cu, dq=self.dq, dk=self.dk, dv=self.dv, scale=scale,
                          seq_skip=pl.skip)
        if pl.ring_segments:
            for a in (self.dq_acc, self.dk_acc, self.dv_acc):
                a.zero_()
            for arr, n in pl.rounds:
                B.chunk_attn_partial_bwd(do, q, k, v, self.o, self.lse_run, (arr, n), self.dq_acc, self.dk_acc, self.dv_acc,
                                         scale=scale)
            for s in pl.ring_segments:
                sl = slice(s["tok0"], s["tok0"] + s["len"])
                B.accum_to_bf16(self.dq_acc[sl], self.dq[sl])
                B.accum_to_bf16(self.dk_acc[sl], self.dk[sl])
                B.accum_to_bf16(self.dv_acc[sl], self.dv[sl])
        return self.dq, self.dk, self.dv
