"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: the 128K-token long-tail
GQA batch (remap -> forward with the long sequence as 4-chunk pairs + merge -> backward -> inverse remap) and
the 64K lognormal MHA batch. The oracle checks sampled outputs it can compute one by one: whole short
sequences, single rows of the long sequences, dQ rows and dK/dV rows near the start, middle and end."""
import os
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2509_21841_amd import synth
from util import assert_close, assert_lse_close, widen

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import bench  # noqa: E402

pytestmark = pytest.mark.gpu


def host_slices(job, seq, q_heads, kv_heads):
    """fp64 host copies of one sequence restricted to some heads (attention layout)."""
    a, b = int(job.cu[seq]), int(job.cu[seq + 1])
    qh = torch.tensor(q_heads, device=job.dev); kh = torch.tensor(kv_heads, device=job.dev)
    f = lambda t, hs: widen(t[a:b].index_select(1, hs).contiguous())
    return f(job.q, qh), f(job.k, kh), f(job.v, kh), f(job.do, qh), a, b


@pytest.mark.parametrize("name", ["longtail-128k-gqa32x8", "lognormal-64k-mha32"])
def test_fullsize_step_matches_oracle_on_samples(name):
    job = bench.Job(name, "cuda:0")
    job.step()
    torch.cuda.synchronize()
    Hq, Hkv, d = job.w["Hq"], job.w["Hkv"], job.w["d"]
    grp = Hq // Hkv
    rng = np.random.default_rng(7)

    # remap: bit-exact against the oracle's row move, whole tensors
    if job.w["remap"]:
        idx = job.idx.cpu().numpy()
        for lin, att in ((job.k_lin, job.k), (job.q_lin, job.q)):
            assert np.array_equal(synth.bf16_bits(att), oracle.remap_tokens(synth.bf16_bits(lin), idx, 0))
        for att, lin in ((job.o, job.o_lin), (job.dk, job.dk_lin), (job.dq, job.dq_lin)):
            assert np.array_equal(synth.bf16_bits(lin), oracle.remap_tokens(synth.bf16_bits(att), idx, 1))

    order = sorted(range(len(job.lengths)), key=lambda s: job.lengths[s])
    longest, shortest, median = order[-1], order[0], order[len(order) // 2]

    # whole sequences (short and median) on the first and last KV group: forward and backward, all rows
    for seq in (shortest, median):
        for g in (0, Hkv - 1):
            heads = list(range(g * grp, (g + 1) * grp))
            q, k, v, do, a, b = host_slices(job, seq, heads, [g])
            cu = np.array([0, b - a], np.int32)
            ro, rl = oracle.varlen_attn_fwd(q, k, v, cu)
            rdq, rdk, rdv = oracle.varlen_attn_bwd(do, q, k, v, cu)
            sel = lambda t, hs: widen(t[a:b][:, hs].contiguous())
            assert_close(f"O seq{seq}", sel(job.o, heads), ro)
            assert_lse_close(f"LSE seq{seq}", widen(job.lse[heads][:, a:b].contiguous()), rl)
            assert_close(f"dQ seq{seq}", sel(job.dq, heads), rdq)
            assert_close(f"dK seq{seq}", sel(job.dk, [g]), rdk)
            assert_close(f"dV seq{seq}", sel(job.dv, [g]), rdv)

    # longest sequence: sampled rows (O, LSE, dQ) and sampled key rows (dK, dV) for two query heads / KV heads
    L = job.lengths[longest]
    for g in (0, Hkv - 1):
        heads = list(range(g * grp, (g + 1) * grp))
        q, k, v, do, a, b = host_slices(job, longest, heads, [g])
        rows = sorted(set([0, 1, 63, 64, 127, 128, L // 4 - 1, L // 4, L // 2, L - 1] + rng.integers(0, L, 12).tolist()))
        pairs = [dict(q_tok0=r, q_len=1, k_tok0=0, k_len=L, q_pos0=r, k_pos0=0, out_row0=n) for n, r in enumerate(rows)]
        ro, rl = oracle.chunk_attn_partial(q, k, v, pairs, len(rows))
        got_o = widen(job.o[a:b][rows][:, heads].contiguous())
        got_l = widen(job.lse[heads][:, a:b][:, rows].contiguous())
        assert_close("O rows of the longest sequence", got_o, ro)
        assert_lse_close("LSE rows of the longest sequence", got_l, rl)
        cu = np.array([0, L], np.int32)
        qs = [(r, hh) for r in rows[::3] for hh in (0, grp - 1)]
        kcols = sorted(set([L - 1, L - 2, L - 65, L - 700] + (L - 1 - rng.integers(0, min(L, 1500), 4)).tolist()))
        ks = [(c, 0) for c in kcols]
        rdq, rdk, rdv = oracle.varlen_attn_bwd_sample(do, q, k, v, cu, qs, ks)
        got_dq = np.stack([widen(job.dq[a + r, heads[hh]].contiguous()) for r, hh in qs])
        got_dk = np.stack([widen(job.dk[a + c, g].contiguous()) for c, _ in ks])
        got_dv = np.stack([widen(job.dv[a + c, g].contiguous()) for c, _ in ks])
        assert_close("dQ rows of the longest sequence", got_dq, rdq)
        assert_close("dK rows of the longest sequence", got_dk, rdk)
        assert_close("dV rows of the longest sequence", got_dv, rdv)

    # properties that hold at any size: finite everywhere, LSE of position 0 equals its single score
    assert torch.isfinite(job.o.float()).all() and torch.isfinite(job.lse).all()
    assert torch.isfinite(job.dq.float()).all() and torch.isfinite(job.dk.float()).all() and torch.isfinite(job.dv.float()).all()
    firsts = torch.from_numpy(job.cu[:-1].astype(np.int64)).to(job.dev)
    s00 = (job.q[firsts, 0].float() * job.k[firsts, 0].float()).sum(-1) / np.sqrt(d)
    assert (job.lse[0, firsts] - s00).abs().max().item() < 1e-3


def test_fullsize_node_placement_matches_oracle_on_samples():
    """The emulated 8-device node at the benchmark's size: partitioner placement, planned remap, ring rounds merged in
    place (forward) and accumulated (backward). Sequences are scattered over the device buffers, so every sample is
    gathered back into sequence order through the layout's runs before the oracle sees it."""
    job = bench.NodeBenchJob("node-p8-longtail-128k", "cuda:0")
    job.step()
    torch.cuda.synchronize()
    plan, nj = job.plan, job.job
    Hq, Hkv, d = job.w["Hq"], job.w["Hkv"], job.w["d"]
    grp = Hq // Hkv
    rng = np.random.default_rng(11)
    idx = plan.idx
    # remap, whole tensors, bit-exact: balanced -> attention is the scatter, attention -> balanced the gather
    assert np.array_equal(synth.bf16_bits(job.k), oracle.remap_tokens(synth.bf16_bits(job.k_lin), idx, 1))
    assert np.array_equal(synth.bf16_bits(job.q), oracle.remap_tokens(synth.bf16_bits(job.q_lin), idx, 1))
    assert np.array_equal(synth.bf16_bits(job.o_lin), oracle.remap_tokens(synth.bf16_bits(nj.o), idx, 0))
    assert np.array_equal(synth.bf16_bits(job.dk_lin), oracle.remap_tokens(synth.bf16_bits(nj.dk), idx, 0))
    # every rank's balanced share is the target
    from oracle import remap_planner as RP
    assert RP.is_feasible(plan.A.tolist(), plan.M)

    # attention-layout positions of every sequence, in sequence order
    pos = {}
    for s in sorted(plan.segments, key=lambda s: (s["seq"], s["pos0"])):
        pos.setdefault(s["seq"], []).append(np.arange(s["tok0"], s["tok0"] + s["len"]))
    pos = {k: np.concatenate(v) for k, v in pos.items()}
    ring_seqs = sorted({s["seq"] for s in plan.ring_segments})
    assert ring_seqs, "the workload is meant to contain a ring sequence"

    def host(seq, q_heads, kv_heads):
        ti = torch.from_numpy(pos[seq]).to(job.dev)
        qh = torch.tensor(q_heads, device=job.dev); kh = torch.tensor(kv_heads, device=job.dev)
        f = lambda t, hs: widen(t[ti].index_select(1, hs).contiguous())
        return f(job.q, qh), f(job.k, kh), f(job.v, kh), f(job.do, qh), ti

    local = sorted((s for s in range(len(plan.lengths)) if s not in ring_seqs), key=lambda s: plan.lengths[s])
    for seq in (local[0], local[len(local) // 2]):
        for g in (0, Hkv - 1):
            heads = list(range(g * grp, (g + 1) * grp))
            q, k, v, do, ti = host(seq, heads, [g])
            cu = np.array([0, len(ti)], np.int32)
            ro, rl = oracle.varlen_attn_fwd(q, k, v, cu)
            rdq, rdk, rdv = oracle.varlen_attn_bwd(do, q, k, v, cu)
            sel = lambda t, hs: widen(t[ti][:, hs].contiguous())
            assert_close(f"O seq{seq}", sel(nj.o, heads), ro)
            assert_lse_close(f"LSE seq{seq}", widen(nj.lse[heads][:, ti].contiguous()), rl)
            assert_close(f"dQ seq{seq}", sel(nj.dq, heads), rdq)
            assert_close(f"dK seq{seq}", sel(nj.dk, [g]), rdk)
            assert_close(f"dV seq{seq}", sel(nj.dv, [g]), rdv)

    seq = max(ring_seqs, key=lambda s: plan.lengths[s])
    L = plan.lengths[seq]
    C = [s for s in plan.ring_segments if s["seq"] == seq][0]["n_chunks"]
    for g in (0, Hkv - 1):
        heads = list(range(g * grp, (g + 1) * grp))
        q, k, v, do, ti = host(seq, heads, [g])
        edges = [c * L // C for c in range(1, C)]
        rows = sorted(set([0, 1, 63, 64, L // 2, L - 1] + edges[:3] + [e - 1 for e in edges[-3:]] + rng.integers(0, L, 10).tolist()))
        pairs = [dict(q_tok0=r, q_len=1, k_tok0=0, k_len=L, q_pos0=r, k_pos0=0, out_row0=n) for n, r in enumerate(rows)]
        ro, rl = oracle.chunk_attn_partial(q, k, v, pairs, len(rows))
        tr = ti[torch.tensor(rows, device=job.dev)]
        assert_close("O rows of the ring sequence", widen(nj.o[tr][:, heads].contiguous()), ro)
        assert_lse_close("LSE rows of the ring sequence", widen(nj.lse_run[heads][:, tr].contiguous()), rl)
        cu = np.array([0, L], np.int32)
        qs = [(r, hh) for r in rows[::3] for hh in (0, grp - 1)]
        kcols = sorted(set([L - 1, L - 2, L - 65, edges[-1], edges[-1] - 1] + (L - 1 - rng.integers(0, min(L, 1500), 4)).tolist()))
        ks = [(c, 0) for c in kcols]
        rdq, rdk, rdv = oracle.varlen_attn_bwd_sample(do, q, k, v, cu, qs, ks)
        got_dq = np.stack([widen(nj.dq[ti[r], heads[hh]].contiguous()) for r, hh in qs])
        got_dk = np.stack([widen(nj.dk[ti[c], g].contiguous()) for c, _ in ks])
        got_dv = np.stack([widen(nj.dv[ti[c], g].contiguous()) for c, _ in ks])
        assert_close("dQ rows of the ring sequence", got_dq, rdq)
        assert_close("dK rows of the ring sequence", got_dk, rdk)
        assert_close("dV rows of the ring sequence", got_dv, rdv)
    for t in (nj.o, nj.dq, nj.dk, nj.dv):
        assert torch.isfinite(t.float()).all()
