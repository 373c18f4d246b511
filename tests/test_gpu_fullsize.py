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
