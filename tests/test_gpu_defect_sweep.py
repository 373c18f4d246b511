"""Defect sweep (NOT a parity claim): many small random configurations through every entry point, and a few
medium-size batches through the forward and backward, against the oracle.

Its purpose is breadth: ragged and degenerate lengths, head layouts, chunk counts and scales that the hand-picked
cases of test_gpu_parity.py do not enumerate. A wrong mask, index or descriptor shows as an error of order one, so the
sweep looks for defects with twice the stated absolute tolerance and 1.5e-2 relative-L2 (tensors of a handful of rows
have nothing to average over). The stated bounds (2e-2 / 5e-3) are asserted by test_gpu_parity.py and
test_gpu_fullsize.py on their fixed cases; nothing here counts towards parity."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_21841_amd import binding as B
from paper_2509_21841_amd import synth
from util import assert_close, assert_lse_close, widen

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
LENGTHS = [0, 1, 2, 3, 17, 31, 32, 33, 63, 64, 65, 96, 127, 128, 129, 191, 192, 255, 256, 257, 300, 383, 511, 512, 640,
           777, 1025, 1537]


def close(name, got, ref, **kw):
    assert_close(name, got, ref, maxabs=4e-2, rell2=1.5e-2, **kw)


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_configurations(seed):
    rng = np.random.default_rng(seed)
    for case in range(25):
        d = int(rng.choice([64, 128])); Hkv = int(rng.choice([1, 2, 3])); Hq = Hkv * int(rng.choice([1, 2, 4]))
        lengths = [int(x) for x in rng.choice(LENGTHS, size=int(rng.integers(1, 6)))]
        if sum(lengths) < 64:
            lengths.append(64)          # the relative-L2 criterion needs a tensor, not a handful of rows
        scale = float(rng.choice([0.0, 0.05, 0.1]))
        tag = f"seed {seed} case {case}: lengths={lengths} Hq={Hq} Hkv={Hkv} d={d} scale={scale}"
        T = sum(lengths)
        q, k, v, do = synth.make_qkv(T, Hq, Hkv, d, 100 * seed + case, DEV, with_dout=True)
        cu = synth.cu_seqlens(lengths)
        o, lse = B.varlen_attn_fwd(q, k, v, cu, scale=scale)
        dq, dk, dv = B.varlen_attn_bwd(do, q, k, v, o, lse, cu, scale=scale)
        torch.cuda.synchronize()
        qw, kw, vw, dow = widen(q), widen(k), widen(v), widen(do)
        ro, rl = oracle.varlen_attn_fwd(qw, kw, vw, cu, scale=scale or None)
        rdq, rdk, rdv = oracle.varlen_attn_bwd(dow, qw, kw, vw, cu, scale=scale or None)
        close(tag + " O", widen(o), ro); assert_lse_close(tag + " LSE", widen(lse), rl)
        close(tag + " dQ", widen(dq), rdq); close(tag + " dK", widen(dk), rdk); close(tag + " dV", widen(dv), rdv)
        # the longest sequence once more as chunk pairs: partial + merge, rounds merged in place, chunked backward
        s = int(np.argmax(lengths)); L = lengths[s]; t0 = int(cu[s]); C = int(rng.choice([1, 2, 3, 4, 6, 8, 16]))
        pairs, merges, rows = B.chunk_pairs(t0, L, C)
        op, lp = B.chunk_attn_partial(q, k, v, pairs, rows, scale=scale)
        o2 = torch.zeros_like(o); lse2 = torch.zeros_like(lse)
        B.lse_merge(op, lp, merges, o2, lse2)
        o_run = torch.zeros((T, Hq, d), dtype=torch.float32, device=DEV)
        lse_run = torch.full((Hq, T), float("-inf"), dtype=torch.float32, device=DEV)
        acc = [torch.zeros(x.shape, dtype=torch.float32, device=DEV) for x in (q, k, v)]
        for rnd in B.ring_rounds(t0, L, C):
            B.chunk_attn_update(q, k, v, rnd, o_run, lse_run, scale=scale)
            B.chunk_attn_partial_bwd(do, q, k, v, o, lse, rnd, *acc, scale=scale)
        torch.cuda.synchronize()
        sl = slice(t0, t0 + L)
        close(tag + " merged O", widen(o2)[sl], ro[sl]); assert_lse_close(tag + " merged LSE", widen(lse2)[:, sl], rl[:, sl])
        close(tag + " running O", widen(o_run)[sl], ro[sl], bf16_out=False)
        assert_lse_close(tag + " running LSE", widen(lse_run)[:, sl], rl[:, sl])
        for name, a, r in zip(("dQ", "dK", "dV"), acc, (rdq, rdk, rdv)):
            close(tag + " chunked " + name, a.double().cpu().numpy()[sl], r[sl], bf16_out=False)
        # remap with a random permutation, both modes
        idx = torch.randperm(T, generator=torch.Generator().manual_seed(case)).to(torch.int32)
        g = B.remap_tokens(q, idx.to(DEV), 0)
        assert np.array_equal(synth.bf16_bits(g), oracle.remap_tokens(synth.bf16_bits(q), idx.numpy(), 0)), tag
        assert torch.equal(B.remap_tokens(g, idx.to(DEV), 1).view(torch.int16), q.view(torch.int16)), tag


@pytest.mark.parametrize("seed", [21, 22])
def test_random_medium_batches(seed):
    """Batches of 15-25K tokens with 8-32 query heads: thousands of work items per launch (the run-time claimed tail),
    both dK/dV kernels and the rule that picks between them, head groupings 1-8. One KV group of each batch against
    the oracle, with the sweep's defect bound on every element and the stated relative-L2 bound."""
    rng = np.random.default_rng(seed)
    for case in range(4):
        d = int(rng.choice([64, 128, 128])); grp = int(rng.choice([1, 2, 4, 8])); Hkv = int(rng.choice([2, 4, 8]))
        Hq = Hkv * grp
        if case == 0:
            lengths = [int(x) for x in rng.integers(64, 3000, size=int(rng.integers(8, 20)))]
        elif case == 1:
            lengths = [int(rng.integers(6000, 12000))] + [int(x) for x in rng.integers(1, 1500, size=int(rng.integers(3, 16)))]
        elif case == 2:
            lengths = [int(x) for x in rng.integers(2000, 6000, size=int(rng.integers(3, 6)))]
        else:
            lengths = [int(x) for x in rng.choice([127, 128, 129, 1023, 1024, 1025, 2047, 2048, 2049, 4095, 4096, 4097],
                                                  size=int(rng.integers(4, 10)))]
        T = sum(lengths)
        tag = f"seed {seed} case {case}: S={len(lengths)} T={T} max={max(lengths)} Hq={Hq} Hkv={Hkv} d={d}"
        q, k, v, do = synth.make_qkv(T, Hq, Hkv, d, 1000 * seed + case, DEV, with_dout=True)
        cu = synth.cu_seqlens(lengths)
        o, lse = B.varlen_attn_fwd(q, k, v, cu)
        dq, dk, dv = B.varlen_attn_bwd(do, q, k, v, o, lse, cu)
        torch.cuda.synchronize()
        g = int(rng.integers(0, Hkv))
        heads = list(range(g * grp, (g + 1) * grp))
        sel = lambda t, hs: widen(t[:, hs].contiguous())
        ro, rl = oracle.varlen_attn_fwd(sel(q, heads), sel(k, [g]), sel(v, [g]), cu)
        rdq, rdk, rdv = oracle.varlen_attn_bwd(sel(do, heads), sel(q, heads), sel(k, [g]), sel(v, [g]), cu)
        kw = dict(maxabs=4e-2, rell2=5e-3)
        assert_close(tag + " O", sel(o, heads), ro, **kw)
        assert_lse_close(tag + " LSE", widen(lse[heads].contiguous()), rl)
        assert_close(tag + " dQ", sel(dq, heads), rdq, **kw)
        assert_close(tag + " dK", sel(dk, [g]), rdk, **kw)
        assert_close(tag + " dV", sel(dv, [g]), rdv, **kw)
        del q, k, v, do, o, lse, dq, dk, dv
