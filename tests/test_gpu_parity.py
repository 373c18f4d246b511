"""Parity of the HIP path (through the C ABI) against the fp64 oracle on seeded synthetic inputs."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_21841_amd import binding as B
from paper_2509_21841_amd import synth
from util import Checks, StatedBoundNotMet, assert_close, assert_lse_close, widen

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make(lengths, Hq, Hkv, d, seed, with_dout=False):
    T = int(sum(lengths))
    ts = synth.make_qkv(T, Hq, Hkv, d, seed, device=DEV, with_dout=with_dout)
    return ts, synth.cu_seqlens(lengths)


# ---- remap -------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,row_elems", [(1, 8), (257, 24), (5000, 1024), (4096, 8192), (3, 64)])
def test_remap_bit_exact(n, row_elems):
    g = torch.Generator(device="cpu"); g.manual_seed(n)
    x = torch.randint(-32768, 32767, (n, row_elems), dtype=torch.int16, generator=g).to(DEV)
    idx = torch.randperm(n, generator=g).to(torch.int32)
    ref = oracle.remap_tokens(x.cpu().numpy(), idx.numpy(), 0)
    got = B.remap_tokens(x, idx.to(DEV), 0)
    assert np.array_equal(got.cpu().numpy(), ref)
    ref1 = oracle.remap_tokens(x.cpu().numpy(), idx.numpy(), 1)
    got1 = B.remap_tokens(x, idx.to(DEV), 1)
    assert np.array_equal(got1.cpu().numpy(), ref1)
    back = B.remap_tokens(got, idx.to(DEV), 1)
    assert torch.equal(back, x)


def test_remap_empty_and_layout_round_trip():
    assert B.remap_tokens(torch.empty((0, 64), dtype=torch.bfloat16, device=DEV), torch.empty(0, dtype=torch.int32, device=DEV)).shape[0] == 0
    lengths = synth.lengths_lognormal(8192, 5, median=256, lo=16, hi=2048)
    idx, attn_lengths, _ = synth.balanced_attention_layout(lengths, R=8)
    (q, k, v), _ = make(lengths, 8, 2, 128, 5)
    idx_d = torch.from_numpy(idx).to(DEV)
    qa = B.remap_tokens(q, idx_d, 0)
    assert np.array_equal(synth.bf16_bits(qa), oracle.remap_tokens(synth.bf16_bits(q), idx, 0))
    assert torch.equal(B.remap_tokens(qa, idx_d, 1).view(torch.int16), q.view(torch.int16))


def test_remap_with_planned_indices_balances_the_ranks():
    """Transfer plan (Sec. 3.4) -> permutation -> device remap: rank slabs of the balanced layout hold exactly the
    tokens the oracle's selection rule names, and the inverse remap restores the attention layout."""
    from oracle import remap_planner as RP
    rng = np.random.default_rng(3)
    P, N = 4, 2
    A = rng.integers(0, 700, size=P * N).tolist()
    M, _ = B.remap_plan(A, P, 1, 6)
    idx = B.remap_indices(A, M)
    assert np.array_equal(idx, RP.remap_indices(A, M))
    T = int(sum(A))
    x = synth.normal_bf16((T, 2, 64), 21, 1, DEV)
    idx_d = torch.from_numpy(idx).to(DEV)
    bal = B.remap_tokens(x, idx_d, 0)
    assert np.array_equal(synth.bf16_bits(bal), oracle.remap_tokens(synth.bf16_bits(x), idx, 0))
    assert torch.equal(B.remap_tokens(bal, idx_d, 1).view(torch.int16), x.view(torch.int16))
    # rank r's balanced slab: its own head, then arrivals; sizes are the balanced targets
    offB = np.concatenate([[0], np.cumsum(RP.targets(A))]); offA = np.concatenate([[0], np.cumsum(A)])
    for r in range(P * N):
        own = idx[offB[r]:offB[r + 1]]
        kept = min(A[r], RP.targets(A)[r])
        assert np.array_equal(own[:kept], np.arange(offA[r], offA[r] + kept))


# ---- merge -------------------------------------------------------------------------------------------
@pytest.mark.parametrize("Hq,d,n,parts", [(4, 64, 37, 3), (32, 128, 300, 4), (2, 128, 9, 1), (3, 64, 20, 8), (2, 128, 11, 16)])
def test_lse_merge_matches_oracle(Hq, d, n, parts):
    g = torch.Generator(device="cpu"); g.manual_seed(Hq * 1000 + n)
    rows = parts * n + 5
    op = torch.randn((rows, Hq, d), generator=g, dtype=torch.float32)
    lp = torch.randn((Hq, rows), generator=g, dtype=torch.float32) * 3
    lp[:, 2] = float("-inf")
    if parts > 1:
        lp[0, [3 + p * n for p in range(parts)]] = float("-inf")   # a row whose parts are all -inf
    merges = [(1, n, [p * n for p in range(parts)])]
    T = n + 3
    o = torch.zeros((T, Hq, d), dtype=torch.bfloat16, device=DEV); lse = torch.zeros((Hq, T), dtype=torch.float32, device=DEV)
    B.lse_merge(op.to(DEV), lp.to(DEV), merges, o, lse)
    ro, rl = oracle.lse_merge(op.double().numpy(), lp.double().numpy(), merges, T, np.zeros((T, Hq, d)), np.zeros((Hq, T)))
    assert_close("merge O", widen(o), ro, maxabs=2e-2, rell2=5e-3)
    assert_lse_close("merge LSE", widen(lse), rl)
    assert (widen(o)[0] == 0).all() and (widen(o)[n + 1:] == 0).all()   # rows outside the merge untouched


# ---- forward -----------------------------------------------------------------------------------------
def run_fwd(lengths, Hq, Hkv, d, seed, scale=0.0):
    (q, k, v), cu = make(lengths, Hq, Hkv, d, seed)
    o, lse = B.varlen_attn_fwd(q, k, v, cu, scale=scale)
    torch.cuda.synchronize()
    ro, rl = oracle.varlen_attn_fwd(widen(q), widen(k), widen(v), cu, scale=scale or None)
    assert_close("O", widen(o), ro)
    assert_lse_close("LSE", widen(lse), rl)
    return (q, k, v), cu, (o, lse), (ro, rl)


def test_fwd_tiny_config_and_chunk_split_of_longest():
    """Config 1: 8 sequences U[16,512], <= 2048 tokens, 4 heads, d 64; the longest sequence is also split
    into 2 chunks (3 causal pairs) and merged."""
    lengths = synth.lengths_tiny(1001)
    (q, k, v), cu, (o, lse), (ro, rl) = run_fwd(lengths, 4, 4, 64, 1001)
    s = int(np.argmax(lengths)); L = lengths[s]; t0 = int(cu[s])
    pairs, merges, rows = B.chunk_pairs(t0, L, 2)
    assert len(pairs) == 3
    op, lp = B.chunk_attn_partial(q, k, v, pairs, rows)
    opairs, omerges, orows = oracle.causal_pairs(t0, L, 2)
    rop, rlp = oracle.chunk_attn_partial(widen(q), widen(k), widen(v), opairs, orows)
    assert_close("O_part", widen(op), rop, bf16_out=False)
    assert_lse_close("LSE_part", widen(lp), rlp)
    o2 = torch.zeros_like(o); lse2 = torch.zeros_like(lse)
    B.lse_merge(op, lp, merges, o2, lse2)
    assert_close("merged O", widen(o2)[t0:t0 + L], ro[t0:t0 + L])
    assert_lse_close("merged LSE", widen(lse2)[:, t0:t0 + L], rl[:, t0:t0 + L])


@pytest.mark.parametrize("lengths,Hq,Hkv,d", [
    ([1], 1, 1, 64), ([1, 1, 2, 3], 2, 1, 128), ([127, 128, 129], 2, 2, 128), ([64, 65, 63, 1], 4, 2, 64),
    ([700, 0, 333, 0], 8, 2, 128), ([1500], 4, 1, 128), ([300, 41], 2, 2, 64)])
def test_fwd_edge_lengths(lengths, Hq, Hkv, d):
    run_fwd(lengths, Hq, Hkv, d, 7)


def test_fwd_custom_scale_and_strided_qkv():
    lengths = [200, 77]
    T, Hq, Hkv, d = 277, 4, 2, 128
    fused = synth.normal_bf16((T, Hq + 2 * Hkv, d), 3, 1, DEV)
    q, k, v = fused[:, :Hq], fused[:, Hq:Hq + Hkv], fused[:, Hq + Hkv:]
    cu = synth.cu_seqlens(lengths)
    o, lse = B.varlen_attn_fwd(q, k, v, cu, scale=0.05)
    ro, rl = oracle.varlen_attn_fwd(widen(q.contiguous()), widen(k.contiguous()), widen(v.contiguous()), cu, scale=0.05)
    assert_close("O", widen(o), ro); assert_lse_close("LSE", widen(lse), rl)


@pytest.mark.parametrize("d", [64, 128])
def test_bwd_strided_inputs_and_outputs(d):
    """Q, K, V (and dQ, dK, dV) as slices of one fused [T, Hq + 2 Hkv, d] buffer, dO and O as slices of wider buffers:
    every token stride differs from heads x d. The results must be bit-identical to those on contiguous tensors."""
    lengths = [700, 129, 64, 2300]
    T, Hq, Hkv = sum(lengths), 4, 2
    cu = synth.cu_seqlens(lengths)
    fused = synth.normal_bf16((T, Hq + 2 * Hkv, d), 5, 1, DEV)
    q, k, v = fused[:, :Hq], fused[:, Hq:Hq + Hkv], fused[:, Hq + Hkv:]
    do_wide = synth.normal_bf16((T, Hq + 3, d), 6, 1, DEV)
    do = do_wide[:, 2:2 + Hq]
    qc, kc, vc, doc = q.contiguous(), k.contiguous(), v.contiguous(), do.contiguous()
    oc, lc = B.varlen_attn_fwd(qc, kc, vc, cu)
    ref = B.varlen_attn_bwd(doc, qc, kc, vc, oc, lc, cu)
    o_wide = torch.zeros((T, Hq + 1, d), dtype=torch.bfloat16, device=DEV)
    o = o_wide[:, 1:]
    o.copy_(oc)
    grads = torch.full((T, Hq + 2 * Hkv, d), 7.0, dtype=torch.bfloat16, device=DEV)
    dq, dk, dv = grads[:, :Hq], grads[:, Hq:Hq + Hkv], grads[:, Hq + Hkv:]
    B.varlen_attn_bwd(do, q, k, v, o, lc, cu, dq=dq, dk=dk, dv=dv)
    torch.cuda.synchronize()
    for got, want in zip((dq, dk, dv), ref):
        assert torch.equal(got.contiguous().view(torch.int16), want.view(torch.int16))


def test_fwd_closed_forms_on_device():
    lengths = [1, 300]
    (q, k, v), cu = make(lengths, 2, 2, 128, 9)
    o, lse = B.varlen_attn_fwd(torch.zeros_like(q), k, v, cu)
    vf = widen(v)
    pm = np.cumsum(vf[1:], axis=0) / np.arange(1, 301)[:, None, None]
    assert_close("prefix mean", widen(o)[1:], pm)
    assert np.abs(widen(lse)[:, 1:] - np.log(np.arange(1, 301))).max() < 1e-3
    assert np.array_equal(widen(o)[0], vf[0])   # length-1 sequence returns V


def test_fwd_deterministic():
    lengths = [513, 200]
    (q, k, v), cu = make(lengths, 4, 2, 128, 13)
    a = B.varlen_attn_fwd(q, k, v, cu); b = B.varlen_attn_fwd(q, k, v, cu)
    assert torch.equal(a[0].view(torch.int16), b[0].view(torch.int16)) and torch.equal(a[1], b[1])


@pytest.mark.parametrize("lengths,Hq,Hkv,d", [([513, 200], 4, 2, 128), ([129, 64, 300, 1], 2, 2, 64), ([2049], 8, 2, 128)])
def test_every_entry_point_is_deterministic(lengths, Hq, Hkv, d):
    """Three runs of forward, backward, the chunked paths and the merge give bit-identical results."""
    (q, k, v, do), cu = make(lengths, Hq, Hkv, d, 59, with_dout=True)
    T = q.shape[0]
    L = lengths[0]
    pairs, merges, rows = B.chunk_pairs(0, L, 4)
    runs = []
    for _ in range(3):
        o, lse = B.varlen_attn_fwd(q, k, v, cu)
        dq, dk, dv = B.varlen_attn_bwd(do, q, k, v, o, lse, cu)
        op, lp = B.chunk_attn_partial(q, k, v, pairs, rows)
        o2 = torch.zeros_like(o); lse2 = torch.zeros_like(lse)
        B.lse_merge(op, lp, merges, o2, lse2)
        o_run = torch.zeros((T, Hq, d), dtype=torch.float32, device=DEV)
        lse_run = torch.full((Hq, T), float("-inf"), dtype=torch.float32, device=DEV)
        acc = [torch.zeros(x.shape, dtype=torch.float32, device=DEV) for x in (q, k, v)]
        for rnd in B.ring_rounds(0, L, 4):
            B.chunk_attn_update(q, k, v, rnd, o_run, lse_run)
            B.chunk_attn_partial_bwd(do, q, k, v, o, lse, rnd, *acc)
        torch.cuda.synchronize()
        runs.append([t.clone() for t in (o, lse, dq, dk, dv, op[:rows], lp[:, :rows], o2, lse2, o_run[:L], lse_run[:, :L], *acc)])
    bits = lambda t: t.view(torch.int16) if t.dtype == torch.bfloat16 else t.view(torch.int32)
    for other in runs[1:]:
        for a, b in zip(runs[0], other):
            assert torch.equal(bits(a), bits(b))


# ---- partials ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("L,C,Hq,Hkv,d", [(1000, 4, 4, 1, 128), (257, 3, 2, 2, 64), (130, 4, 2, 1, 128)])
def test_chunked_then_merged_equals_whole(L, C, Hq, Hkv, d):
    lengths = [50, L, 31]
    (q, k, v), cu = make(lengths, Hq, Hkv, d, 17)
    t0 = int(cu[1])
    pairs, merges, rows = B.chunk_pairs(t0, L, C)
    op, lp = B.chunk_attn_partial(q, k, v, pairs, rows)
    opairs, _, orows = oracle.causal_pairs(t0, L, C)
    rop, rlp = oracle.chunk_attn_partial(widen(q), widen(k), widen(v), opairs, orows)
    assert_close("O_part", widen(op), rop, bf16_out=False); assert_lse_close("LSE_part", widen(lp), rlp)
    o = torch.zeros_like(q); lse = torch.zeros((Hq, q.shape[0]), dtype=torch.float32, device=DEV)
    B.lse_merge(op, lp, merges, o, lse)
    ro, rl = oracle.varlen_attn_fwd(widen(q), widen(k), widen(v), cu)
    assert_close("merged O", widen(o)[t0:t0 + L], ro[t0:t0 + L])
    assert_lse_close("merged LSE", widen(lse)[:, t0:t0 + L], rl[:, t0:t0 + L])


@pytest.mark.parametrize("L,G,Hq,Hkv,d", [(1000, 4, 4, 2, 128), (333, 2, 2, 2, 64), (70, 8, 2, 1, 128)])
def test_rank_share_pairs_through_the_kernels(L, G, Hq, Hkv, d):
    """What ONE ring rank computes (Sec. 3.2: rank r of a ring of G owns chunks r and 2G-1-r of 2G chunks and, over the
    rounds, sees every KV chunk at or before them): the pairs of zp_chunk_pairs(rank = r) through chunk_attn_partial
    and lse_merge give exactly the whole-sequence attention rows of that rank's Q chunks and touch no other row."""
    lengths = [40, L, 25]
    (q, k, v), cu = make(lengths, Hq, Hkv, d, 61)
    t0 = int(cu[1])
    ro, rl = oracle.varlen_attn_fwd(widen(q), widen(k), widen(v), cu)
    b = oracle.chunk_bounds(L, 2 * G)
    covered = np.zeros(L, bool)
    for r in range(G):
        pairs, merges, rows = B.chunk_pairs(t0, L, 2 * G, rank=r)
        # the descriptors are the oracle's pairs (qc, kc <= qc) of the two chunks this rank owns
        want = [(qc, kc) for qc in sorted((r, 2 * G - 1 - r)) for kc in range(qc + 1)]
        assert [(p.q_pos0, p.k_pos0, p.q_len, p.k_len) for p in pairs] == \
            [(b[qc], b[kc], b[qc + 1] - b[qc], b[kc + 1] - b[kc]) for qc, kc in want]
        op, lp = B.chunk_attn_partial(q, k, v, pairs, rows)
        o = torch.zeros_like(q); lse = torch.zeros((Hq, q.shape[0]), dtype=torch.float32, device=DEV)
        B.lse_merge(op, lp, merges, o, lse)
        torch.cuda.synchronize()
        mine = np.zeros(q.shape[0], bool)
        for c in (r, 2 * G - 1 - r):
            mine[t0 + b[c]:t0 + b[c + 1]] = True
        if mine.any():
            assert_close(f"rank {r} O", widen(o)[mine], ro[mine])
            assert_lse_close(f"rank {r} LSE", widen(lse)[:, mine], rl[:, mine])
        assert not o[torch.from_numpy(~mine).to(DEV)].any() and not lse[:, torch.from_numpy(~mine).to(DEV)].any()
        covered[mine[t0:t0 + L]] = True
    assert covered.all()      # the ranks' shares tile the sequence


def test_partial_rows_without_visible_keys():
    (q, k, v), cu = make([400], 2, 1, 128, 19)
    pairs = [dict(q_tok0=100, q_len=200, k_tok0=200, k_len=150, q_pos0=100, k_pos0=200, out_row0=3)]
    op, lp = B.chunk_attn_partial(q, k, v, pairs, 210)
    rop, rlp = oracle.chunk_attn_partial(widen(q), widen(k), widen(v), pairs, 210)
    assert_close("O_part", widen(op)[3:203], rop[3:203], bf16_out=False); assert_lse_close("LSE_part", widen(lp)[:, 3:203], rlp[:, 3:203])
    assert np.isneginf(widen(lp)[:, 3:103]).all()


@pytest.mark.parametrize("L,C,Hq,Hkv,d", [(1000, 4, 4, 2, 128), (777, 3, 2, 2, 64), (130, 8, 2, 1, 128), (5, 8, 2, 1, 64),
                                          (2100, 16, 2, 1, 128)])
def test_rounds_merged_in_place_equal_whole(L, C, Hq, Hkv, d):
    """chunk_attn_update over the ring rounds: after every round the running rows equal the oracle's partial results
    merged so far; after the last they equal the whole-sequence attention."""
    lengths = [50, L, 31]
    (q, k, v), cu = make(lengths, Hq, Hkv, d, 47)
    T = q.shape[0]
    t0 = int(cu[1])
    pairs, _, _ = B.chunk_pairs(t0, L, C)
    opairs, _, _ = oracle.causal_pairs(t0, L, C)
    order = [(qc, kc) for qc in range(C) for kc in range(qc + 1)]
    by = dict(zip(order, opairs))
    o_run = torch.full((T, Hq, d), float("nan"), dtype=torch.float32, device=DEV)     # anything: LSE = -inf says "empty"
    lse_run = torch.full((Hq, T), float("-inf"), dtype=torch.float32, device=DEV)
    ro = np.zeros((T, Hq, d)); rl = np.full((Hq, T), -np.inf)
    qw, kw, vw = widen(q), widen(k), widen(v)
    for rnd, ornd in zip(B.ring_rounds(t0, L, C), oracle.ring_rounds(C)):
        B.chunk_attn_update(q, k, v, rnd, o_run, lse_run)
        # oracle: this round's partials, then merged with the running rows as one more part
        plist = []
        rows = 0
        for pr in ornd:
            p = dict(by[pr]); p["out_row0"] = rows; rows += p["q_len"]; plist.append(p)
        pop, plp = oracle.chunk_attn_partial(qw, kw, vw, plist, rows)
        for p in plist:
            n, a, r0 = p["q_len"], p["q_tok0"], p["out_row0"]
            if n == 0:
                continue
            stack_o = np.concatenate([ro[a:a + n], pop[r0:r0 + n]]); stack_l = np.concatenate([rl[:, a:a + n], plp[:, r0:r0 + n]], axis=1)
            mo, ml = oracle.lse_merge(stack_o, stack_l, [(0, n, [0, n])], n)
            ro[a:a + n] = mo; rl[:, a:a + n] = ml
        torch.cuda.synchronize()
        seen = ~np.isneginf(rl[0])
        assert_lse_close("running LSE", widen(lse_run), rl)
        assert_close("running O", widen(o_run)[seen], ro[seen], bf16_out=False)
    wo, wl = oracle.varlen_attn_fwd(qw, kw, vw, cu)
    sl = slice(t0, t0 + L)
    assert_close("final O", widen(o_run)[sl], wo[sl], bf16_out=False); assert_lse_close("final LSE", widen(lse_run)[:, sl], wl[:, sl])
    assert np.isneginf(widen(lse_run)[:, :t0]).all() and np.isneginf(widen(lse_run)[:, t0 + L:]).all()
    bits = B.accum_to_bf16(torch.nan_to_num(o_run)).view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(bits, oracle.f32_to_bf16_bits(torch.nan_to_num(o_run).cpu().numpy()))


# ---- backward ----------------------------------------------------------------------------------------
def run_bwd(lengths, Hq, Hkv, d, seed, scale=0.0):
    (q, k, v, do), cu = make(lengths, Hq, Hkv, d, seed, with_dout=True)
    o, lse = B.varlen_attn_fwd(q, k, v, cu, scale=scale)
    dq, dk, dv = B.varlen_attn_bwd(do, q, k, v, o, lse, cu, scale=scale)
    torch.cuda.synchronize()
    rdq, rdk, rdv = oracle.varlen_attn_bwd(widen(do), widen(q), widen(k), widen(v), cu, scale=scale or None)
    assert_close("dQ", widen(dq), rdq); assert_close("dK", widen(dk), rdk); assert_close("dV", widen(dv), rdv)


def test_bwd_tiny_config():
    run_bwd(synth.lengths_tiny(1001), 4, 4, 64, 1001)


@pytest.mark.parametrize("lengths,Hq,Hkv,d", [
    ([1], 1, 1, 64), ([1, 1, 2, 3], 2, 1, 128), ([127, 128, 129], 2, 2, 128), ([64, 65, 63, 1], 4, 2, 64),
    ([700, 0, 333, 0], 8, 2, 128), ([900], 4, 1, 128), ([300, 41], 2, 2, 64)])
def test_bwd_edge_lengths(lengths, Hq, Hkv, d):
    run_bwd(lengths, Hq, Hkv, d, 23)


def test_bwd_custom_scale_and_deterministic():
    run_bwd([260, 100], 4, 2, 128, 29, scale=0.05)
    (q, k, v, do), cu = make([513, 200], 4, 2, 128, 31, with_dout=True)
    o, lse = B.varlen_attn_fwd(q, k, v, cu)
    a = B.varlen_attn_bwd(do, q, k, v, o, lse, cu); b = B.varlen_attn_bwd(do, q, k, v, o, lse, cu)
    for x, y in zip(a, b):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16))


@pytest.mark.parametrize("lengths,Hq,Hkv,d", [
    ([2048] * 4, 16, 16, 64),                                  # d=64 kernels, 1024 items each
    # forward, dQ and the short-sequence dK/dV kernel. The stated max-abs bound is NOT met by a few dK/dV elements of
    # these two GQA batches, all at 4 <= |ref| < 8 where the bf16 output grid alone takes 1.56e-2 of the 2e-2
    pytest.param([1536, 700, 2304, 1024, 128] * 3, 32, 8, 128, marks=pytest.mark.xfail(
        strict=True, raises=StatedBoundNotMet,
        reason="stated max-abs bound not met: dV 4 and 5, dK 1 of 2185728 elements per KV group, largest 2.45e-2 at |ref| 5.3")),
    # the long-sequence dK/dV kernel, 1024 items
    pytest.param([4096] * 4, 32, 8, 128, marks=pytest.mark.xfail(
        strict=True, raises=StatedBoundNotMet,
        reason="stated max-abs bound not met: dV 4, dK 1 of 2097152 elements of one KV group, largest 2.66e-2 at |ref| 5.0")),
])
def test_launches_with_a_claimed_tail(lengths, Hq, Hkv, d):
    """Launches of a thousand items and more hand the last of them out at run time (per-XCD counters, stealing): every
    item must still be computed exactly once, in every kernel and head dimension. The small parity cases above never
    reach that item count; these do, at sizes the oracle still finishes in seconds on a sample of KV groups."""
    (q, k, v, do), cu = make(lengths, Hq, Hkv, d, 67, with_dout=True)
    o, lse = B.varlen_attn_fwd(q, k, v, cu)
    dq, dk, dv = B.varlen_attn_bwd(do, q, k, v, o, lse, cu)
    torch.cuda.synchronize()
    grp = Hq // Hkv
    c = Checks()
    for g in (0, Hkv - 1):
        heads = list(range(g * grp, (g + 1) * grp))
        sel = lambda t, hs: widen(t[:, hs].contiguous())
        qw, kw, vw, dow = sel(q, heads), sel(k, [g]), sel(v, [g]), sel(do, heads)
        ro, rl = oracle.varlen_attn_fwd(qw, kw, vw, cu)
        rdq, rdk, rdv = oracle.varlen_attn_bwd(dow, qw, kw, vw, cu)
        c.close(f"O group {g}", sel(o, heads), ro)
        c.lse(f"LSE group {g}", widen(lse[heads].contiguous()), rl)
        c.close(f"dQ group {g}", sel(dq, heads), rdq)
        c.close(f"dK group {g}", sel(dk, [g]), rdk)
        c.close(f"dV group {g}", sel(dv, [g]), rdv)
    c.finish()


def test_two_streams_keep_their_own_scratch():
    """Calls issued on two streams overlap on the device; each stream has its own work-list scratch in the binding and
    the library's staging pool hands every call its own pinned slot, so both must give the single-stream results."""
    (qa, ka, va, doa), cua = make([900, 1300, 257, 64], 8, 2, 128, 81, with_dout=True)
    (qb, kb, vb, dob), cub = make([2048, 31, 700], 4, 4, 64, 82, with_dout=True)
    oa, la = B.varlen_attn_fwd(qa, ka, va, cua); ga = B.varlen_attn_bwd(doa, qa, ka, va, oa, la, cua)
    ob, lb = B.varlen_attn_fwd(qb, kb, vb, cub); gb = B.varlen_attn_bwd(dob, qb, kb, vb, ob, lb, cub)
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    for _ in range(3):
        with torch.cuda.stream(s1):
            o1, l1 = B.varlen_attn_fwd(qa, ka, va, cua, stream=s1); g1 = B.varlen_attn_bwd(doa, qa, ka, va, o1, l1, cua, stream=s1)
        with torch.cuda.stream(s2):
            o2, l2 = B.varlen_attn_fwd(qb, kb, vb, cub, stream=s2); g2 = B.varlen_attn_bwd(dob, qb, kb, vb, o2, l2, cub, stream=s2)
        s1.synchronize(); s2.synchronize()
        for got, ref in ((o1, oa), (l1, la), (o2, ob), (l2, lb), *zip(g1, ga), *zip(g2, gb)):
            assert torch.equal(got, ref)


def test_bwd_closed_forms_on_device():
    """Q = K = 0: the probabilities are uniform over the visible keys, so dQ and dK vanish exactly and
    dV_j = sum over the heads of the group and over queries i >= j of dO_i / (i + 1)."""
    lengths = [1, 300]
    Hq, Hkv, d = 4, 2, 128
    (q, k, v, do), cu = make(lengths, Hq, Hkv, d, 37, with_dout=True)
    q = torch.zeros_like(q); k = torch.zeros_like(k)
    o, lse = B.varlen_attn_fwd(q, k, v, cu)
    dq, dk, dv = B.varlen_attn_bwd(do, q, k, v, o, lse, cu)
    torch.cuda.synchronize()
    assert not dq.any() and not dk.any()
    dof = widen(do)
    w = dof[1:] / np.arange(1, 301)[:, None, None]                       # dO_i / (i + 1), i = 0..299
    suffix = np.cumsum(w[::-1], axis=0)[::-1]                            # sum over i >= j
    ref = suffix.reshape(300, Hkv, Hq // Hkv, d).sum(axis=2)
    assert_close("dV", widen(dv)[1:], ref)
    assert_close("dV of the length-1 sequence", widen(dv)[:1], dof[:1].reshape(1, Hkv, Hq // Hkv, d).sum(axis=2))


# ---- chunked backward --------------------------------------------------------------------------------
def run_chunked_bwd(lengths, which, C, Hq, Hkv, d, seed, scale=0.0):
    """Ring rounds of the chunked sequence `which` (Sec. 3.2): each round is one call that adds its pairs'
    contributions; after the last round the accumulators hold that sequence's rows of the whole backward."""
    (q, k, v, do), cu = make(lengths, Hq, Hkv, d, seed, with_dout=True)
    o, lse = B.varlen_attn_fwd(q, k, v, cu, scale=scale)
    t0, L = int(cu[which]), lengths[which]
    pairs, _, _ = B.chunk_pairs(t0, L, C)
    acc = [torch.zeros(x.shape, dtype=torch.float32, device=DEV) for x in (q, k, v)]
    for rnd in B.ring_rounds(t0, L, C):
        B.chunk_attn_partial_bwd(do, q, k, v, o, lse, rnd, *acc, scale=scale)
    torch.cuda.synchronize()
    rdq, rdk, rdv = oracle.varlen_attn_bwd(widen(do), widen(q), widen(k), widen(v), cu, scale=scale or None)
    sl = slice(t0, t0 + L)
    for name, a, r in zip(("dQ", "dK", "dV"), acc, (rdq, rdk, rdv)):
        assert_close(name, a.double().cpu().numpy()[sl], r[sl], bf16_out=False)
        assert not a[:t0].any() and not a[t0 + L:].any()      # rows of the other sequences are untouched
        bits = B.accum_to_bf16(a).view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(bits, oracle.f32_to_bf16_bits(a.cpu().numpy()))     # the final rounding is bit-exact
    return acc


@pytest.mark.parametrize("L,C,Hq,Hkv,d", [(1000, 4, 4, 2, 128), (777, 3, 2, 2, 64), (130, 8, 2, 1, 128), (5, 8, 2, 1, 64),
                                          (600, 1, 4, 4, 128), (1500, 2, 8, 2, 128), (2100, 16, 2, 1, 128)])
def test_chunked_backward_rounds_equal_whole_backward(L, C, Hq, Hkv, d):
    run_chunked_bwd([50, L, 31], 1, C, Hq, Hkv, d, 37)


def test_chunked_backward_custom_scale_and_single_round_against_oracle():
    run_chunked_bwd([300], 0, 2, 4, 2, 128, 41, scale=0.07)
    # one off-diagonal round on its own, against the oracle's pair-restricted sums
    lengths = [900]
    (q, k, v, do), cu = make(lengths, 4, 2, 128, 43, with_dout=True)
    o, lse = B.varlen_attn_fwd(q, k, v, cu)
    pairs, _, _ = B.chunk_pairs(0, 900, 4)
    rnd = B.ring_rounds(0, 900, 4)[2]
    acc = [torch.zeros(x.shape, dtype=torch.float32, device=DEV) for x in (q, k, v)]
    B.chunk_attn_partial_bwd(do, q, k, v, o, lse, rnd, *acc)
    B.chunk_attn_partial_bwd(do, q, k, v, o, lse, rnd, *acc)     # a second call adds the same again
    torch.cuda.synchronize()
    ro, rl = oracle.varlen_attn_fwd(widen(q), widen(k), widen(v), cu)
    D = np.einsum("thc,thc->ht", widen(do), widen(o))           # the device's own O, as the kernel reads it
    opairs, _, _ = oracle.causal_pairs(0, 900, 4)
    by = {}
    n = 0
    for qc in range(4):
        for kc in range(qc + 1):
            by[(qc, kc)] = opairs[n]; n += 1
    ref = [np.zeros(x.shape) for x in (q, k, v)]
    oracle.chunk_attn_partial_bwd(widen(do), widen(q), widen(k), widen(v), [by[pr] for pr in oracle.ring_rounds(4)[2]], rl, D, *ref)
    for name, a, r in zip(("dQ", "dK", "dV"), acc, ref):
        assert_close(name, a.double().cpu().numpy(), 2 * r, bf16_out=False)


def test_mfma_probe_runs_and_is_deterministic():
    a = B.mfma_probe(50, True).clone(); b = B.mfma_probe(50, True)
    torch.cuda.synchronize()
    assert torch.isfinite(a).all() and torch.equal(a, b) and a.abs().max() > 0
    assert not B.mfma_probe(50, False).any()


# ---- a whole node's placement on one GPU ----------------------------------------------------------------
@pytest.mark.parametrize("lengths,P,N,L,Hq,Hkv,d", [
    # one intra-node ring, local sequences. The stated max-abs bound is NOT met by dV here: 2 of 739072 elements,
    # largest 2.15e-2 at |ref| 6.4, where the bf16 output grid alone takes 1.56e-2 of the 2e-2 (everything else passes)
    pytest.param([700, 90, 300, 1500, 64, 200, 33], 4, 1, 800, 4, 2, 128, marks=pytest.mark.xfail(
        strict=True, raises=StatedBoundNotMet, reason="stated max-abs bound not met: dV, 2 of 739072 elements, largest 2.15e-2 at |ref| 6.4")),
    ([2600, 150, 400, 90, 1100, 60], 2, 2, 700, 2, 1, 64),           # an inter-node ring over both nodes
    ([100, 200, 50], 4, 1, 400, 2, 2, 64)])                          # everything local
def test_node_placement_end_to_end(lengths, P, N, L, Hq, Hkv, d):
    """Partitioner -> attention layout -> remap plan -> engine, against the oracle's whole-sequence attention of the
    batch as drawn: inputs arrive in the token-balanced layout, outputs are compared there too."""
    from paper_2509_21841_amd.node import NodeJob, NodePlan
    plan = NodePlan(lengths, P, N, L, b_intra=1, b_inter=5)
    T = plan.T
    (q0, k0, v0, do0), cu0 = make(lengths, Hq, Hkv, d, 53, with_dout=True)      # the batch as drawn
    to_bal = torch.from_numpy(plan.orig[plan.idx]).to(DEV)                      # balanced position -> drawn position
    qb, kb, vb, dob = (x[to_bal].contiguous() for x in (q0, k0, v0, do0))       # what the linear modules hand over
    job = NodeJob(plan, Hq, Hkv, d, DEV)
    qa, ka, va, doa = (job.to_attention(x) for x in (qb, kb, vb, dob))
    assert torch.equal(qa.view(torch.int16), q0[torch.from_numpy(plan.orig).to(DEV)].view(torch.int16))
    o, _ = job.forward(qa, ka, va)
    ob = job.to_balanced(o)
    dq, dk, dv = job.backward(doa, qa, ka, va)
    dqb, dkb, dvb = (job.to_balanced(x) for x in (dq, dk, dv))
    torch.cuda.synchronize()
    ro, _ = oracle.varlen_attn_fwd(widen(q0), widen(k0), widen(v0), cu0)
    rdq, rdk, rdv = oracle.varlen_attn_bwd(widen(do0), widen(q0), widen(k0), widen(v0), cu0)
    sel = plan.orig[plan.idx]
    # the balanced layout gives every rank its target share
    from oracle import remap_planner as RP
    assert [int(x) for x in np.asarray(plan.M).sum(axis=1)] == RP.surplus_deficit(plan.A)[0]
    c = Checks()
    c.close("O", widen(ob), ro[sel]); c.close("dQ", widen(dqb), rdq[sel])
    c.close("dK", widen(dkb), rdk[sel]); c.close("dV", widen(dvb), rdv[sel])
    c.finish()
