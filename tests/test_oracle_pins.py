"""Pins of the fp64 oracle against things other than itself: closed forms, invariants, brute force with a
different loop order, finite differences and a library routine (CPU only)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_21841_amd import synth


def rand_case(lengths, Hq, Hkv, d, seed, bf16=True):
    T = int(sum(lengths))
    if bf16:
        q, k, v, do = synth.make_qkv(T, Hq, Hkv, d, seed, with_dout=True)
        f = lambda x: oracle.bf16_bits_to_f64(synth.bf16_bits(x))
        return f(q), f(k), f(v), f(do), synth.cu_seqlens(lengths)
    r = np.random.default_rng(seed)
    return (r.standard_normal((T, Hq, d)), r.standard_normal((T, Hkv, d)), r.standard_normal((T, Hkv, d)),
            r.standard_normal((T, Hq, d)), synth.cu_seqlens(lengths))


def brute_fwd(q, k, v, cu, scale):
    """Materialised-P definition, keys outermost in the score loop, two-pass softmax."""
    T, Hq, d = q.shape
    grp = Hq // k.shape[1]
    o = np.zeros_like(q); lse = np.zeros((Hq, T))
    for s in range(len(cu) - 1):
        t0, t1 = int(cu[s]), int(cu[s + 1]); L = t1 - t0
        for h in range(Hq):
            S = np.full((L, L), -np.inf)
            for j in range(L):
                for i in range(j, L):
                    S[i, j] = scale * sum(q[t0 + i, h, c] * k[t0 + j, h // grp, c] for c in range(d))
            for i in range(L):
                e = np.exp(S[i] - S[i].max()); Z = e.sum()
                P = e / Z
                lse[h, t0 + i] = np.log(Z) + S[i].max()
                o[t0 + i, h] = P @ v[t0:t1, h // grp]
    return o, lse


def test_bf16_widening_exact():
    x = torch.tensor([1.0, -2.5, 3.140625, 1e-3, 65280.0, -0.0], dtype=torch.bfloat16)
    assert np.array_equal(oracle.bf16_bits_to_f64(synth.bf16_bits(x)), x.to(torch.float64).numpy())


@pytest.mark.parametrize("d", [4, 64])
def test_brute_force_tiny(d):  # a different loop order and softmax form agree
    lengths = [1, 7, 19, 2] if d == 64 else [1, 13, 40, 2, 5]
    q, k, v, _, cu = rand_case(lengths, 4, 2, d, 7, bf16=False)
    o, lse = oracle.varlen_attn_fwd(q, k, v, cu, scale=0.37)
    ob, lb = brute_fwd(q, k, v, cu, 0.37)
    assert np.abs(o - ob).max() < 1e-12 and np.abs(lse - lb).max() < 1e-12


def test_length_one_returns_v():
    q, k, v, _, cu = rand_case([1, 1, 1], 4, 2, 8, 3, bf16=False)
    o, lse = oracle.varlen_attn_fwd(q, k, v, cu)
    for t in range(3):
        for h in range(4):
            assert np.array_equal(o[t, h], v[t, h // 2])
            assert abs(lse[h, t] - (q[t, h] @ k[t, h // 2]) / np.sqrt(8)) < 1e-14


def test_zero_q_gives_prefix_mean_and_log_count():
    lengths = [5, 33]
    q, k, v, _, cu = rand_case(lengths, 2, 2, 16, 5, bf16=False)
    o, lse = oracle.varlen_attn_fwd(np.zeros_like(q), k, v, cu, scale=3.0)
    for s, L in enumerate(lengths):
        t0 = cu[s]
        for i in range(L):
            assert np.abs(o[t0 + i] - v[t0:t0 + i + 1].mean(axis=0)).max() < 1e-13
            assert np.abs(lse[:, t0 + i] - np.log(i + 1)).max() < 1e-13  # natural log, diagonal included


def test_constant_v_and_default_scale():
    q, k, v, do, cu = rand_case([17, 9], 4, 4, 8, 11, bf16=False)
    c = np.arange(8.0)
    v[:] = c
    o, _ = oracle.varlen_attn_fwd(q, k, v, cu)
    assert np.abs(o - c).max() < 1e-13
    # constant V makes O independent of the scores: no gradient reaches Q or K
    dq, dk, dv = oracle.varlen_attn_bwd(do, q, k, v, cu)
    assert np.abs(dq).max() < 1e-12 and np.abs(dk).max() < 1e-12
    # default scale is 1/sqrt(d)
    o1, l1 = oracle.varlen_attn_fwd(q, k, v + np.random.default_rng(0).standard_normal(v.shape), cu)
    o2, l2 = oracle.varlen_attn_fwd(q, k, v + np.random.default_rng(0).standard_normal(v.shape), cu, scale=8 ** -0.5)
    assert np.abs(o1 - o2).max() < 1e-13 and np.abs(l1 - l2).max() < 1e-13


def test_sdpa_library_second_opinion_fwd_and_bwd():
    lengths = [31, 64, 5]
    Hq, Hkv, d = 4, 2, 16
    q, k, v, do, cu = rand_case(lengths, Hq, Hkv, d, 21, bf16=False)
    o, lse = oracle.varlen_attn_fwd(q, k, v, cu)
    dq, dk, dv = oracle.varlen_attn_bwd(do, q, k, v, cu)
    tq, tk, tv = [torch.from_numpy(x).requires_grad_(True) for x in (q, k, v)]
    outs = []
    for s in range(len(lengths)):
        a, b = int(cu[s]), int(cu[s + 1])
        kk = tk[a:b].repeat_interleave(Hq // Hkv, dim=1); vv = tv[a:b].repeat_interleave(Hq // Hkv, dim=1)
        outs.append(torch.nn.functional.scaled_dot_product_attention(
            tq[a:b].transpose(0, 1)[None], kk.transpose(0, 1)[None], vv.transpose(0, 1)[None], is_causal=True)[0].transpose(0, 1))
    ot = torch.cat(outs)
    ot.backward(torch.from_numpy(do))
    assert np.abs(ot.detach().numpy() - o).max() < 1e-12
    assert np.abs(tq.grad.numpy() - dq).max() < 1e-12
    assert np.abs(tk.grad.numpy() - dk).max() < 1e-12
    assert np.abs(tv.grad.numpy() - dv).max() < 1e-12


def test_finite_differences_bwd():
    lengths = [12, 30]
    Hq, Hkv, d = 4, 2, 8
    q, k, v, do, cu = rand_case(lengths, Hq, Hkv, d, 33, bf16=False)
    dq, dk, dv = oracle.varlen_attn_bwd(do, q, k, v, cu, scale=0.5)
    loss = lambda q_, k_, v_: float((oracle.varlen_attn_fwd(q_, k_, v_, cu, scale=0.5)[0] * do).sum())
    r = np.random.default_rng(1)
    eps = 1e-5
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        for _ in range(40):
            idx = tuple(r.integers(0, n) for n in x.shape)
            xp, xm = x.copy(), x.copy(); xp[idx] += eps; xm[idx] -= eps
            args_p = {"q": (xp, k, v), "k": (q, xp, v), "v": (q, k, xp)}[name]
            args_m = {"q": (xm, k, v), "k": (q, xm, v), "v": (q, k, xm)}[name]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - g[idx]) < 1e-7 * max(1.0, abs(g[idx])), (name, idx, fd, g[idx])


def test_bwd_sample_equals_full():
    lengths = [20, 45, 3]
    q, k, v, do, cu = rand_case(lengths, 4, 2, 8, 41)
    dq, dk, dv = oracle.varlen_attn_bwd(do, q, k, v, cu)
    qs = [(0, 0), (19, 3), (20, 1), (64, 2), (67, 0)]
    ks = [(0, 0), (19, 1), (33, 0), (64, 1), (67, 1)]
    sq, sk, sv = oracle.varlen_attn_bwd_sample(do, q, k, v, cu, qs, ks)
    for n, (t, h) in enumerate(qs):
        assert np.array_equal(sq[n], dq[t, h])
    for n, (t, g) in enumerate(ks):
        assert np.array_equal(sk[n], dk[t, g]) and np.array_equal(sv[n], dv[t, g])


@pytest.mark.parametrize("C", [1, 2, 3, 4])
def test_chunked_then_merged_equals_whole(C):
    lengths = [37, 101, 6]
    q, k, v, _, cu = rand_case(lengths, 4, 2, 16, 51)
    o, lse = oracle.varlen_attn_fwd(q, k, v, cu)
    T = q.shape[0]
    om = np.full_like(o, np.nan); lm = np.full_like(lse, np.nan)
    for s, L in enumerate(lengths):
        pairs, merges, rows = oracle.causal_pairs(int(cu[s]), L, C)
        assert len(pairs) == C * (C + 1) // 2
        op, lp = oracle.chunk_attn_partial(q, k, v, pairs, rows)
        assert not np.isnan(op).any()
        om, lm = oracle.lse_merge(op, lp, merges, T, om, lm)
    assert np.abs(om - o).max() < 1e-13 and np.abs(lm - lse).max() < 1e-13


def test_chunk_bounds_are_floor_and_near_equal():
    for L in (1, 7, 100, 38400, 65535):
        for C in (1, 2, 4, 8):
            b = oracle.chunk_bounds(L, C)
            assert b[0] == 0 and b[-1] == L and all(b[c] == (c * L) // C for c in range(C + 1))
            sizes = np.diff(b)
            assert sizes.max() - sizes.min() <= 1


def test_partial_with_no_visible_key_and_partial_visibility():
    q, k, v, _, cu = rand_case([16], 2, 1, 8, 61)
    # keys 8..15 against queries 4..11: queries 4..7 see nothing, query 8+r sees r+1 keys
    pairs = [dict(q_tok0=4, q_len=8, k_tok0=8, k_len=8, q_pos0=4, k_pos0=8, out_row0=0)]
    op, lp = oracle.chunk_attn_partial(q, k, v, pairs, 8)
    assert np.all(np.isneginf(lp[:, :4])) and np.all(op[:4] == 0)
    for r in range(4):
        i = 8 + r
        sc = (k[8:i + 1, 0] @ q[i, 1]) / np.sqrt(8)
        assert abs(lp[1, 4 + r] - np.log(np.exp(sc).sum())) < 1e-13
    # merging with an all -inf partial changes nothing; all -inf rows stay (-inf, 0)
    o2, l2 = oracle.lse_merge(np.concatenate([op, op]), np.concatenate([lp, lp], axis=1), [(0, 8, [0, 8])], 8)
    assert np.all(np.isneginf(l2[:, :4])) and np.all(o2[:4] == 0)


def test_merge_closed_forms_and_associativity():
    r = np.random.default_rng(3)
    n, H, d = 5, 2, 4
    op = r.standard_normal((3 * n, H, d)); lp = r.standard_normal((H, 3 * n))
    # one part: identity
    o1, l1 = oracle.lse_merge(op, lp, [(0, n, [n])], n)
    assert np.array_equal(o1, op[n:2 * n]) and np.array_equal(l1, lp[:, n:2 * n])
    # two parts with equal LSE: plain average, LSE + ln 2
    lp2 = lp.copy(); lp2[:, n:2 * n] = lp2[:, :n]
    o2, l2 = oracle.lse_merge(op, lp2, [(0, n, [0, n])], n)
    assert np.abs(o2 - 0.5 * (op[:n] + op[n:2 * n])).max() < 1e-14
    assert np.abs(l2 - (lp2[:, :n] + np.log(2))).max() < 1e-14
    # weights are exp(LSE_p - LSE): softmax over the parts
    o3, l3 = oracle.lse_merge(op, lp, [(0, n, [0, n, 2 * n])], n)
    w = np.exp(lp.reshape(H, 3, n)); w = w / w.sum(axis=1, keepdims=True)
    ref = sum(w[:, p].T[:, :, None] * op[p * n:(p + 1) * n] for p in range(3))
    assert np.abs(o3 - ref).max() < 1e-14
    # associativity / commutativity: ((0,1),2) == (2,0,1)
    o01, l01 = oracle.lse_merge(op, lp, [(0, n, [0, n])], n)
    oc = np.concatenate([o01, op[2 * n:]]); lc = np.concatenate([l01, lp[:, 2 * n:]], axis=1)
    o4, l4 = oracle.lse_merge(oc, lc, [(0, n, [n, 0])], n)
    assert np.abs(o4 - o3).max() < 1e-14 and np.abs(l4 - l3).max() < 1e-14


def test_packing_order_invariance_and_no_leakage():
    lengths = [9, 30, 17, 4]
    q, k, v, do, cu = rand_case(lengths, 2, 2, 8, 71)
    o, lse = oracle.varlen_attn_fwd(q, k, v, cu)
    dq, dk, dv = oracle.varlen_attn_bwd(do, q, k, v, cu)
    perm = [2, 0, 3, 1]
    tok = np.concatenate([np.arange(cu[s], cu[s + 1]) for s in perm])
    cu2 = synth.cu_seqlens([lengths[s] for s in perm])
    o2, lse2 = oracle.varlen_attn_fwd(q[tok], k[tok], v[tok], cu2)
    dq2, dk2, dv2 = oracle.varlen_attn_bwd(do[tok], q[tok], k[tok], v[tok], cu2)
    assert np.array_equal(o2, o[tok]) and np.array_equal(lse2, lse[:, tok])
    assert np.array_equal(dq2, dq[tok]) and np.array_equal(dk2, dk[tok]) and np.array_equal(dv2, dv[tok])
    # dropping the last sequences changes no earlier output
    n = int(cu[2])
    o3, _ = oracle.varlen_attn_fwd(q[:n], k[:n], v[:n], cu[:3])
    assert np.array_equal(o3, o[:n])


def test_gqa_equals_mha_on_repeated_kv():
    lengths = [23, 8]
    q, k, v, do, cu = rand_case(lengths, 8, 2, 8, 81)
    o, lse = oracle.varlen_attn_fwd(q, k, v, cu)
    dq, dk, dv = oracle.varlen_attn_bwd(do, q, k, v, cu)
    kr, vr = np.repeat(k, 4, axis=1), np.repeat(v, 4, axis=1)
    o2, lse2 = oracle.varlen_attn_fwd(q, kr, vr, cu)
    dq2, dk2, dv2 = oracle.varlen_attn_bwd(do, q, kr, vr, cu)
    assert np.array_equal(o, o2) and np.array_equal(lse, lse2) and np.array_equal(dq, dq2)
    assert np.abs(dk2.reshape(-1, 2, 4, 8).sum(2) - dk).max() < 1e-12
    assert np.abs(dv2.reshape(-1, 2, 4, 8).sum(2) - dv).max() < 1e-12


def test_causality():
    q, k, v, do, cu = rand_case([40], 2, 1, 8, 91)
    o, lse = oracle.varlen_attn_fwd(q, k, v, cu)
    dq, dk, dv = oracle.varlen_attn_bwd(do, q, k, v, cu)
    j = 25
    q2, k2, v2, do2 = q.copy(), k.copy(), v.copy(), do.copy()
    q2[j:] += 1.0; k2[j:] -= 2.0; v2[j:] *= 3.0
    o2, lse2 = oracle.varlen_attn_fwd(q2, k2, v2, cu)
    assert np.array_equal(o2[:j], o[:j]) and np.array_equal(lse2[:, :j], lse[:, :j])
    assert not np.array_equal(o2[j], o[j])
    # dK_j, dV_j depend only on rows i >= j: changing dO on earlier rows leaves them unchanged
    do2[:j] = 0.0
    _, dk2, dv2 = oracle.varlen_attn_bwd(do2, q, k, v, cu)
    assert np.array_equal(dk2[j:], dk[j:]) and np.array_equal(dv2[j:], dv[j:])


def test_ring_schedule_balance_and_cover():
    """Sec. 3.2: 2G chunks, rank i owns chunks i and 2G-1-i, G rounds.  Every rank does exactly two
    block-units per round (a diagonal pair is half a block) and the ranks together cover each causal
    chunk pair exactly once."""
    golden = {}
    for line in open(__import__("os").path.join(__import__("os").path.dirname(__file__), "golden", "ring_chunk_ownership.txt")):
        if line.strip() and not line.startswith("#"):
            G, rank, a, b = map(int, line.split())
            golden[(G, rank)] = (a, b)
    for G in (1, 2, 3, 4, 8):
        sched = oracle.ring_schedule(G)
        seen = []
        for i in range(G):
            owned = {qc for rnd in sched[i] for qc, _ in rnd}
            if (G, i) in golden:
                assert owned == set(golden[(G, i)])
            for rnd in sched[i]:
                units = sum(0.5 if qc == kc else 1.0 for qc, kc in rnd)
                assert units == 2.0
                seen += rnd
        C = 2 * G
        assert sorted(seen) == sorted((qc, kc) for qc in range(C) for kc in range(qc + 1))


def test_remap_pins():
    r = np.random.default_rng(5)
    n = 257
    x = r.integers(0, 2 ** 16, size=(n, 3, 8), dtype=np.uint16)
    idx = r.permutation(n).astype(np.int32)
    inv = np.empty_like(idx); inv[idx] = np.arange(n, dtype=np.int32)
    g = oracle.remap_tokens(x, idx, 0)
    assert np.array_equal(g, x[idx])                                   # gather is numpy fancy indexing
    assert np.array_equal(oracle.remap_tokens(g, idx, 1), x)           # scatter undoes gather
    assert np.array_equal(oracle.remap_tokens(g, inv, 0), x)           # inverse permutation undoes it too
    assert np.array_equal(oracle.remap_tokens(x, inv, 1), g)           # gather(idx) == scatter(idx^-1)
    assert np.array_equal(oracle.remap_tokens(x, np.arange(n), 0), x)  # identity is a copy
    rows = lambda a: sorted(bytes(row) for row in a.reshape(n, -1))
    assert rows(g) == rows(x)                                          # multiset of rows preserved


def test_balanced_layout_is_a_permutation_moving_whole_sequences():
    lengths = synth.lengths_lognormal(8192, 9, lo=16, hi=2048, median=256)
    idx, attn_lengths, order = synth.balanced_attention_layout(lengths, R=4)
    assert sorted(idx.tolist()) == list(range(8192))
    assert sorted(attn_lengths) == sorted(lengths) and [lengths[s] for s in order] == attn_lengths
    cu = synth.cu_seqlens(lengths); pos = 0
    for s in order:
        assert np.array_equal(idx[pos:pos + lengths[s]], np.arange(cu[s], cu[s + 1])); pos += lengths[s]


@pytest.mark.parametrize("C", [1, 2, 4])
def test_chunked_backward_sums_to_whole_backward(C):
    """Sec. 3.2 / 5.4: the per-pair backward contributions, with the merged row statistics, add up to the backward
    of the whole sequence; within a round no Q chunk and no KV chunk appears twice."""
    lengths = [29, 70]
    q, k, v, do, cu = rand_case(lengths, 4, 2, 8, 101)
    o, lse = oracle.varlen_attn_fwd(q, k, v, cu)
    D = np.einsum("thc,thc->ht", do, o)
    dq, dk, dv = oracle.varlen_attn_bwd(do, q, k, v, cu)
    aq, ak, av = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for s, L in enumerate(lengths):
        pairs, _, _ = oracle.causal_pairs(int(cu[s]), L, C)
        order = [(qc, kc) for qc in range(C) for kc in range(qc + 1)]     # the enumeration order of causal_pairs
        by = dict(zip(order, pairs))
        for rnd in oracle.ring_rounds(C):
            assert len({qc for qc, _ in rnd}) == len(rnd) and len({kc for _, kc in rnd}) == len(rnd)
            oracle.chunk_attn_partial_bwd(do, q, k, v, [by[pr] for pr in rnd], lse, D, aq, ak, av)
    assert sorted(pr for rnd in oracle.ring_rounds(C) for pr in rnd) == sorted((qc, kc) for qc in range(C) for kc in range(qc + 1))
    assert np.abs(aq - dq).max() < 1e-12 and np.abs(ak - dk).max() < 1e-12 and np.abs(av - dv).max() < 1e-12


def test_chunked_backward_single_pair_closed_form():
    """One query row against one key chunk, d = 1, checked against the formulas written out by hand."""
    q = np.array([[[0.5]], [[2.0]]]); k = np.array([[[1.0]], [[-1.0]]]); v = np.array([[[3.0]], [[5.0]]])
    do = np.array([[[1.0]], [[2.0]]]); cu = np.array([0, 2], np.int32)
    o, lse = oracle.varlen_attn_fwd(q, k, v, cu, scale=1.0)
    D = np.einsum("thc,thc->ht", do, o)
    aq, ak, av = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    pair = dict(q_tok0=1, q_len=1, k_tok0=0, k_len=1, q_pos0=1, k_pos0=0, out_row0=0)   # row 1 against key 0 only
    oracle.chunk_attn_partial_bwd(do, q, k, v, [pair], lse, D, aq, ak, av, scale=1.0)
    p10 = np.exp(2.0 * 1.0) / (np.exp(2.0) + np.exp(-2.0))
    ds = p10 * (2.0 * 3.0 - D[0, 1])
    assert abs(aq[1, 0, 0] - ds * 1.0) < 1e-14 and abs(ak[0, 0, 0] - ds * 2.0) < 1e-14 and abs(av[0, 0, 0] - p10 * 2.0) < 1e-14
    assert aq[0, 0, 0] == 0 and ak[1, 0, 0] == 0 and av[1, 0, 0] == 0


def test_f32_to_bf16_rounding_pins():
    """Round to nearest even on the 16 dropped bits: hand-picked bit patterns."""
    f = lambda bits: np.array([bits], np.uint32).view(np.float32)
    r = lambda bits: int(oracle.f32_to_bf16_bits(f(bits))[0])
    assert r(0x3F800000) == 0x3F80            # 1.0
    assert r(0x3F808000) == 0x3F80            # tie, keep even
    assert r(0x3F818000) == 0x3F82            # tie, round up to even
    assert r(0x3F808001) == 0x3F81            # above the tie
    assert r(0x3F807FFF) == 0x3F80            # below the tie
    assert r(0xBF818000) == 0xBF82            # sign is carried
    assert r(0x7F7FFFFF) == 0x7F80            # largest float rounds to infinity
    assert r(0x00000000) == 0 and r(0x80000000) == 0x8000
    x = np.random.default_rng(3).standard_normal(4096).astype(np.float32)
    back = oracle.bf16_bits_to_f64(oracle.f32_to_bf16_bits(x))
    assert (np.abs(back - x) <= np.abs(x) * 2.0 ** -8).all()    # half an ulp of an 8-bit significand (7 stored bits)
