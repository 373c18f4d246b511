"""Host-side checks that need no GPU: the library loads, exports every declared symbol, validates arguments
before touching the device, and its chunk-pair helper agrees with the oracle's enumeration."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2509_21841_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions(header="zeppelin_attn.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(\w+)\s*\([^;{]*\)\s*;", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"varlen_attn_fwd", "varlen_attn_bwd", "chunk_attn_partial", "lse_merge", "remap_tokens",
            "zp_workspace_bytes", "zp_strerror", "zp_chunk_pairs"} <= set(names)
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n
    assert not any(n.startswith("zp_mfma") or n.startswith("zp_profile") for n in names)   # measurement aids live elsewhere
    # the bench-side header: per-kernel timing comes from the engine's library, the probe from its own small one
    bench = declared_functions("zeppelin_attn_bench.h")
    assert sorted(bench) == ["zp_mfma_probe", "zp_profile_count", "zp_profile_enable", "zp_profile_get"]
    for n in bench:
        assert hasattr(B.bench_lib() if n == "zp_mfma_probe" else L, n), n
    assert not hasattr(L, "zp_mfma_probe")
    assert sorted(f for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h")) == ["zeppelin_attn.h", "zeppelin_attn_bench.h"]


def test_strerror_texts():
    L = B.lib()
    assert L.zp_strerror(0) == b"ok"
    for code in (-1, -2, -3):
        assert len(L.zp_strerror(code)) > 3


def _fwd_rc(sh, cu, q=1 << 12, k=1 << 12, v=1 << 12, o=1 << 12, lse=1 << 12, qs=None, ws=1 << 12, wsb=1 << 20):
    L = B.lib()
    cu = np.ascontiguousarray(cu, np.int32)
    qs = sh.Hq * sh.d if qs is None else qs
    return L.varlen_attn_fwd(q, k, v, qs, sh.Hkv * sh.d, sh.Hkv * sh.d, cu.ctypes.data_as(ctypes.c_void_p), None, o,
                             sh.Hq * sh.d, lse, ctypes.byref(sh), ws, wsb, None)


def test_fwd_argument_validation_without_device():
    ok = B.make_shape(100, 2, 4, 2, 64)
    assert _fwd_rc(ok, [0, 40, 100], q=0) == -1                      # null pointer
    assert _fwd_rc(ok, [1, 40, 100]) == -1                           # cu[0] != 0
    assert _fwd_rc(ok, [0, 60, 40]) == -1                            # not monotone
    assert _fwd_rc(ok, [0, 40, 99]) == -1                            # cu[S] != T
    assert _fwd_rc(B.make_shape(100, 2, 4, 2, 96), [0, 40, 100]) == -2   # head dim
    assert _fwd_rc(B.make_shape(100, 2, 4, 3, 64), [0, 40, 100]) == -2   # Hq % Hkv
    assert _fwd_rc(ok, [0, 40, 100], qs=100) == -1                   # token stride below Hq*d
    assert _fwd_rc(ok, [0, 40, 100], ws=0) == -3                     # no workspace
    assert _fwd_rc(ok, [0, 40, 100], wsb=16) == -3                   # workspace too small
    assert _fwd_rc(ok, [0, 40, 100], ws=(1 << 12) + 16) == -3        # misaligned workspace
    assert _fwd_rc(B.make_shape(0, 1, 4, 2, 64), [0, 0]) == 0        # empty batch is a no-op


def test_remap_and_merge_validation_without_device():
    L = B.lib()
    assert L.remap_tokens(1 << 12, 1 << 20, 24, 1 << 22, 10, 0, None) == -2     # row_bytes % 16
    assert L.remap_tokens(1 << 12, 1 << 20, 32, 1 << 22, 10, 2, None) == -1     # bad mode
    assert L.remap_tokens(1 << 12, (1 << 12) + 64, 32, 1 << 22, 10, 0, None) == -1  # overlap
    assert L.remap_tokens(0, 1 << 20, 32, 1 << 22, 10, 0, None) == -1
    assert L.remap_tokens(1 << 12, 1 << 20, 32, 1 << 22, 0, 0, None) == 0       # nothing to move
    sh = B.make_shape(100, 0, 4, 4, 64)
    m = (B.ZpMerge * 1)()
    m[0].out_tok0, m[0].len, m[0].n_parts = 90, 20, 1                            # runs past T
    assert L.lse_merge(1 << 12, 1 << 12, 100, m, 1, 1 << 12, 256, 1 << 12, ctypes.byref(sh), 1 << 12, 1 << 20, None) == -1
    m[0].out_tok0, m[0].len, m[0].n_parts = 0, 20, 17                            # too many parts
    assert L.lse_merge(1 << 12, 1 << 12, 100, m, 1, 1 << 12, 256, 1 << 12, ctypes.byref(sh), 1 << 12, 1 << 20, None) == -1
    p = (B.ZpPair * 1)()
    p[0].q_tok0, p[0].q_len, p[0].k_tok0, p[0].k_len, p[0].out_row0 = 0, 50, 60, 50, 0   # keys past T
    assert L.chunk_attn_partial(1 << 12, 1 << 12, 1 << 12, 256, 256, 256, p, 1, 1 << 12, 1 << 12, 50, ctypes.byref(sh),
                                1 << 12, 1 << 20, None) == -1


def test_chunked_backward_validation_without_device():
    L = B.lib()
    sh = B.make_shape(200, 0, 4, 4, 64)
    A = 1 << 12

    def rc(pairs, ws=A, wsb=1 << 22, dq=A):
        arr = (B.ZpPair * len(pairs))()
        for n, (qt, ql, kt, kl) in enumerate(pairs):
            arr[n].q_tok0, arr[n].q_len, arr[n].k_tok0, arr[n].k_len, arr[n].q_pos0, arr[n].k_pos0 = qt, ql, kt, kl, qt, kt
        return L.chunk_attn_partial_bwd(A, A, A, A, A, A, 256, 256, 256, 256, 256, arr, len(pairs), dq, A, A,
                                        ctypes.byref(sh), ws, wsb, None)

    assert rc([(100, 50, 0, 50), (120, 50, 50, 50)]) == -1      # two pairs share query rows: the adds would race
    assert rc([(100, 50, 0, 50), (150, 50, 40, 50)]) == -1      # two pairs share key rows
    assert rc([(100, 101, 0, 50)]) == -1                        # queries past T
    assert rc([(100, 50, 0, 50)], dq=0) == -1                   # null accumulator
    assert rc([(100, 50, 0, 50)], dq=A + 4) == -1               # misaligned accumulator
    assert rc([(100, 50, 0, 50)], ws=0) == -3
    assert rc([(100, 50, 0, 50)], wsb=64) == -3
    assert rc([]) == 0                                          # empty round
    arr = (B.ZpPair * 2)()
    for n, (qt, ql, kt, kl) in enumerate([(100, 50, 0, 50), (120, 50, 50, 50)]):
        arr[n].q_tok0, arr[n].q_len, arr[n].k_tok0, arr[n].k_len, arr[n].q_pos0, arr[n].k_pos0 = qt, ql, kt, kl, qt, kt
    upd = lambda n, o=A: L.chunk_attn_update(A, A, A, 256, 256, 256, arr, n, o, A, ctypes.byref(sh), A, 1 << 22, None)
    assert upd(2) == -1                                         # two pairs share query rows
    assert upd(1, o=0) == -1 and upd(0) == 0
    assert L.zp_accum_to_bf16(A, A, 12, None) == -1             # not a multiple of 8 elements
    assert L.zp_accum_to_bf16(0, A, 64, None) == -1
    assert L.zp_accum_to_bf16(A, A, 0, None) == 0
    assert B.workspace_bytes(B.FN_PARTIAL_BWD, sh, None, 3) > 2 * 4 * 200 * 4


@pytest.mark.parametrize("L,C", [(101, 4), (38400, 4), (7, 3), (64, 1), (5, 8)])
def test_chunk_pairs_match_oracle_enumeration(L, C):
    pairs, merges, rows = B.chunk_pairs(17, L, C)
    op, om, orows = oracle.causal_pairs(17, L, C)
    assert rows == orows and len(pairs) == len(op) and len(merges) == len(om)
    for a, b in zip(pairs, op):
        assert {f: getattr(a, f) for f, _ in B.ZpPair._fields_} == b
    for a, (tok0, ln, prow) in zip(merges, om):
        assert (a.out_tok0, a.len, a.n_parts) == (tok0, ln, len(prow)) and list(a.part_row0[:a.n_parts]) == prow


@pytest.mark.parametrize("G", [1, 2, 4])
def test_rank_share_matches_ring_schedule(G):
    C, L = 2 * G, 1000
    sched = oracle.ring_schedule(G)
    b = oracle.chunk_bounds(L, C)
    for rank in range(G):
        pairs, merges, rows = B.chunk_pairs(0, L, C, rank=rank)
        got = sorted((b.index(p.q_pos0), b.index(p.k_pos0)) for p in pairs)
        want = sorted(pr for rnd in sched[rank] for pr in rnd)
        assert got == want
        assert sorted(m.out_tok0 for m in merges) == sorted({b[rank], b[C - 1 - rank]})


def test_table2_length_mixes():
    """The synthetic batches follow the printed histograms (GitHub renormalised) and pack the budget exactly."""
    from paper_2509_21841_amd import synth
    for name, probs in synth.TABLE2.items():
        L = synth.lengths_table2(131072, 5, name)
        assert sum(L) == 131072 and min(L) >= 1
        big = synth.lengths_table2(1 << 30, 7, name)[:-1]          # the last draw is cut by the budget
        hist = np.histogram(big, bins=synth.TABLE2_EDGES)[0] / len(big)
        want = np.asarray(probs) / sum(probs)
        assert np.abs(hist - want).max() < 0.02, (name, hist, want)


def test_noalloc_forward_rejects_oversize_batches_without_device():
    """The fixed limits of the entry point that allocates nothing are checked on the host, before the device is touched."""
    L = B.lib()

    def rc(sh, cu, skip=None):
        cu = np.ascontiguousarray(cu, np.int32)
        sk = None if skip is None else np.ascontiguousarray(skip, np.uint8).ctypes.data_as(ctypes.c_void_p)
        return L.varlen_attn_fwd_noalloc(1 << 12, 1 << 12, 1 << 12, sh.Hq * sh.d, sh.Hkv * sh.d, sh.Hkv * sh.d,
                                         cu.ctypes.data_as(ctypes.c_void_p), sk, 1 << 12, sh.Hq * sh.d, 1 << 12,
                                         ctypes.byref(sh), None)

    S = B.NOALLOC_MAX_SEQS + 1
    assert rc(B.make_shape(S, S, 4, 2, 64), np.arange(S + 1)) == -5                    # too many sequences
    T = (B.NOALLOC_MAX_TILES + 1) * 128
    assert rc(B.make_shape(T, 1, 4, 2, 64), [0, T]) == -5                              # too many tiles
    assert rc(B.make_shape(T, 2, 4, 2, 64), [0, 128, T], skip=[1, 1]) == 0             # flagged sequences do not count (nothing left: no-op)
    assert rc(B.make_shape(100, 2, 4, 2, 64), [0, 60, 40]) == -1                       # the ordinary checks still run
    assert rc(B.make_shape(100, 2, 4, 2, 96), [0, 40, 100]) == -2
    assert rc(B.make_shape(0, 1, 4, 2, 64), [0, 0]) == 0
    assert len(L.zp_strerror(-5)) > 10


def _pair_tuple(p):
    return tuple(getattr(p, f) if not isinstance(p, dict) else p[f] for f in ("q_tok0", "q_len", "k_tok0", "k_len", "q_pos0", "k_pos0"))


@pytest.mark.parametrize("tok0,L,C", [(0, 1000, 4), (37, 777, 3), (5, 130, 8), (0, 5, 8), (11, 2100, 16), (3, 64, 1)])
def test_ring_round_pairs_match_the_oracle_rounds_and_the_ring_schedule(tok0, L, C):
    """zp_chunk_segments + zp_ring_round_pairs against the oracle: round t is the oracle's pairs (qc, qc - t) with the
    oracle's chunk descriptors; over all rounds they are exactly what the ranks of a ring of C/2 devices compute over
    its rounds (Sec. 3.2), each pair once."""
    opairs, _, _ = oracle.causal_pairs(tok0, L, C)
    by = dict(zip([(qc, kc) for qc in range(C) for kc in range(qc + 1)], opairs))
    rounds = B.ring_rounds(tok0, L, C)
    assert len(rounds) == C == len(oracle.ring_rounds(C))
    seen = []
    for (arr, n), ornd in zip(rounds, oracle.ring_rounds(C)):
        assert [_pair_tuple(arr[i]) for i in range(n)] == [_pair_tuple(by[pr]) for pr in ornd]
        # inside a round no query run and no key run appears twice
        qs = [arr[i].q_tok0 for i in range(n) if arr[i].q_len]
        ks = [arr[i].k_tok0 for i in range(n) if arr[i].k_len]
        assert len(set(qs)) == len(qs) and len(set(ks)) == len(ks)
        seen += ornd
    if C % 2 == 0:
        G = C // 2
        ring = [pr for rank in oracle.ring_schedule(G) for rnd in rank for pr in rnd]
        assert sorted(ring) == sorted(seen) and len(set(ring)) == len(ring)


def test_ring_round_pairs_over_scattered_runs_and_bad_input():
    # two ring sequences whose chunks sit in different device buffers (as zp_node_segments lays them out) + a whole one
    segs = [dict(seq=0, chunk=0, n_chunks=4, pos0=0, len=25, tok0=0, node=0, device=0),
            dict(seq=0, chunk=3, n_chunks=4, pos0=75, len=25, tok0=25, node=0, device=0),
            dict(seq=2, chunk=0, n_chunks=1, pos0=0, len=9, tok0=50, node=0, device=0),
            dict(seq=0, chunk=1, n_chunks=4, pos0=25, len=25, tok0=59, node=0, device=1),
            dict(seq=0, chunk=2, n_chunks=4, pos0=50, len=25, tok0=84, node=0, device=1),
            dict(seq=1, chunk=1, n_chunks=2, pos0=3, len=4, tok0=109, node=0, device=1),
            dict(seq=1, chunk=0, n_chunks=2, pos0=0, len=3, tok0=113, node=0, device=1)]
    at = {(s["seq"], s["chunk"]): s for s in segs}
    for t in range(4):
        (arr, n), rounds = B.ring_round_pairs(segs, t)
        assert rounds == 4
        want = [(0, qc, qc - t) for qc in range(t, 4)] + [(1, qc, qc - t) for qc in range(t, 2)]
        got = [_pair_tuple(arr[i]) for i in range(n)]
        assert got == [(at[(s, qc)]["tok0"], at[(s, qc)]["len"], at[(s, kc)]["tok0"], at[(s, kc)]["len"],
                        at[(s, qc)]["pos0"], at[(s, kc)]["pos0"]) for s, qc, kc in want]
    with pytest.raises(B.ZpError):
        B.ring_round_pairs(segs[:4], 0)             # a ring sequence with a chunk missing
    with pytest.raises(B.ZpError):
        B.ring_round_pairs(segs + [segs[0]], 0)     # a chunk twice
    # layout position -> drawn position
    lengths = [100, 7, 9]
    orig = B.segment_positions(lengths, segs, 116)
    first = np.concatenate([[0], np.cumsum(lengths)])
    want = np.zeros(116, np.int64)
    for s in segs:
        want[s["tok0"]:s["tok0"] + s["len"]] = first[s["seq"]] + s["pos0"] + np.arange(s["len"])
    assert np.array_equal(orig, want) and sorted(orig.tolist()) == list(range(116))
    with pytest.raises(B.ZpError):
        B.segment_positions(lengths, segs[:-1], 116)    # the runs do not tile the layout
