"""AddressSanitizer + UndefinedBehaviorSanitizer over the CPU side: the fp64 oracle and the library's host planners are
compiled with -fsanitize=address,undefined into one driver program (tests/sanitize_driver.cpp), run on seeded requests,
and must (a) report nothing and (b) return what the ordinary builds return. The staging pool's slot state machine runs
under the same sanitizers with several threads (tests/pool_threads.cpp). CPU only."""
import os
import struct
import subprocess

import numpy as np
import pytest

import oracle
from oracle import remap_planner as RP
from paper_2509_21841_amd import binding as B

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    out = tmp_path_factory.mktemp("san")
    obj = str(out / "oracle.o")
    subprocess.check_call(["gcc", *SAN, "-c", os.path.join(ROOT, "oracle", "zeppelin_oracle.c"), "-o", obj])
    exe = str(out / "sanitize_driver")
    csrc = os.path.join(ROOT, "paper_2509_21841_amd", "csrc")
    subprocess.check_call(["g++", "-std=c++17", *SAN, os.path.join(HERE, "sanitize_driver.cpp"), obj,
                           os.path.join(csrc, "zp_partition.cpp"), os.path.join(csrc, "zp_remap_plan.cpp"), "-lm", "-o", exe])
    return exe, out


def run(exe, mode, request: bytes, out_dir):
    fin, fout = str(out_dir / f"{mode}.in"), str(out_dir / f"{mode}.out")
    open(fin, "wb").write(request)
    r = subprocess.run([exe, mode, fin, fout], capture_output=True, text=True, env=ENV, timeout=600)
    assert r.returncode == 0 and not r.stderr.strip(), f"sanitizer report or failure (exit {r.returncode}):\n{r.stderr[-3000:]}"
    data = open(fout, "rb").read()
    pos = 0

    def nxt(dtype):
        nonlocal pos
        n = struct.unpack_from("<q", data, pos)[0]
        pos += 8
        a = np.frombuffer(data, dtype=dtype, count=n, offset=pos)
        pos += n * np.dtype(dtype).itemsize
        return a
    return nxt


def i64(*xs):
    return struct.pack("<%dq" % len(xs), *xs)


def test_oracle_under_sanitizers(driver):
    exe, out = driver
    rng = np.random.default_rng(5)
    lengths = [37, 0, 1, 130, 64]
    T, Hq, Hkv, d, scale = sum(lengths), 4, 2, 16, 0.21
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    q, k, v, do = (rng.standard_normal((T, h, d)) for h in (Hq, Hkv, Hkv, Hq))
    t0 = int(cu[3])
    pairs, merges, rows = oracle.causal_pairs(t0, 130, 3)
    idx = rng.permutation(T).astype(np.int32)
    pa = b"".join(struct.pack("<7i", *(p[f] for f in ("q_tok0", "q_len", "k_tok0", "k_len", "q_pos0", "k_pos0", "out_row0"))) for p in pairs)
    ma = b"".join(struct.pack("<19i", tok0, ln, len(r), *(list(r) + [0] * (16 - len(r)))) for tok0, ln, r in merges)
    req = i64(T, Hq, Hkv, d, len(lengths), len(pairs), rows, len(merges)) + struct.pack("<d", scale) + cu.tobytes() + \
        q.tobytes() + k.tobytes() + v.tobytes() + do.tobytes() + pa + ma + idx.tobytes()
    nxt = run(exe, "oracle", req, out)
    close = lambda a, b: np.testing.assert_allclose(np.asarray(a).ravel(), np.asarray(b).ravel(), rtol=1e-12, atol=1e-13)
    ro, rl = oracle.varlen_attn_fwd(q, k, v, cu, scale=scale)
    close(nxt("<f8"), ro); close(nxt("<f8"), rl)
    for want in oracle.varlen_attn_bwd(do, q, k, v, cu, scale=scale):
        close(nxt("<f8"), want)
    rop, rlp = oracle.chunk_attn_partial(q, k, v, pairs, rows, scale=scale)
    got_op, got_lp = nxt("<f8"), nxt("<f8")
    close(got_op, rop)
    assert np.array_equal(np.isneginf(got_lp), np.isneginf(rlp.ravel()))
    close(got_lp[np.isfinite(got_lp)], rlp.ravel()[np.isfinite(rlp.ravel())])
    mo, ml = oracle.lse_merge(rop, rlp, merges, T, np.zeros((T, Hq, d)), np.zeros((Hq, T)))
    close(nxt("<f8"), mo); close(nxt("<f8"), ml)
    sdq, sdk, sdv = oracle.varlen_attn_bwd_sample(do, q, k, v, cu, [(0, 0), (T // 2, Hq - 1), (T - 1, 0)],
                                                   [(0, 0), (T // 2, Hkv - 1), (T - 1, 0)], scale=scale)
    close(nxt("<f8"), sdq); close(nxt("<f8"), sdk); close(nxt("<f8"), sdv)
    D = np.einsum("thc,thc->ht", do, ro)
    ref = [np.zeros(x.shape) for x in (q, k, v)]
    oracle.chunk_attn_partial_bwd(do, q, k, v, pairs, rl, D, *ref, scale=scale)
    for want in ref:
        close(nxt("<f8"), want)
    assert np.array_equal(nxt("<f8"), oracle.remap_tokens(q, idx, 0).ravel())
    assert np.array_equal(nxt("<f8"), oracle.remap_tokens(q, idx, 1).ravel())


def test_host_planners_under_sanitizers(driver):
    exe, out = driver
    rng = np.random.default_rng(9)
    cases = [([10, 4, 3, 2, 1], 2, 1, 10), ([40, 34, 7, 5], 2, 4, 16), ([28, 14, 3, 2, 1], 2, 3, 10), ([32, 16, 16], 4, 1, 16),
             ([10, 10, 0, 0], 2, 1, 8), ([0, 0, 0], 2, 1, 4), ([64000, 10, 10], 4, 2, 8000), ([5], 1, 1, 1)]
    for _ in range(12):
        P, N = int(rng.choice([1, 2, 4, 8])), int(rng.choice([1, 2, 4]))
        S = int(rng.integers(1, 40))
        lengths = np.clip(np.rint(np.exp(rng.normal(6.0, 1.4, S))), 0, 100000).astype(int).tolist()
        L = max(1, int(np.ceil(sum(lengths) * float(rng.choice([1.0, 1.2, 3.0])) / (P * N))))
        cases.append((lengths, P, N, L))
    req = i64(len(cases))
    for lengths, P, N, L in cases:
        req += i64(P, N, L, len(lengths), 1, 5) + np.asarray(lengths, np.int32).tobytes()
    nxt = run(exe, "planners", req, out)
    for lengths, P, N, L in cases:
        pl, s1, s0 = B.partition(lengths, P, N, L)
        want = [p[f] for p in pl for f in ("seq", "zone", "ring", "rank", "node", "device", "tokens")] + [s1] + s0
        assert nxt("<i4").tolist() == want
        segs, A = B.node_segments(lengths, pl, P, N)
        assert nxt("<i4").tolist() == [s[f] for s in segs for f in ("seq", "chunk", "n_chunks", "pos0", "len", "tok0", "node", "device")]
        assert np.array_equal(nxt("<i4"), A)
        T = sum(lengths)
        assert np.array_equal(nxt("<i8"), B.segment_positions(lengths, segs, T))
        flat = []
        if any(s["n_chunks"] > 1 for s in segs):
            _, rounds = B.ring_round_pairs(segs, 0)
            for t in range(rounds):
                (arr, n), _ = B.ring_round_pairs(segs, t)
                flat.append(n)
                for i in range(n):
                    flat += [arr[i].q_tok0, arr[i].q_len, arr[i].k_tok0, arr[i].k_len, arr[i].q_pos0, arr[i].k_pos0]
        assert nxt("<i4").tolist() == flat
        M, obj = B.remap_plan(A, P, 1, 5)
        assert np.array_equal(nxt("<i4").reshape(P * N, P * N), M)
        assert np.array_equal(nxt("<i4"), B.remap_indices(A, M))
        assert int(nxt("<i8")[0]) == obj == RP.objective(M, P, 1, 5)
        if lengths and lengths[0] > 0:
            b = oracle.chunk_bounds(lengths[0], 5)
            assert nxt("<i4").tolist() == [x for c in range(5) for x in (b[c], b[c + 1] - b[c], 3 + b[c])]


def test_staging_pool_threads_under_sanitizers(tmp_path):
    exe = str(tmp_path / "pool_threads")
    subprocess.check_call(["g++", "-std=c++17", "-pthread", *SAN, os.path.join(HERE, "pool_threads.cpp"), "-o", exe])
    # the pool keeps its buffers until the process ends (by design), so the leak check is off for this program
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600,
                       env=dict(ENV, ASAN_OPTIONS="detect_leaks=0"))
    assert r.returncode == 0 and "errors 0" in r.stdout and not r.stderr.strip(), r.stdout + r.stderr[-3000:]
