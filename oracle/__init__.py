"""fp64 CPU oracle for the packed variable-length attention engine -- TEST INFRASTRUCTURE.

Thin ctypes front end of ``zeppelin_oracle.c`` plus the few integer rules (chunk boundaries, causal
chunk pairs, the ring schedule) written out in plain Python.  Only ``tests/``, the smoke check and
the bench's ``cpu_baseline`` leg may import this package.  It imports nothing from the HIP package
and the HIP package imports nothing from here.

Paper passages followed: Sec. 2.1 (causal lower-triangular mask, token-wise linear modules),
Sec. 3.2 (2G equal-length chunks per ring of size G, rank i owns chunks i and 2G-1-i, G rounds of
compute against the KV in hand, local sequences by a standard varlen kernel), Sec. 3.4 (remapping
between the attention layout and the token-balanced layout, and its inverse).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "zeppelin_oracle.c")
_LIB = os.path.join(_HERE, "libzeppelin_oracle.so")
MAX_PARTS = 16


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Pair(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("q_tok0", "q_len", "k_tok0", "k_len", "q_pos0", "k_pos0", "out_row0")]


class _Merge(ctypes.Structure):
    _fields_ = [("out_tok0", ctypes.c_int32), ("len", ctypes.c_int32), ("n_parts", ctypes.c_int32),
                ("part_row0", ctypes.c_int32 * MAX_PARTS)]


_lib = None


def _L():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def num_threads() -> int:
    return int(_L().zo_num_threads())


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns (uint16) to float64."""
    b = np.ascontiguousarray(bits).view(np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def default_scale(d: int) -> float:
    return 1.0 / float(np.sqrt(d))


def varlen_attn_fwd(q, k, v, cu_seqlens, scale=None):
    """q [T,Hq,d], k/v [T,Hkv,d] float64 -> (o [T,Hq,d], lse [Hq,T])."""
    q, qp = _f64(q); k, kp = _f64(k); v, vp = _f64(v)
    cu, cup = _i32(cu_seqlens)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    scale = default_scale(d) if scale is None else float(scale)
    o = np.empty_like(q); lse = np.empty((Hq, T), np.float64)
    rc = _L().zo_varlen_attn_fwd(qp, kp, vp, ctypes.c_int64(T), Hq, Hkv, d, cup, len(cu) - 1, ctypes.c_double(scale),
                                 o.ctypes.data_as(ctypes.c_void_p), lse.ctypes.data_as(ctypes.c_void_p))
    if rc:
        raise ValueError("oracle: invalid argument")
    return o, lse


def varlen_attn_bwd(dout, q, k, v, cu_seqlens, scale=None):
    """-> (dq [T,Hq,d], dk [T,Hkv,d], dv [T,Hkv,d]); uses the oracle's own forward O and LSE."""
    dout, dop = _f64(dout); q, qp = _f64(q); k, kp = _f64(k); v, vp = _f64(v)
    cu, cup = _i32(cu_seqlens)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    scale = default_scale(d) if scale is None else float(scale)
    dq = np.empty_like(q); dk = np.empty_like(k); dv = np.empty_like(v)
    rc = _L().zo_varlen_attn_bwd(dop, qp, kp, vp, ctypes.c_int64(T), Hq, Hkv, d, cup, len(cu) - 1,
                                 ctypes.c_double(scale), dq.ctypes.data_as(ctypes.c_void_p),
                                 dk.ctypes.data_as(ctypes.c_void_p), dv.ctypes.data_as(ctypes.c_void_p))
    if rc:
        raise ValueError("oracle: invalid argument")
    return dq, dk, dv


def varlen_attn_bwd_sample(dout, q, k, v, cu_seqlens, q_samples, k_samples, scale=None):
    """q_samples: [(token, q_head)], k_samples: [(token, kv_head)] -> (dq [n_q,d], dk [n_k,d], dv [n_k,d])."""
    dout, dop = _f64(dout); q, qp = _f64(q); k, kp = _f64(k); v, vp = _f64(v)
    cu, cup = _i32(cu_seqlens)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    scale = default_scale(d) if scale is None else float(scale)
    qs = np.asarray(q_samples, np.int32).reshape(-1, 2); ks = np.asarray(k_samples, np.int32).reshape(-1, 2)
    qt, qtp = _i32(qs[:, 0]); qh, qhp = _i32(qs[:, 1]); kt, ktp = _i32(ks[:, 0]); kh, khp = _i32(ks[:, 1])
    dq = np.empty((len(qs), d)); dk = np.empty((len(ks), d)); dv = np.empty((len(ks), d))
    rc = _L().zo_varlen_attn_bwd_sample(dop, qp, kp, vp, ctypes.c_int64(T), Hq, Hkv, d, cup, len(cu) - 1,
                                        ctypes.c_double(scale), qtp, qhp, len(qs), dq.ctypes.data_as(ctypes.c_void_p),
                                        ktp, khp, len(ks), dk.ctypes.data_as(ctypes.c_void_p),
                                        dv.ctypes.data_as(ctypes.c_void_p))
    if rc:
        raise ValueError("oracle: invalid argument")
    return dq, dk, dv


def chunk_attn_partial(q, k, v, pairs, part_rows, scale=None):
    """pairs: list of dicts/tuples (q_tok0,q_len,k_tok0,k_len,q_pos0,k_pos0,out_row0)
    -> (o_part [part_rows,Hq,d], lse_part [Hq,part_rows]); rows no pair writes stay NaN."""
    q, qp = _f64(q); k, kp = _f64(k); v, vp = _f64(v)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    scale = default_scale(d) if scale is None else float(scale)
    arr = (_Pair * max(len(pairs), 1))()
    for n, p in enumerate(pairs):
        vals = [p[f] for f, _ in _Pair._fields_] if isinstance(p, dict) else list(p)
        for (f, _), val in zip(_Pair._fields_, vals):
            setattr(arr[n], f, int(val))
    o_part = np.full((part_rows, Hq, d), np.nan); lse_part = np.full((Hq, part_rows), np.nan)
    rc = _L().zo_chunk_attn_partial(qp, kp, vp, ctypes.c_int64(T), Hq, Hkv, d, arr, len(pairs), ctypes.c_double(scale),
                                    o_part.ctypes.data_as(ctypes.c_void_p), lse_part.ctypes.data_as(ctypes.c_void_p),
                                    ctypes.c_int64(part_rows))
    if rc:
        raise ValueError("oracle: invalid argument")
    return o_part, lse_part


def chunk_attn_partial_bwd(dout, q, k, v, pairs, lse, D, dq, dk, dv, scale=None):
    """Adds the pairs' backward contributions to dq [T,Hq,d], dk, dv [T,Hkv,d] (float64, modified in place and
    returned). lse, D: [Hq,T] statistics of the whole rows (D = sum_c dO*O)."""
    dout, dop = _f64(dout); q, qp = _f64(q); k, kp = _f64(k); v, vp = _f64(v)
    lse, lp = _f64(lse); D, Dp = _f64(D)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    scale = default_scale(d) if scale is None else float(scale)
    arr = (_Pair * max(len(pairs), 1))()
    for n, p in enumerate(pairs):
        vals = [p[f] if isinstance(p, dict) else getattr(p, f) for f, _ in _Pair._fields_]
        for (f, _), val in zip(_Pair._fields_, vals):
            setattr(arr[n], f, int(val))
    for a in (dq, dk, dv):
        assert a.dtype == np.float64 and a.flags.c_contiguous
    rc = _L().zo_chunk_attn_partial_bwd(dop, qp, kp, vp, ctypes.c_int64(T), Hq, Hkv, d, arr, len(pairs),
                                        ctypes.c_double(scale), lp, Dp, dq.ctypes.data_as(ctypes.c_void_p),
                                        dk.ctypes.data_as(ctypes.c_void_p), dv.ctypes.data_as(ctypes.c_void_p))
    if rc:
        raise ValueError("oracle: invalid argument")
    return dq, dk, dv


def f32_to_bf16_bits(x):
    """bfloat16 bit patterns (uint16) of float32 values, round to nearest, ties to even; NaN stays NaN (quiet)."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    keep = u >> 16
    rem = u & 0xFFFF
    up = (rem > 0x8000) | ((rem == 0x8000) & ((keep & 1) == 1))
    out = (keep + up).astype(np.uint32)
    nan = np.isnan(np.ascontiguousarray(x, np.float32))
    out = np.where(nan, (u >> 16) | 0x40, out)
    return out.astype(np.uint16)


def ring_rounds(C: int):
    """Causal chunk pairs grouped into rounds in which every Q chunk and every KV chunk appears at most once:
    round t holds the pairs (qc, qc - t)."""
    return [[(qc, qc - t) for qc in range(t, C)] for t in range(C)]


def lse_merge(o_part, lse_part, merges, T, o=None, lse=None):
    """merges: list of (out_tok0, len, [part_row0...]). Rows outside every merge keep o/lse as passed
    (NaN when not passed). -> (o [T,Hq,d], lse [Hq,T])."""
    o_part, opp = _f64(o_part); lse_part, lpp = _f64(lse_part)
    part_rows, Hq, d = o_part.shape
    arr = (_Merge * max(len(merges), 1))()
    for n, (tok0, ln, rows) in enumerate(merges):
        arr[n].out_tok0, arr[n].len, arr[n].n_parts = int(tok0), int(ln), len(rows)
        if len(rows) > MAX_PARTS:
            raise ValueError("too many parts")
        for p, r in enumerate(rows):
            arr[n].part_row0[p] = int(r)
    o = np.full((T, Hq, d), np.nan) if o is None else np.ascontiguousarray(o, np.float64)
    lse = np.full((Hq, T), np.nan) if lse is None else np.ascontiguousarray(lse, np.float64)
    rc = _L().zo_lse_merge(opp, lpp, ctypes.c_int64(part_rows), arr, len(merges), ctypes.c_int64(T), Hq, d,
                           o.ctypes.data_as(ctypes.c_void_p), lse.ctypes.data_as(ctypes.c_void_p))
    if rc:
        raise ValueError("oracle: invalid argument")
    return o, lse


def remap_tokens(src: np.ndarray, idx, mode: int = 0) -> np.ndarray:
    """Row move on raw bytes. src: any array whose first axis is the token axis."""
    src = np.ascontiguousarray(src)
    n = src.shape[0]
    row_bytes = src.nbytes // max(n, 1)
    idx, ip = _i32(idx)
    dst = np.zeros_like(src)
    rc = _L().zo_remap_tokens(src.ctypes.data_as(ctypes.c_void_p), dst.ctypes.data_as(ctypes.c_void_p),
                              ctypes.c_int64(row_bytes), ip, ctypes.c_int64(n), int(mode))
    if rc:
        raise ValueError("oracle: invalid argument")
    return dst


# ---- integer rules of Sec. 3.2, written out ------------------------------------------------------

def chunk_bounds(L: int, C: int):
    """Boundaries of C (near-)equal-length chunks of a length-L sequence: chunk c = [b[c], b[c+1])."""
    return [(c * L) // C for c in range(C + 1)]


def causal_pairs(tok0: int, L: int, C: int):
    """All (Q chunk, KV chunk) pairs with kc <= qc of one sequence starting at packed token tok0.
    Returns (pairs, merges, part_rows): pair rows are laid out pair after pair; one merge per Q chunk."""
    b = chunk_bounds(L, C)
    pairs, merges, row = [], [], 0
    for qc in range(C):
        qlen = b[qc + 1] - b[qc]
        rows = []
        for kc in range(qc + 1):
            pairs.append(dict(q_tok0=tok0 + b[qc], q_len=qlen, k_tok0=tok0 + b[kc], k_len=b[kc + 1] - b[kc],
                              q_pos0=b[qc], k_pos0=b[kc], out_row0=row))
            rows.append(row)
            row += qlen
        merges.append((tok0 + b[qc], qlen, rows))
    return pairs, merges, row


def ring_schedule(G: int):
    """Ring of size G over 2G chunks: rank i owns chunks {i, 2G-1-i}; in round t it holds the KV chunks
    of rank (i - t) mod G.  Returns sched[rank][round] = list of (qc, kc) chunk pairs that have any
    causally visible key (kc <= qc)."""
    own = lambda r: (r, 2 * G - 1 - r)
    sched = []
    for i in range(G):
        rounds = []
        for t in range(G):
            src = (i - t) % G
            rounds.append([(qc, kc) for qc in own(i) for kc in own(src) if kc <= qc])
        sched.append(rounds)
    return sched
