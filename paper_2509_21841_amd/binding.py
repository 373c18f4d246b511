"""ctypes binding of libzeppelin_attn.so: argument marshalling only.

Same names as the C ABI (include/zeppelin_attn.h). Tensors are torch CUDA(HIP) tensors used purely as device
buffers; every step of the path runs in the library's HIP kernels. There is no CPU fallback: a missing
library or a failing call raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libzeppelin_attn.so")
MAX_PARTS = 16
FN_FWD, FN_BWD, FN_PARTIAL, FN_MERGE, FN_PARTIAL_BWD = 0, 1, 2, 3, 4


class ZpShape(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("S", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("d", ctypes.c_int32), ("scale", ctypes.c_float)]


class ZpPair(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("q_tok0", "q_len", "k_tok0", "k_len", "q_pos0", "k_pos0", "out_row0")]


class ZpMerge(ctypes.Structure):
    _fields_ = [("out_tok0", ctypes.c_int32), ("len", ctypes.c_int32), ("n_parts", ctypes.c_int32),
                ("part_row0", ctypes.c_int32 * MAX_PARTS)]


class ZpPlacement(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("seq", "zone", "ring", "rank", "node", "device", "tokens")]


class ZpSegment(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("seq", "chunk", "n_chunks", "pos0", "len", "tok0", "node", "device")]


class ZpError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"zeppelin_attn error {code}: {text}")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """Loads the built library; builds it first only if no built library exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
    L.zp_strerror.restype = ctypes.c_char_p
    L.zp_strerror.argtypes = [ctypes.c_int]
    L.zp_workspace_bytes.restype = sz
    L.zp_workspace_bytes.argtypes = [ctypes.c_int, ctypes.POINTER(ZpShape), vp, i64]
    L.varlen_attn_fwd.restype = ctypes.c_int
    L.varlen_attn_fwd.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp, vp, i64, vp, ctypes.POINTER(ZpShape), vp, sz, vp]
    L.varlen_attn_fwd_noalloc.restype = ctypes.c_int
    L.varlen_attn_fwd_noalloc.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp, vp, i64, vp, ctypes.POINTER(ZpShape), vp]
    L.varlen_attn_bwd.restype = ctypes.c_int
    L.varlen_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, vp, vp, vp, vp, vp, i64, i64,
                                  ctypes.POINTER(ZpShape), vp, sz, vp]
    L.chunk_attn_partial.restype = ctypes.c_int
    L.chunk_attn_partial.argtypes = [vp, vp, vp, i64, i64, i64, ctypes.POINTER(ZpPair), i32, vp, vp, i64,
                                     ctypes.POINTER(ZpShape), vp, sz, vp]
    L.chunk_attn_update.restype = ctypes.c_int
    L.chunk_attn_update.argtypes = [vp, vp, vp, i64, i64, i64, ctypes.POINTER(ZpPair), i32, vp, vp,
                                    ctypes.POINTER(ZpShape), vp, sz, vp]
    L.chunk_attn_partial_bwd.restype = ctypes.c_int
    L.chunk_attn_partial_bwd.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, ctypes.POINTER(ZpPair), i32,
                                         vp, vp, vp, ctypes.POINTER(ZpShape), vp, sz, vp]
    L.zp_accum_to_bf16.restype = ctypes.c_int
    L.zp_accum_to_bf16.argtypes = [vp, vp, i64, vp]
    L.zp_remap_plan.restype = ctypes.c_int
    L.zp_remap_plan.argtypes = [vp, i32, i32, i32, i32, vp, ctypes.POINTER(i64)]
    L.zp_remap_indices.restype = ctypes.c_int
    L.zp_remap_indices.argtypes = [vp, vp, i32, vp, i64]
    L.lse_merge.restype = ctypes.c_int
    L.lse_merge.argtypes = [vp, vp, i64, ctypes.POINTER(ZpMerge), i32, vp, i64, vp, ctypes.POINTER(ZpShape), vp, sz, vp]
    L.remap_tokens.restype = ctypes.c_int
    L.remap_tokens.argtypes = [vp, vp, i64, vp, i64, i32, vp]
    L.zp_partition.restype = ctypes.c_int
    L.zp_partition.argtypes = [vp, i32, i32, i32, i32, ctypes.POINTER(ZpPlacement), i32, ctypes.POINTER(i32),
                               ctypes.POINTER(i32), vp]
    L.zp_node_segments.restype = ctypes.c_int
    L.zp_node_segments.argtypes = [vp, i32, ctypes.POINTER(ZpPlacement), i32, i32, i32, ctypes.POINTER(ZpSegment), i32,
                                   ctypes.POINTER(i32), vp]
    L.zp_chunk_segments.restype = ctypes.c_int
    L.zp_chunk_segments.argtypes = [i32, i32, i32, i32, ctypes.POINTER(ZpSegment), i32]
    L.zp_ring_round_pairs.restype = ctypes.c_int
    L.zp_ring_round_pairs.argtypes = [ctypes.POINTER(ZpSegment), i32, i32, i32, ctypes.POINTER(ZpPair), i32,
                                      ctypes.POINTER(i32), ctypes.POINTER(i32)]
    L.zp_segment_positions.restype = ctypes.c_int
    L.zp_segment_positions.argtypes = [vp, i32, ctypes.POINTER(ZpSegment), i32, vp, i64]
    L.zp_profile_enable.restype = ctypes.c_int
    L.zp_profile_enable.argtypes = [ctypes.c_int]
    L.zp_profile_count.restype = ctypes.c_int
    L.zp_profile_get.restype = ctypes.c_int
    L.zp_profile_get.argtypes = [ctypes.c_int, ctypes.c_char_p, ctypes.c_int, ctypes.POINTER(ctypes.c_float)]
    L.zp_chunk_pairs.restype = ctypes.c_int
    L.zp_chunk_pairs.argtypes = [i32, i32, i32, i32, i32, ctypes.POINTER(ZpPair), i32, ctypes.POINTER(ZpMerge), i32,
                                 ctypes.POINTER(i32), ctypes.POINTER(i64)]
    _lib = L
    return L


def _check(rc: int):
    if rc != 0:
        raise ZpError(rc, lib().zp_strerror(rc).decode())


def _stream_ptr(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _cu_host(cu_seqlens) -> np.ndarray:
    if isinstance(cu_seqlens, torch.Tensor):
        cu_seqlens = cu_seqlens.cpu().numpy()
    return np.ascontiguousarray(cu_seqlens, dtype=np.int32)


def _tok_stride(t: torch.Tensor) -> int:
    assert t.dim() == 3 and t.stride(2) == 1 and t.stride(1) == t.shape[2], "need [T,H,d] with contiguous heads"
    return t.stride(0) if t.shape[0] > 1 else t.shape[1] * t.shape[2]


_ws_cache: dict = {}


def workspace(nbytes: int, device, tag: str = "default", stream=None) -> torch.Tensor:
    """A cached device scratch tensor of at least nbytes (256-byte aligned by the torch allocator), one per device,
    entry point and stream: calls on one stream are ordered and may share it, calls on different streams may not."""
    key = (str(device), tag, _stream_ptr(stream).value or 0)
    t = _ws_cache.get(key)
    if t is None or t.numel() < nbytes:
        t = torch.empty(max(int(nbytes), 4096), dtype=torch.uint8, device=device)
        _ws_cache[key] = t
    return t


def workspace_bytes(which: int, shape: ZpShape, cu_host=None, n_desc: int = 0) -> int:
    cup = cu_host.ctypes.data_as(ctypes.c_void_p) if cu_host is not None else None
    return int(lib().zp_workspace_bytes(which, ctypes.byref(shape), cup, n_desc))


def make_shape(T, S, Hq, Hkv, d, scale=0.0) -> ZpShape:
    return ZpShape(int(T), int(S), int(Hq), int(Hkv), int(d), float(scale or 0.0))


def varlen_attn_fwd(q, k, v, cu_seqlens, o=None, lse=None, scale=0.0, ws=None, stream=None, seq_skip=None):
    """q [T,Hq,d], k/v [T,Hkv,d] bf16 device tensors -> (o [T,Hq,d] bf16, lse [Hq,T] f32).
    seq_skip: optional per-sequence flags; flagged sequences are left for chunk_attn_partial + lse_merge."""
    cu = _cu_host(cu_seqlens)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    sh = make_shape(T, len(cu) - 1, Hq, Hkv, d, scale)
    if o is None:
        o = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((Hq, T), dtype=torch.float32, device=q.device)
    need = workspace_bytes(FN_FWD, sh, cu)
    if ws is None:
        ws = workspace(need, q.device, "fwd", stream)
    skip = None if seq_skip is None else np.ascontiguousarray(seq_skip, dtype=np.uint8)
    assert skip is None or len(skip) == len(cu) - 1
    skp = None if skip is None else skip.ctypes.data_as(ctypes.c_void_p)
    _check(lib().varlen_attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), _tok_stride(q), _tok_stride(k), _tok_stride(v),
                                 cu.ctypes.data_as(ctypes.c_void_p), skp, o.data_ptr(), _tok_stride(o), lse.data_ptr(),
                                 ctypes.byref(sh), ws.data_ptr(), ws.numel(), _stream_ptr(stream)))
    return o, lse


NOALLOC_MAX_SEQS, NOALLOC_MAX_TILES = 768, 8192


def varlen_attn_fwd_noalloc(q, k, v, cu_seqlens, o, lse, scale=0.0, stream=None, seq_skip=None):
    """varlen_attn_fwd through the entry point that allocates nothing: the caller brings o and lse, there is no
    workspace (the tile table is a fixed device array inside the library)."""
    cu = _cu_host(cu_seqlens)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    sh = make_shape(T, len(cu) - 1, Hq, Hkv, d, scale)
    skip = None if seq_skip is None else np.ascontiguousarray(seq_skip, dtype=np.uint8)
    assert skip is None or len(skip) == len(cu) - 1
    skp = None if skip is None else skip.ctypes.data_as(ctypes.c_void_p)
    _check(lib().varlen_attn_fwd_noalloc(q.data_ptr(), k.data_ptr(), v.data_ptr(), _tok_stride(q), _tok_stride(k),
                                         _tok_stride(v), cu.ctypes.data_as(ctypes.c_void_p), skp, o.data_ptr(),
                                         _tok_stride(o), lse.data_ptr(), ctypes.byref(sh), _stream_ptr(stream)))
    return o, lse


def varlen_attn_bwd(dout, q, k, v, o, lse, cu_seqlens, dq=None, dk=None, dv=None, scale=0.0, ws=None, stream=None,
                    seq_skip=None):
    """-> (dq [T,Hq,d], dk [T,Hkv,d], dv [T,Hkv,d]) bf16. Rows of sequences flagged in seq_skip are not written."""
    cu = _cu_host(cu_seqlens)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    sh = make_shape(T, len(cu) - 1, Hq, Hkv, d, scale)
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    need = workspace_bytes(FN_BWD, sh, cu)
    if ws is None:
        ws = workspace(need, q.device, "bwd", stream)
    assert _tok_stride(dk) == _tok_stride(dv)
    skip = None if seq_skip is None else np.ascontiguousarray(seq_skip, dtype=np.uint8)
    assert skip is None or len(skip) == len(cu) - 1
    _check(lib().varlen_attn_bwd(dout.data_ptr(), q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                                 _tok_stride(dout), _tok_stride(q), _tok_stride(k), _tok_stride(v), _tok_stride(o),
                                 cu.ctypes.data_as(ctypes.c_void_p),
                                 None if skip is None else skip.ctypes.data_as(ctypes.c_void_p),
                                 dq.data_ptr(), dk.data_ptr(), dv.data_ptr(),
                                 _tok_stride(dq), _tok_stride(dk), ctypes.byref(sh), ws.data_ptr(), ws.numel(),
                                 _stream_ptr(stream)))
    return dq, dk, dv


def _pairs_array(pairs):
    if isinstance(pairs, tuple) and len(pairs) == 2 and isinstance(pairs[0], ctypes.Array):
        return pairs                      # (array, count) prepared earlier
    if isinstance(pairs, ctypes.Array):
        return pairs, len(pairs)
    arr = (ZpPair * max(len(pairs), 1))()
    for n, p in enumerate(pairs):
        if isinstance(p, ZpPair):
            vals = [getattr(p, f) for f, _ in ZpPair._fields_]
        else:
            vals = [p[f] for f, _ in ZpPair._fields_] if isinstance(p, dict) else list(p)
        for (f, _), val in zip(ZpPair._fields_, vals):
            setattr(arr[n], f, int(val))
    return arr, len(pairs)


def _merges_array(merges):
    if isinstance(merges, ctypes.Array):
        return merges, len(merges)
    arr = (ZpMerge * max(len(merges), 1))()
    for n, (tok0, ln, rows) in enumerate(merges):
        arr[n].out_tok0, arr[n].len, arr[n].n_parts = int(tok0), int(ln), len(rows)
        for p, r in enumerate(rows[:MAX_PARTS]):
            arr[n].part_row0[p] = int(r)
        if len(rows) > MAX_PARTS:
            arr[n].n_parts = len(rows)  # rejected by the library
    return arr, len(merges)


def chunk_attn_partial(q, k, v, pairs, part_rows, o_part=None, lse_part=None, scale=0.0, ws=None, stream=None):
    """-> (o_part [part_rows,Hq,d] f32, lse_part [Hq,part_rows] f32)."""
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    sh = make_shape(T, 0, Hq, Hkv, d, scale)
    arr, n = _pairs_array(pairs)
    if o_part is None:
        o_part = torch.empty((part_rows, Hq, d), dtype=torch.float32, device=q.device)
    if lse_part is None:
        lse_part = torch.empty((Hq, part_rows), dtype=torch.float32, device=q.device)
    need = workspace_bytes(FN_PARTIAL, sh, None, n)
    if ws is None:
        ws = workspace(need, q.device, "partial", stream)
    _check(lib().chunk_attn_partial(q.data_ptr(), k.data_ptr(), v.data_ptr(), _tok_stride(q), _tok_stride(k), _tok_stride(v),
                                    arr, n, o_part.data_ptr(), lse_part.data_ptr(), int(part_rows), ctypes.byref(sh),
                                    ws.data_ptr(), ws.numel(), _stream_ptr(stream)))
    return o_part, lse_part


def chunk_attn_update(q, k, v, pairs, o_run, lse_run, scale=0.0, ws=None, stream=None):
    """One ring round merged in place into the running fp32 (o_run [T,Hq,d], lse_run [Hq,T])."""
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    sh = make_shape(T, 0, Hq, Hkv, d, scale)
    arr, n = _pairs_array(pairs)
    assert o_run.dtype == torch.float32 and o_run.is_contiguous() and lse_run.dtype == torch.float32 and lse_run.is_contiguous()
    need = workspace_bytes(FN_PARTIAL, sh, None, n)
    if ws is None:
        ws = workspace(need, q.device, "partial", stream)
    _check(lib().chunk_attn_update(q.data_ptr(), k.data_ptr(), v.data_ptr(), _tok_stride(q), _tok_stride(k), _tok_stride(v),
                                   arr, n, o_run.data_ptr(), lse_run.data_ptr(), ctypes.byref(sh), ws.data_ptr(),
                                   ws.numel(), _stream_ptr(stream)))
    return o_run, lse_run


def chunk_attn_partial_bwd(dout, q, k, v, o, lse, pairs, dq_acc, dk_acc, dv_acc, scale=0.0, ws=None, stream=None):
    """One ring round of the chunked backward: ADDS the pairs' contributions to the float accumulators
    dq_acc [T,Hq,d], dk_acc / dv_acc [T,Hkv,d] (contiguous). Q ranges and KV ranges of the pairs must be disjoint."""
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    sh = make_shape(T, 0, Hq, Hkv, d, scale)
    arr, n = _pairs_array(pairs)
    for a in (dq_acc, dk_acc, dv_acc):
        assert a.dtype == torch.float32 and a.is_contiguous()
    need = workspace_bytes(FN_PARTIAL_BWD, sh, None, n)
    if ws is None:
        ws = workspace(need, q.device, "partial_bwd", stream)
    _check(lib().chunk_attn_partial_bwd(dout.data_ptr(), q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
                                        lse.data_ptr(), _tok_stride(dout), _tok_stride(q), _tok_stride(k), _tok_stride(v),
                                        _tok_stride(o), arr, n, dq_acc.data_ptr(), dk_acc.data_ptr(), dv_acc.data_ptr(),
                                        ctypes.byref(sh), ws.data_ptr(), ws.numel(), _stream_ptr(stream)))
    return dq_acc, dk_acc, dv_acc


def accum_to_bf16(src, dst=None, stream=None):
    """Rounds a contiguous float32 accumulator tensor to bfloat16 on the device."""
    assert src.dtype == torch.float32 and src.is_contiguous()
    if dst is None:
        dst = torch.empty(src.shape, dtype=torch.bfloat16, device=src.device)
    _check(lib().zp_accum_to_bf16(src.data_ptr(), dst.data_ptr(), src.numel(), _stream_ptr(stream)))
    return dst


MFMA_PROBE_FLOP_PER_ITER = 256.0 * 4 * 32 * 32768.0


BENCH_LIB_PATH = os.path.join(_HERE, "libzeppelin_bench.so")
_bench_lib = None


def bench_lib() -> ctypes.CDLL:
    """The bench-side library (measurement aids only; include/zeppelin_attn_bench.h)."""
    global _bench_lib
    if _bench_lib is None:
        if not os.path.exists(BENCH_LIB_PATH):
            from . import build as _build
            _build.build()
        _bench_lib = ctypes.CDLL(BENCH_LIB_PATH)
        _bench_lib.zp_mfma_probe.restype = ctypes.c_int
        _bench_lib.zp_mfma_probe.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
    return _bench_lib


def mfma_probe(iters: int, random_operands: bool, out=None, stream=None):
    """Enqueues the register-only MFMA loop; the caller times it (MFMA_PROBE_FLOP_PER_ITER * iters flop)."""
    if out is None:
        out = torch.empty(256 * 256, dtype=torch.float32, device="cuda")
    rc = bench_lib().zp_mfma_probe(out.data_ptr(), int(iters), int(bool(random_operands)), _stream_ptr(stream))
    if rc != 0:
        raise RuntimeError(f"zp_mfma_probe failed: {rc}")
    return out


def _segments_array(segs):
    if isinstance(segs, tuple) and len(segs) == 2 and isinstance(segs[0], ctypes.Array):
        return segs
    arr = (ZpSegment * max(len(segs), 1))()
    for i, sg in enumerate(segs):
        for f, _ in ZpSegment._fields_:
            setattr(arr[i], f, int(sg[f]))
    return arr, len(segs)


def chunk_segments(tok0: int, L: int, C: int, seq: int = 0):
    """Host helper: the runs of one contiguous sequence cut into C equal-length chunks -> (ctypes array, C)."""
    out = (ZpSegment * C)()
    n = lib().zp_chunk_segments(int(seq), int(tok0), int(L), int(C), out, C)
    if n < 0:
        _check(n)
    return out, n


def ring_round_pairs(segs, t: int, include_whole: bool = False):
    """Host helper: the chunk pairs (qc, qc - t) of every ring sequence among the runs -> ((pairs array, n), rounds).
    include_whole: whole sequences count as rings of one chunk."""
    arr, n_segs = _segments_array(segs)
    n = ctypes.c_int32(0)
    rounds = ctypes.c_int32(0)
    rc = lib().zp_ring_round_pairs(arr, n_segs, int(t), int(include_whole), None, 0, ctypes.byref(n), ctypes.byref(rounds))
    if rc not in (0, -3):
        _check(rc)
    pairs = (ZpPair * max(n.value, 1))()
    _check(lib().zp_ring_round_pairs(arr, n_segs, int(t), int(include_whole), pairs, n.value, ctypes.byref(n),
                                     ctypes.byref(rounds)))
    return (pairs, n.value), rounds.value


def ring_rounds(tok0: int, L: int, C: int):
    """All C rounds of one contiguous sequence cut into C chunks: [(pairs array, n)] with round t = pairs (qc, qc - t)."""
    segs = chunk_segments(tok0, L, C)
    return [ring_round_pairs(segs, t, include_whole=True)[0] for t in range(C)]


def segment_positions(lengths, segs, n_tok: int):
    """Host helper: attention-layout token -> token of the batch as drawn (int64 array of n_tok entries)."""
    lens = np.ascontiguousarray(lengths, dtype=np.int32)
    arr, n_segs = _segments_array(segs)
    orig = np.zeros(int(n_tok), np.int64)
    _check(lib().zp_segment_positions(lens.ctypes.data_as(ctypes.c_void_p), len(lens), arr, n_segs,
                                      orig.ctypes.data_as(ctypes.c_void_p), int(n_tok)))
    return orig


def lse_merge(o_part, lse_part, merges, o, lse, ws=None, stream=None):
    """Combines partial rows into o [T,Hq,d] bf16 and lse [Hq,T] f32 (only the tokens the merges cover)."""
    part_rows, Hq, d = o_part.shape
    T = o.shape[0]
    sh = make_shape(T, 0, Hq, Hq, d, 0.0)
    arr, n = _merges_array(merges)
    need = workspace_bytes(FN_MERGE, sh, None, n)
    if ws is None:
        ws = workspace(need, o.device, "merge", stream)
    _check(lib().lse_merge(o_part.data_ptr(), lse_part.data_ptr(), int(part_rows), arr, n, o.data_ptr(), _tok_stride(o),
                           lse.data_ptr(), ctypes.byref(sh), ws.data_ptr(), ws.numel(), _stream_ptr(stream)))
    return o, lse


def remap_tokens(src, idx, mode: int = 0, dst=None, stream=None):
    """Row gather (mode 0: dst[i] = src[idx[i]]) or scatter (mode 1: dst[idx[i]] = src[i]); idx int32 on device."""
    assert src.is_contiguous()
    n = src.shape[0]
    row_bytes = int(np.prod(src.shape[1:])) * src.element_size()
    if dst is None:
        dst = torch.empty_like(src)
    _check(lib().remap_tokens(src.data_ptr(), dst.data_ptr(), int(row_bytes), idx.data_ptr(), int(n), int(mode),
                              _stream_ptr(stream)))
    return dst


def chunk_pairs(tok0: int, L: int, C: int, rank: int = -1, row0: int = 0):
    """Host helper: (pairs, merges, rows_used) as ctypes arrays for one sequence cut into C chunks."""
    max_pairs = C * (C + 1) // 2
    pairs = (ZpPair * max_pairs)()
    merges = (ZpMerge * C)()
    nm = ctypes.c_int32(0)
    rows = ctypes.c_int64(0)
    n = lib().zp_chunk_pairs(int(tok0), int(L), int(C), int(rank), int(row0), pairs, max_pairs, merges, C,
                             ctypes.byref(nm), ctypes.byref(rows))
    if n < 0:
        _check(n)
    return (ZpPair * n)(*pairs[:n]), (ZpMerge * nm.value)(*merges[:nm.value]), int(rows.value)


def profile_enable(on: bool) -> None:
    """Starts (clearing old records) or stops the library's per-kernel hipEvent timing."""
    _check(lib().zp_profile_enable(1 if on else 0))


def profile_records():
    """[(kernel label, ms)] for every launch since profile_enable(True); waits for them to finish."""
    out = []
    buf = ctypes.create_string_buffer(64)
    ms = ctypes.c_float(0)
    for i in range(lib().zp_profile_count()):
        _check(lib().zp_profile_get(i, buf, 64, ctypes.byref(ms)))
        out.append((buf.value.decode(), float(ms.value)))
    return out


def remap_plan(A, P: int, b_intra: int = 1, b_inter: int = 1):
    """Host helper: transfer matrix of the remapping layer -> (M as a d x d int32 array, objective)."""
    A = np.ascontiguousarray(A, dtype=np.int32)
    d = len(A)
    M = np.zeros((d, d), np.int32)
    obj = ctypes.c_int64(0)
    _check(lib().zp_remap_plan(A.ctypes.data_as(ctypes.c_void_p), d, int(P), int(b_intra), int(b_inter),
                               M.ctypes.data_as(ctypes.c_void_p), ctypes.byref(obj)))
    return M, int(obj.value)


def remap_indices(A, M):
    """Host helper: idx[balanced position] = attention-layout position for a transfer matrix M."""
    A = np.ascontiguousarray(A, dtype=np.int32)
    M = np.ascontiguousarray(M, dtype=np.int32)
    idx = np.zeros(int(A.sum()), np.int32)
    _check(lib().zp_remap_indices(A.ctypes.data_as(ctypes.c_void_p), M.ctypes.data_as(ctypes.c_void_p), len(A),
                                  idx.ctypes.data_as(ctypes.c_void_p), len(idx)))
    return idx


def node_segments(lengths, placements, P: int, N: int):
    """Host helper: attention layout of a placement list -> (runs as dicts, tokens per device)."""
    lens = np.ascontiguousarray(lengths, dtype=np.int32)
    arr = (ZpPlacement * max(len(placements), 1))()
    for i, pl in enumerate(placements):
        for f, _ in ZpPlacement._fields_:
            setattr(arr[i], f, int(pl[f]))
    cap = 2 * len(placements) + 1
    out = (ZpSegment * cap)()
    n = ctypes.c_int32(0)
    A = np.zeros(P * N, np.int32)
    _check(lib().zp_node_segments(lens.ctypes.data_as(ctypes.c_void_p), len(lens), arr, len(placements), int(P), int(N),
                                  out, cap, ctypes.byref(n), A.ctypes.data_as(ctypes.c_void_p)))
    segs = [{f: getattr(out[i], f) for f, _ in ZpSegment._fields_} for i in range(n.value)]
    return segs, A


def partition(lengths, P: int, N: int, L: int):
    """Host helper: hierarchical partitioner -> (placements as dicts, s1, [s0 per node])."""
    lens = np.ascontiguousarray(lengths, dtype=np.int32)
    cap = max(len(lens) * max(P, 1) * max(N, 1), 1)
    out = (ZpPlacement * cap)()
    n = ctypes.c_int32(0)
    s1 = ctypes.c_int32(0)
    s0 = np.zeros(N, np.int32)
    _check(lib().zp_partition(lens.ctypes.data_as(ctypes.c_void_p), len(lens), int(P), int(N), int(L), out, cap,
                              ctypes.byref(n), ctypes.byref(s1), s0.ctypes.data_as(ctypes.c_void_p)))
    pl = [{f: getattr(out[i], f) for f, _ in ZpPlacement._fields_} for i in range(n.value)]
    return pl, int(s1.value), [int(x) for x in s0]
