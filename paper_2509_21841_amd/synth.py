"""Seeded synthetic workloads: sequence-length mixes, packed Q/K/V/dO tensors and token layouts.

Holds none of the attention arithmetic; the tests, the bench and the smoke check all draw their
inputs here so that the HIP path and the CPU oracle see the same buffers.

The length mixes stand in for the long-tailed corpora the paper trains on (Fig. 1, Table 2); the
paper itself ran synthetic batches matched to length histograms (Sec. 5.1).
"""
from __future__ import annotations

import numpy as np
import torch


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([int(seed), int(stream)]))


def lengths_tiny(seed: int = 1001, n: int = 8, lo: int = 16, hi: int = 512, budget: int = 2048):
    """n lengths uniform over [lo, hi], redrawn until they pack into <= budget tokens."""
    r = _rng(seed, 0)
    while True:
        L = r.integers(lo, hi + 1, size=n)
        if int(L.sum()) <= budget:
            return [int(x) for x in L]


def lengths_lognormal(total: int, seed: int, median: int = 1024, sigma: float = 1.0, lo: int = 64, hi: int = 32768):
    """Lengths clip(round(exp(N(ln median, sigma^2))), lo, hi) until `total` tokens are packed; the last
    sequence takes the remainder (merged into the previous one if below lo)."""
    r = _rng(seed, 0)
    out, left = [], total
    while left > 0:
        L = int(np.clip(np.rint(np.exp(r.normal(np.log(median), sigma))), lo, hi))
        if L >= left:
            if left < lo and out:
                out[-1] += left
            else:
                out.append(left)
            left = 0
        else:
            out.append(L)
            left -= L
    return out


def lengths_longtail(total: int, seed: int, p_long: float = 0.1, short=(128, 4096), long=(16384, 65536),
                     long_multiple: int = 256):
    """90% short ~ U[short], 10% long ~ U[long] rounded to a multiple of `long_multiple`; stops at the budget,
    truncating the last draw (merged into the previous if below its class minimum); at least one long."""
    r = _rng(seed, 0)
    while True:
        out, is_long, left = [], [], total
        while left > 0:
            if r.random() < p_long:
                L = int(r.integers(long[0], long[1] + 1)); L = max(long_multiple, (L // long_multiple) * long_multiple)
                lng, mn = True, long[0]
            else:
                L = int(r.integers(short[0], short[1] + 1)); lng, mn = False, short[0]
            if L >= left:
                L = left
                if L < mn and out:
                    out[-1] += L
                else:
                    if lng:
                        L2 = (L // long_multiple) * long_multiple
                        if L2 >= mn:
                            out.append(L2); is_long.append(True)
                            if L - L2 > 0:
                                out.append(L - L2); is_long.append(False)
                        else:
                            out.append(L); is_long.append(False)
                    else:
                        out.append(L); is_long.append(False)
                left = 0
            else:
                out.append(L); is_long.append(lng); left -= L
        if any(is_long):
            return out, is_long


# Proportion of sequences per length bin (Table 2); bin k covers [edge[k], edge[k+1]) tokens. The GitHub row adds up
# to 0.945 as printed and is renormalised; inside a bin lengths are drawn uniformly (the paper does not say).
TABLE2_EDGES = [64, 1024, 2048, 4096, 8192, 16384, 32768, 65536, 131072, 262144]
TABLE2 = {
    "arxiv": [0.032, 0.03, 0.08, 0.219, 0.338, 0.224, 0.077, 0.0, 0.0],
    "github": [0.0, 0.34, 0.095, 0.104, 0.107, 0.102, 0.088, 0.064, 0.045],
    "prolong64k": [0.231, 0.042, 0.021, 0.012, 0.013, 0.008, 0.673, 0.0, 0.0],
}


def lengths_table2(total: int, seed: int, dataset: str, multiple: int = 64):
    """Lengths drawn bin by bin from a Table 2 histogram until `total` tokens are packed. Lengths are rounded down to a
    multiple of `multiple` (>= multiple); a draw that does not fit takes what is left of the budget."""
    p = np.asarray(TABLE2[dataset], dtype=np.float64)
    p = p / p.sum()
    r = _rng(seed, 0)
    out, left = [], int(total)
    while left > 0:
        k = int(r.choice(len(p), p=p))
        L = int(r.integers(TABLE2_EDGES[k], TABLE2_EDGES[k + 1]))
        L = max(multiple, (L // multiple) * multiple)
        L = min(L, left)
        out.append(L)
        left -= L
    return out


def cu_seqlens(lengths) -> np.ndarray:
    cu = np.zeros(len(lengths) + 1, np.int32)
    cu[1:] = np.cumsum(np.asarray(lengths, np.int64))
    return cu


def normal_bf16(shape, seed: int, stream: int, device="cpu") -> torch.Tensor:
    """i.i.d. N(0,1) rounded to bfloat16 (round-to-nearest-even), seeded per (seed, stream, device type)."""
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) * 1000003 + int(stream))
    n = int(np.prod(shape))
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    flat = out.view(-1)
    step = 1 << 26
    for a in range(0, n, step):
        b = min(n, a + step)
        flat[a:b] = torch.randn(b - a, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    return out


def make_qkv(T: int, Hq: int, Hkv: int, d: int, seed: int, device="cpu", with_dout: bool = False):
    q = normal_bf16((T, Hq, d), seed, 1, device)
    k = normal_bf16((T, Hkv, d), seed, 2, device)
    v = normal_bf16((T, Hkv, d), seed, 3, device)
    if with_dout:
        return q, k, v, normal_bf16((T, Hq, d), seed, 4, device)
    return q, k, v


def balanced_attention_layout(lengths, R: int = 8):
    """Stand-in for the partitioner's output: sequences sorted by descending L^2 are each placed whole on the
    virtual rank with the least accumulated L^2 (ties -> lowest rank); the attention layout is ranks 0..R-1
    concatenated in placement order.  The linear layout is the drawn packing order.
    Returns (idx, attn_lengths, order): idx[t_attn] = t_linear, the lengths in attention-layout order, and the
    sequence order."""
    lengths = [int(x) for x in lengths]
    cu = cu_seqlens(lengths)
    order = sorted(range(len(lengths)), key=lambda s: (-lengths[s] ** 2, s))
    load = [0] * R
    buckets = [[] for _ in range(R)]
    for s in order:
        r = min(range(R), key=lambda i: (load[i], i))
        buckets[r].append(s)
        load[r] += lengths[s] ** 2
    seq_order = [s for b in buckets for s in b]
    idx = np.concatenate([np.arange(cu[s], cu[s + 1], dtype=np.int32) for s in seq_order]) if seq_order else np.zeros(0, np.int32)
    return idx, [lengths[s] for s in seq_order], seq_order


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """Raw uint16 bit patterns of a bfloat16 tensor, on the host."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
