"""Hierarchical sequence partitioner of Sec. 3.1, written out step by step -- TEST INFRASTRUCTURE.

Alg. 1 (inter-node partitioning) and Alg. 2 (intra-node partitioning) in the paper's order and notation:
S sequences of lengths |s|, P devices per node, N nodes, token capacity L per device; thresholds s1 (inter-node
zone) and s0 (intra-node zone); zones z2 (inter-node), z1 (intra-node), z0 (local).

Readings where the listing is silent:
 * a sequence of z2 is split evenly over k = min(N, ceil(|s| / s_avg)) node buckets, the k least loaded ones
   (ties: lowest index); with z2 empty the step is skipped;
 * "split s evenly to P devices" / "split into ceil(|s|^2 / c_avg) fragments": the sequence runs on a ring of
   G devices (G = k*P for z2, G = min(P, ceil(|s|^2 / c_avg)) for z1), is cut into 2G equal-length chunks
   (chunk c = [floor(c|s|/2G), floor((c+1)|s|/2G)) ) and ring rank r holds chunks r and 2G-1-r (Sec. 3.2);
 * a z1 sequence with G = 1 is placed whole; round-robin continues across the sequences of z1;
 * loads compared in the greedy steps are token counts, as the listing writes them;
 * the budgets s_avg and c_avg are rationals: the ceilings are taken exactly (integer arithmetic), so that a
   sequence of exactly k budgets gets k buckets whatever a floating-point quotient would round to.
Returns placements: dicts {seq, zone, ring, rank, node, device, tokens}.
"""
from __future__ import annotations



def ceil_ratio(num: int, den: int) -> int:
    """ceil(num / den) in exact integer arithmetic; an all-zero zone (den = 0) asks for one bucket."""
    return -(-num // den) if den > 0 else 1


def ring_tokens(length: int, G: int, r: int) -> int:
    b = lambda c: (c * length) // (2 * G)
    return (b(r + 1) - b(r)) + (b(2 * G - r) - b(2 * G - 1 - r))


def inter_node(lengths, P: int, N: int, L: int):
    """Alg. 1. Returns (node_buckets, s1): node_buckets[n] = list of ('whole', seq) or ('frag', seq, k, m)
    (fragment m of k of an inter-node sequence)."""
    order = sorted(range(len(lengths)), key=lambda s: (-lengths[s], s))
    s1 = P * L
    while True:
        node_buckets = [[] for _ in range(N)]
        load = [0] * N
        flag = False
        z01 = [s for s in order if lengths[s] < s1]
        z2 = [s for s in order if lengths[s] >= s1]
        if z2:
            z2_tokens = sum(lengths[s] for s in z2)          # s_avg = z2_tokens / N, kept as an exact fraction
            for s in z2:
                k = max(1, min(N, ceil_ratio(lengths[s] * N, z2_tokens)))  # ceil(|s| / s_avg); an empty sequence still gets a bucket
                nodes = sorted(range(N), key=lambda n: (load[n], n))[:k]
                for m, n in enumerate(sorted(nodes)):
                    node_buckets[n].append(("frag", s, k, m))
                    load[n] += sum(ring_tokens(lengths[s], k * P, m * P + p) for p in range(P))
        for s in z01:
            idx = min(range(N), key=lambda n: (load[n], n))
            if lengths[s] + load[idx] > P * L:
                s1 = max(lengths[t] for t in z01)
                flag = True
                break
            node_buckets[idx].append(("whole", s))
            load[idx] += lengths[s]
        if not flag:
            return node_buckets, s1


def intra_node(lengths, bucket, P: int, L: int, node: int):
    """Alg. 2 for one node bucket. Returns (placements, s0)."""
    z2 = [it for it in bucket if it[0] == "frag"]
    z01 = sorted([it[1] for it in bucket if it[0] == "whole"], key=lambda s: (-lengths[s], s))
    s0 = L
    while True:
        out = []
        load = [0] * P
        flag = False
        for _, s, k, m in z2:
            G = k * P
            for p in range(P):
                t = ring_tokens(lengths[s], G, m * P + p)
                out.append(dict(seq=s, zone=2, ring=G, rank=m * P + p, node=node, device=p, tokens=t))
                load[p] += t
        z0 = [s for s in z01 if lengths[s] < s0]
        z1 = [s for s in z01 if lengths[s] >= s0]
        if z1:
            z1_cost = sum(lengths[s] ** 2 for s in z1)       # c_avg = z1_cost / P, kept as an exact fraction
            nxt = 0
            for s in z1:
                G = max(1, min(P, ceil_ratio(lengths[s] ** 2 * P, z1_cost)))  # ceil(|s|^2 / c_avg); an empty sequence still gets a bucket
                for r in range(G):
                    p = nxt % P
                    nxt += 1
                    t = ring_tokens(lengths[s], G, r) if G > 1 else lengths[s]
                    out.append(dict(seq=s, zone=1, ring=G, rank=r, node=node, device=p, tokens=t))
                    load[p] += t
        for s in z0:
            idx = min(range(P), key=lambda p: (load[p], p))
            if lengths[s] + load[idx] > L:
                s0 = max(lengths[t] for t in z0)
                flag = True
                break
            out.append(dict(seq=s, zone=0, ring=1, rank=0, node=node, device=idx, tokens=lengths[s]))
            load[idx] += lengths[s]
        if not flag:
            return out, s0


def partition(lengths, P: int, N: int, L: int):
    """Alg. 1 then Alg. 2 on every node. Returns (placements, s1, [s0 per node])."""
    lengths = [int(x) for x in lengths]
    node_buckets, s1 = inter_node(lengths, P, N, L)
    out, s0s = [], []
    for n, b in enumerate(node_buckets):
        pl, s0 = intra_node(lengths, b, P, L, n)
        out += pl
        s0s.append(s0)
    return out, s1, s0s
