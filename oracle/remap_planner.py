"""TEST INFRASTRUCTURE ONLY (imported by tests/, the smoke check and the CPU-baseline leg of the benchmark).

Oracle of the remapping layer's transfer plan (Sec. 3.4, Eq. 2): the optimisation problem written out as its
definition, not a fast algorithm.

A[i]  tokens rank i holds in the attention layout; B[i] the balanced target (readings: B_i = floor(T/d) + [i < T mod d],
integral M).  M[i][j] tokens moved from rank i to rank j, with
    sum_j M[i][j] = max(A_i - B_i, 0),   sum_i M[i][j] = max(B_j - A_j, 0),   M >= 0,
and the cost to minimise is  max_i sum_j T[i][j] * M[i][j]  with T[i][j] = b_inter if i and j sit in different nodes
(rank r is in node r // P) and b_intra otherwise ("*" in Eq. 2 read as the elementwise product).

optimum_bruteforce enumerates every integral feasible M (tiny instances); optimum_lp solves the linear relaxation with
scipy's LP solver (a lower bound of the integral optimum).  remap_indices applies the token-selection rule to a given
M: a surplus rank sends the tail of its buffer, split among destinations in ascending rank order; a rank's balanced
buffer is its kept head followed by the arrivals in ascending source order.
"""
import itertools

import numpy as np


def targets(A):
    A = [int(a) for a in A]
    d, T = len(A), sum(A)
    return [T // d + (1 if i < T % d else 0) for i in range(d)]


def surplus_deficit(A):
    Bt = targets(A)
    return [max(a - b, 0) for a, b in zip(A, Bt)], [max(b - a, 0) for a, b in zip(A, Bt)]


def cost_matrix(d, P, b_intra, b_inter):
    return [[(b_inter if i // P != j // P else b_intra) for j in range(d)] for i in range(d)]


def is_feasible(A, M):
    s, t = surplus_deficit(A)
    d = len(A)
    M = np.asarray(M)
    return (M.shape == (d, d) and (M >= 0).all() and [int(x) for x in M.sum(axis=1)] == s
            and [int(x) for x in M.sum(axis=0)] == t)


def objective(M, P, b_intra, b_inter):
    d = len(M)
    Tm = cost_matrix(d, P, b_intra, b_inter)
    return max(sum(Tm[i][j] * int(M[i][j]) for j in range(d)) for i in range(d))


def _compositions(total, caps):
    """All ways to write `total` as an ordered sum of len(caps) non-negative integers with part k <= caps[k]."""
    if len(caps) == 1:
        if total <= caps[0]:
            yield (total,)
        return
    for x in range(min(total, caps[0]) + 1):
        for rest in _compositions(total - x, caps[1:]):
            yield (x,) + rest


def optimum_bruteforce(A, P, b_intra, b_inter):
    """Minimum of the objective over every integral feasible M, and one minimiser. Exponential: tiny inputs only."""
    s, t = surplus_deficit(A)
    d = len(A)
    best, best_M = None, None

    def rec(i, remaining, rows):
        nonlocal best, best_M
        if i == d:
            if all(r == 0 for r in remaining):
                val = objective(rows, P, b_intra, b_inter)
                if best is None or val < best:
                    best, best_M = val, [list(r) for r in rows]
            return
        for row in _compositions(s[i], remaining):
            rec(i + 1, [r - x for r, x in zip(remaining, row)], rows + [row])

    rec(0, list(t), [])
    return best, best_M


def optimum_lp(A, P, b_intra, b_inter):
    """Optimum of the linear relaxation (real-valued M) by scipy.optimize.linprog: variables M (d*d) and the bound z."""
    from scipy.optimize import linprog
    s, t = surplus_deficit(A)
    d = len(A)
    Tm = cost_matrix(d, P, b_intra, b_inter)
    n = d * d + 1
    c = np.zeros(n); c[-1] = 1.0
    A_ub = np.zeros((d, n)); b_ub = np.zeros(d)
    for i in range(d):
        for j in range(d):
            A_ub[i, i * d + j] = Tm[i][j]
        A_ub[i, -1] = -1.0
    A_eq = np.zeros((2 * d, n)); b_eq = np.zeros(2 * d)
    for i in range(d):
        for j in range(d):
            A_eq[i, i * d + j] = 1.0
            A_eq[d + j, i * d + j] = 1.0
        b_eq[i] = s[i]; b_eq[d + i] = t[i]
    r = linprog(c, A_ub=A_ub, b_ub=b_ub, A_eq=A_eq, b_eq=b_eq, bounds=[(0, None)] * n, method="highs")
    assert r.status == 0, r.message
    return float(r.fun)


def remap_indices(A, M):
    """idx[linear position] = attention-layout position, both counted over the concatenation of the rank buffers."""
    A = [int(a) for a in A]
    d = len(A)
    Bt = targets(A)
    s, _ = surplus_deficit(A)
    offA = [0]
    for a in A:
        offA.append(offA[-1] + a)
    # where, inside sender i's buffer, the segment for destination j starts: the tail, destinations ascending
    seg_start = [[0] * d for _ in range(d)]
    for i in range(d):
        p = A[i] - s[i]
        for j in range(d):
            seg_start[i][j] = p
            p += int(M[i][j])
    idx = []
    for r in range(d):
        kept = min(A[r], Bt[r])
        buf = [offA[r] + p for p in range(kept)]
        for i in range(d):
            buf += [offA[i] + seg_start[i][r] + p for p in range(int(M[i][r]))]
        assert len(buf) == Bt[r]
        idx += buf
    return np.asarray(idx, dtype=np.int32)
