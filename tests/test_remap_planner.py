"""CPU pins of the remap-plan oracle (Sec. 3.4, Eq. 2) and tests of the host planner behind the C ABI against it."""
import os

import numpy as np
import pytest

from oracle import remap_planner as RP
from paper_2509_21841_amd import binding as B

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def golden_plans():
    out = []
    for line in open(os.path.join(GOLD, "remap_plan_examples.txt")):
        if line.startswith("#") or not line.strip():
            continue
        head, A, opt, _ = [x.strip() for x in line.split("|")]
        P, bi, bo = [int(x) for x in head.split()]
        out.append((P, bi, bo, [int(x) for x in A.split()], int(opt)))
    return out


def golden_indices():
    out, cur = [], {}
    for line in open(os.path.join(GOLD, "remap_indices_example.txt")):
        if line.startswith("A:"):
            cur = {"A": [int(x) for x in line[2:].split()]}
        elif line.startswith("M:"):
            cur["M"] = [[int(x) for x in row.split()] for row in line[2:].split("/")]
        elif line.startswith("idx:"):
            cur["idx"] = [int(x) for x in line[4:].split()]
            out.append(cur)
    return out


# ---- the oracle against what the mathematics fixes ---------------------------------------------------
@pytest.mark.parametrize("P,bi,bo,A,opt", golden_plans())
def test_oracle_bruteforce_matches_hand_worked_optima(P, bi, bo, A, opt):
    val, M = RP.optimum_bruteforce(A, P, bi, bo)
    assert val == opt and RP.is_feasible(A, M) and RP.objective(M, P, bi, bo) == opt


def test_oracle_single_node_closed_form_holds_for_every_feasible_plan():
    """All T_ij equal and the row sums fixed by the first constraint: every feasible M costs b * (largest surplus)."""
    rng = np.random.default_rng(5)
    for _ in range(20):
        A = rng.integers(0, 7, size=4).tolist()
        s, t = RP.surplus_deficit(A)
        seen = 0
        # enumerate every feasible M through the brute-force recursion's building block
        def rec(i, remaining, rows):
            nonlocal seen
            if i == 4:
                if all(r == 0 for r in remaining):
                    seen += 1
                    assert RP.objective(rows, 4, 3, 11) == 3 * max(s)
                return
            for row in RP._compositions(s[i], remaining):
                rec(i + 1, [r - x for r, x in zip(remaining, row)], rows + [row])
        rec(0, list(t), [])
        assert seen >= 1


def test_oracle_bruteforce_against_lp_relaxation():
    """Library second opinion: the LP relaxation bounds the integral optimum from below, within one token's cost."""
    rng = np.random.default_rng(7)
    for _ in range(25):
        P = int(rng.choice([1, 2, 3]))
        d = P * int(rng.choice([1, 2]))
        A = rng.integers(0, 6, size=d).tolist()
        bi, bo = int(rng.integers(1, 4)), int(rng.integers(4, 9))
        bf, _ = RP.optimum_bruteforce(A, P, bi, bo)
        lp = RP.optimum_lp(A, P, bi, bo)
        assert lp - 1e-7 <= bf <= lp + bo + 1e-7, (A, P, bi, bo, bf, lp)


@pytest.mark.parametrize("ex", golden_indices())
def test_oracle_indices_match_hand_worked_permutations(ex):
    assert RP.remap_indices(ex["A"], ex["M"]).tolist() == ex["idx"]


def test_oracle_targets_and_conservation():
    assert RP.targets([7, 0, 0]) == [3, 2, 2] and RP.targets([4, 4]) == [4, 4] and RP.targets([0, 0, 1]) == [1, 0, 0]
    s, t = RP.surplus_deficit([9, 1, 5, 1])
    assert sum(s) == sum(t) == 6


# ---- the host planner (C ABI) against the oracle ------------------------------------------------------
@pytest.mark.parametrize("P,bi,bo,A,opt", golden_plans())
def test_planner_reaches_hand_worked_optima(P, bi, bo, A, opt):
    M, val = B.remap_plan(A, P, bi, bo)
    assert RP.is_feasible(A, M) and val == opt == RP.objective(M, P, bi, bo)


def test_planner_is_optimal_on_tiny_instances():
    rng = np.random.default_rng(11)
    for _ in range(60):
        P = int(rng.choice([1, 2, 3]))
        d = P * int(rng.choice([1, 2, 3])) if P < 3 else P * int(rng.choice([1, 2]))
        A = rng.integers(0, 6, size=d).tolist()
        bi = int(rng.integers(1, 4)); bo = bi + int(rng.integers(0, 6))
        M, val = B.remap_plan(A, P, bi, bo)
        assert RP.is_feasible(A, M), (A, M)
        assert val == RP.objective(M, P, bi, bo)
        bf, _ = RP.optimum_bruteforce(A, P, bi, bo)
        assert val == bf, (A, P, bi, bo, val, bf)


def test_planner_within_one_token_of_lp_bound_at_scale():
    rng = np.random.default_rng(13)
    for P, N in [(8, 1), (8, 2), (8, 4), (4, 3)]:
        d = P * N
        A = rng.integers(0, 40000, size=d).tolist()
        M, val = B.remap_plan(A, P, 1, 7)
        assert RP.is_feasible(A, M)
        lp = RP.optimum_lp(A, P, 1, 7)
        assert lp - 1e-6 * lp <= val <= lp + 7 + 1e-6 * lp, (val, lp)
        # intra-node traffic never crosses: a node that can absorb its own surplus sends nothing out
        Ma = np.asarray(M)
        s, t = RP.surplus_deficit(A)
        for n in range(N):
            sl = slice(n * P, (n + 1) * P)
            out_flow = Ma[sl].sum() - Ma[sl, sl].sum()
            assert out_flow == max(sum(s[sl]) - sum(t[sl]), 0)


def test_planner_indices_match_oracle_rule_and_are_permutations():
    rng = np.random.default_rng(17)
    for P, N in [(2, 2), (8, 1), (4, 2)]:
        A = rng.integers(0, 300, size=P * N).tolist()
        M, _ = B.remap_plan(A, P, 1, 4)
        idx = B.remap_indices(A, M)
        assert np.array_equal(idx, RP.remap_indices(A, M))
        assert sorted(idx.tolist()) == list(range(sum(A)))
    for ex in golden_indices():
        assert B.remap_indices(ex["A"], ex["M"]).tolist() == ex["idx"]


def test_planner_argument_validation():
    L = B.lib()
    import ctypes
    A = (ctypes.c_int32 * 4)(1, 2, 3, 4); M = (ctypes.c_int32 * 16)(); obj = ctypes.c_int64(0)
    assert L.zp_remap_plan(A, 4, 0, 1, 2, M, ctypes.byref(obj)) == -1      # P < 1
    assert L.zp_remap_plan(A, 4, 2, 3, 2, M, ctypes.byref(obj)) == -1      # b_inter < b_intra
    assert L.zp_remap_plan(A, 4, 2, 0, 2, M, ctypes.byref(obj)) == -1      # b_intra < 1
    assert L.zp_remap_plan(None, 4, 2, 1, 2, M, ctypes.byref(obj)) == -1
    A[1] = -1
    assert L.zp_remap_plan(A, 4, 2, 1, 2, M, ctypes.byref(obj)) == -1      # negative count
    A[1] = 2
    assert L.zp_remap_plan(A, 4, 2, 1, 2, M, ctypes.byref(obj)) == 0
    idx = (ctypes.c_int32 * 10)()
    M[0] = 5                                                                # rows no longer match the surplus
    assert L.zp_remap_indices(A, M, 4, idx, 10) == -1
