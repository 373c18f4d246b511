"""Hierarchical partitioner (Sec. 3.1): the step-by-step oracle against hand-worked examples and the properties
the paper states, and the library's host implementation against the oracle (CPU only)."""
import collections
import os

import numpy as np
import pytest

from oracle import partitioner as opt
from paper_2509_21841_amd import binding as B
from paper_2509_21841_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))
KEYS = ("seq", "zone", "ring", "rank", "node", "device", "tokens")


def golden_cases():
    cases, cur = [], None
    for line in open(os.path.join(HERE, "golden", "partition_examples.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.split()
        if tok[0] == "case":
            cur = dict(name=tok[1], P=int(tok[2]), N=int(tok[3]), L=int(tok[4]), lengths=[int(x) for x in tok[5:]], rows=[])
            cases.append(cur)
        elif tok[0] == "thresholds":
            cur["s1"], cur["s0"] = int(tok[1]), [int(x) for x in tok[2:]]
        else:
            cur["rows"].append(dict(zip(KEYS, map(int, tok))))
    return cases


def canon(pl):
    return sorted(tuple(p[k] for k in KEYS) for p in pl)


@pytest.mark.parametrize("case", golden_cases(), ids=lambda c: c["name"])
def test_oracle_and_library_match_hand_worked_examples(case):
    for impl in (opt.partition, B.partition):
        pl, s1, s0 = impl(case["lengths"], case["P"], case["N"], case["L"])
        assert canon(pl) == canon(case["rows"]) and s1 == case["s1"] and s0 == case["s0"]


# Plausible mistakes planted in a COPY of the oracle's source (on the CPU, never in the library): each one must make
# at least one hand-worked example fail, otherwise the examples do not pin that step of Alg. 1 / Alg. 2.
PLANTED_MISTAKES = {
    "s_avg over every sequence instead of the inter-node zone":
        ("z2_tokens = sum(lengths[s] for s in z2)", "z2_tokens = sum(lengths[s] for s in order)"),
    "floor instead of ceil for the number of node buckets":
        ("ceil_ratio(lengths[s] * N, z2_tokens)", "((lengths[s] * N) // z2_tokens)"),
    "most loaded nodes instead of least loaded":
        ("key=lambda n: (load[n], n))[:k]", "key=lambda n: (-load[n], n))[:k]"),
    "fragments numbered in load order instead of node order":
        ("enumerate(sorted(nodes))", "enumerate(nodes)"),
    "threshold s1 not lowered to the longest remaining sequence":
        ("s1 = max(lengths[t] for t in z01)", "s1 = min(lengths[t] for t in z01)"),
    "c_avg over every sequence of the node instead of the intra-node zone":
        ("z1_cost = sum(lengths[s] ** 2 for s in z1)", "z1_cost = sum(lengths[s] ** 2 for s in z01)"),
    "floor instead of ceil for the number of fragments":
        ("ceil_ratio(lengths[s] ** 2 * P, z1_cost)", "((lengths[s] ** 2 * P) // z1_cost)"),
    "linear cost |s| instead of |s|^2":
        ("ceil_ratio(lengths[s] ** 2 * P, z1_cost)", "ceil_ratio(lengths[s] * P, sum(lengths[t] for t in z1))"),
    "round-robin restarts at device 0 for every intra-node sequence":
        ("            for s in z1:\n", "            for s in z1:\n                nxt = 0\n"),
    "threshold s0 not lowered to the longest remaining sequence":
        ("s0 = max(lengths[t] for t in z0)", "s0 = min(lengths[t] for t in z0)"),
    "ring rank holds two neighbouring chunks instead of chunks r and 2G-1-r":
        ("return (b(r + 1) - b(r)) + (b(2 * G - r) - b(2 * G - 1 - r))", "return b(2 * r + 2) - b(2 * r)"),
    "local sequences to the most loaded device":
        ("idx = min(range(P), key=lambda p: (load[p], p))", "idx = max(range(P), key=lambda p: (load[p], -p))"),
    "local sequences to the most loaded node":
        ("idx = min(range(N), key=lambda n: (load[n], n))", "idx = max(range(N), key=lambda n: (load[n], -n))"),
}


@pytest.mark.parametrize("what", sorted(PLANTED_MISTAKES))
def test_hand_worked_examples_catch_planted_mistakes(what):
    old, new = PLANTED_MISTAKES[what]
    src = open(opt.__file__).read()
    assert src.count(old) == 1, f"the oracle no longer contains the line this mistake is planted in: {old!r}"
    ns = {"__name__": "planted"}
    exec(compile(src.replace(old, new), "planted_" + os.path.basename(opt.__file__), "exec"), ns)
    caught = []
    for case in golden_cases():
        try:
            pl, s1, s0 = ns["partition"](case["lengths"], case["P"], case["N"], case["L"])
            ok = canon(pl) == canon(case["rows"]) and s1 == case["s1"] and s0 == case["s0"]
        except Exception:
            ok = False
        if not ok:
            caught.append(case["name"])
    assert caught, f"no hand-worked example notices: {what}"


def check_properties(lengths, P, N, L, pl, s1, s0):
    by_seq = collections.defaultdict(list)
    for p in pl:
        by_seq[p["seq"]].append(p)
    assert sorted(by_seq) == [s for s in range(len(lengths))]                      # every sequence placed
    assert sum(p["tokens"] for p in pl) == sum(lengths)                            # token conservation
    load = collections.Counter(); has_local = set()
    for s, items in by_seq.items():
        zone = items[0]["zone"]; G = items[0]["ring"]
        assert all(i["zone"] == zone and i["ring"] == G for i in items)
        assert sorted(i["rank"] for i in items) == list(range(G))                  # every ring rank exactly once
        assert sum(i["tokens"] for i in items) == lengths[s]
        if zone == 2:
            assert lengths[s] >= s1 and G % P == 0                                 # spans whole nodes
        elif zone == 1:
            assert s0[items[0]["node"]] <= lengths[s] < s1 and len({i["node"] for i in items}) == 1 and G <= P
        else:
            assert lengths[s] < s0[items[0]["node"]] and G == 1
        for i in items:
            load[(i["node"], i["device"])] += i["tokens"]
            if zone == 0:
                has_local.add((i["node"], i["device"]))
            # a ring rank holds chunks r and 2G-1-r of 2G equal-length chunks (Sec. 3.2)
            if G > 1:
                assert i["tokens"] == opt.ring_tokens(lengths[s], G, i["rank"])
    for dev in has_local:                                                          # greedy step never overfills
        assert load[dev] <= L
    return load


@pytest.mark.parametrize("seed", range(12))
def test_properties_and_library_equals_oracle_on_random_batches(seed):
    r = np.random.default_rng(seed)
    P, N = int(r.choice([1, 2, 4, 8])), int(r.choice([1, 2, 4]))
    S = int(r.integers(1, 60))
    lengths = np.clip(np.rint(np.exp(r.normal(6.5, 1.3, S))), 1, 200000).astype(int).tolist()
    slack = float(r.choice([1.0, 1.1, 1.5, 3.0]))
    L = max(1, int(np.ceil(sum(lengths) * slack / (P * N))))
    pl, s1, s0 = opt.partition(lengths, P, N, L)
    check_properties(lengths, P, N, L, pl, s1, s0)
    pl2, s1b, s0b = B.partition(lengths, P, N, L)
    assert canon(pl2) == canon(pl) and s1b == s1 and s0b == s0


def test_degenerate_cases():
    # everything short and roomy: all local, balanced within one sequence length
    lengths = [100] * 64
    pl, s1, s0 = opt.partition(lengths, 8, 1, 1000)
    load = check_properties(lengths, 8, 1, 1000, pl, s1, s0)
    assert all(p["zone"] == 0 for p in pl) and set(load.values()) == {800}
    # one sequence larger than a node: a ring over every device of every node it needs
    lengths = [64000, 10, 10]
    pl, s1, s0 = opt.partition(lengths, 4, 2, 8000)
    big = [p for p in pl if p["seq"] == 0]
    assert big[0]["zone"] == 2 and big[0]["ring"] == 8 and len(big) == 8 and all(p["tokens"] == 8000 for p in big)
    assert canon(B.partition(lengths, 4, 2, 8000)[0]) == canon(pl)
    # empty sequences behind sequences that already overfill a node or a device: the thresholds fall to 0, the empty
    # sequences join a ring zone (length 0 against a non-zero budget, or a zero budget) and must still be placed
    for lengths, P, L in (([10, 10, 0, 0], 2, 8), ([0, 0, 0], 2, 4), ([9, 0], 1, 4)):
        pl, s1, s0 = opt.partition(lengths, P, 1, L)
        assert sorted({p["seq"] for p in pl}) == list(range(len(lengths))) and sum(p["tokens"] for p in pl) == sum(lengths)
        pl2, s1b, s0b = B.partition(lengths, P, 1, L)
        assert canon(pl2) == canon(pl) and (s1b, s0b) == (s1, s0)
    # empty batch
    assert opt.partition([], 2, 2, 10)[0] == [] and B.partition([], 2, 2, 10)[0] == []


def test_paper_sized_batches():
    for lengths, P, N, L in ((synth.lengths_lognormal(262144, 1005), 8, 4, 10240),
                             (synth.lengths_longtail(131072, 1003)[0], 8, 2, 10240)):
        pl, s1, s0 = opt.partition(lengths, P, N, L)
        check_properties(lengths, P, N, L, pl, s1, s0)
        assert canon(B.partition(lengths, P, N, L)[0]) == canon(pl)


# ---- placement -> attention layout -> remap plan (host composition, no device) -------------------------
@pytest.mark.parametrize("lengths,P,N,L", [([700, 90, 300, 1500, 64, 200, 33], 4, 1, 800),
                                           ([2600, 150, 400, 90, 1100, 60], 2, 2, 700),
                                           ([100, 200, 50], 4, 1, 400), ([5000], 8, 1, 1000)])
def test_node_plan_composition(lengths, P, N, L):
    from paper_2509_21841_amd.node import NodePlan
    from paper_2509_21841_amd import binding as B
    plan = NodePlan(lengths, P, N, L, b_intra=1, b_inter=4)
    T = sum(lengths)
    # runs tile the concatenated device buffers, device by device, and cover every token of every sequence once
    assert plan.T == T and int(plan.cu[-1]) == T
    assert sorted(plan.orig.tolist()) == list(range(T)) and sorted(plan.idx.tolist()) == list(range(T))
    tok = 0
    for s in plan.segments:
        assert s["tok0"] == tok and s["len"] >= 0
        tok += s["len"]
    per_rank = np.zeros(P * N, np.int64)
    for s in plan.segments:
        per_rank[s["node"] * P + s["device"]] += s["len"]
    assert np.array_equal(per_rank, plan.A)
    # a ring rank of G holds chunks r and 2G-1-r: the oracle's ring ownership
    by = {}
    for s in plan.segments:
        if s["n_chunks"] > 1:
            by.setdefault((s["seq"], s["node"], s["device"]), []).append(s["chunk"])
    for (seq, _, _), chunks in by.items():
        C = [s for s in plan.segments if s["seq"] == seq][0]["n_chunks"]
        assert sorted(chunks) == sorted([min(chunks), C - 1 - min(chunks)])
    # within a round no query run and no key run appears twice; over the rounds every causal chunk pair appears once
    seen = set()
    for arr, n in plan.rounds:
        qs = [(arr[i].q_tok0, arr[i].q_len) for i in range(n) if arr[i].q_len]
        ks = [(arr[i].k_tok0, arr[i].k_len) for i in range(n) if arr[i].k_len]
        assert len(set(qs)) == len(qs) and len(set(ks)) == len(ks)
        for i in range(n):
            key = (arr[i].q_tok0, arr[i].k_tok0, arr[i].q_pos0, arr[i].k_pos0)
            assert key not in seen and arr[i].k_pos0 <= arr[i].q_pos0
            seen.add(key)
    n_ring = {}
    for s in plan.segments:
        if s["n_chunks"] > 1:
            n_ring[s["seq"]] = s["n_chunks"]
    assert len(seen) == sum(C * (C + 1) // 2 for C in n_ring.values())
