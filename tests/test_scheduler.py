"""Dual-balanced scheduler (paper: Alg. 1).  First the plain-Python statement of the algorithm is pinned to
what the paper and arithmetic fix (WaterFill's stated objective by exhaustive search, token-by-token filling,
hand-traced placements, conservation and capacity invariants); then the C++ library is compared with it,
bit for bit, on random clusters.  Host only."""
import ctypes
import itertools
import os
import re

import numpy as np
import pytest

import paper_2605_21100_amd as nanocp
from oracle import scheduler as ref

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


# ---------------------------------------------------------------- pins of the plain-Python statement

def _compositions(total, parts):
    if parts == 1:
        yield (total,)
        return
    for first in range(total + 1):
        for rest in _compositions(total - first, parts - 1):
            yield (first,) + rest


@pytest.mark.parametrize("loads,length", [([0], 5), ([3, 3], 4), ([5, 1, 3], 6), ([5, 1, 3], 0), ([2, 9, 4, 4], 7),
                                          ([7, 0, 0], 1), ([1, 2, 3, 4], 9), ([10, 0], 3)])
def test_water_fill_attains_the_minimal_peak(loads, length):
    """WaterFill: sum(split) = l_r and the peak post-allocation load is minimal (objective as stated in the paper)."""
    split = ref.water_fill(loads, length)
    assert sum(split) == length and min(split) >= 0
    best = min(max(k + t for k, t in zip(loads, c)) for c in _compositions(length, len(loads)))
    assert max(k + t for k, t in zip(loads, split)) == best


@pytest.mark.parametrize("seed", range(5))
def test_water_fill_equals_token_by_token_filling(seed):
    """'distributes tokens to lower-loaded instances first': one token at a time to the least-loaded participant."""
    rng = np.random.default_rng(seed)
    loads = rng.integers(0, 30, size=int(rng.integers(1, 7))).tolist()
    length = int(rng.integers(0, 80))
    cur, greedy = list(loads), [0] * len(loads)
    for _ in range(length):
        i = min(range(len(cur)), key=lambda j: (cur[j], j))
        cur[i] += 1
        greedy[i] += 1
    assert ref.water_fill(loads, length) == greedy


def test_water_fill_hand_case():
    # loads 5,1,3 and 6 tokens: 2 tokens lift the second to 3, the next 4 lift second and third to 5
    assert ref.water_fill([5, 1, 3], 6) == [0, 4, 2]
    assert ref.water_fill([5, 1, 3], 7) == [1, 4, 2]             # remainder to the lowest index at the level
    assert ref.water_fill([4, 4], 3) == [2, 1]


def test_rebalance_hand_case():
    # singleton requests are bound first (they have no choice); the flexible one then avoids the crowded instance
    P = [[0, 1], [0], [0], [1, 2, 3]]
    m, B = ref.rebalance(4, P)
    assert m[1] == 0 and m[2] == 0 and m[0] == 1 and m[3] == 2      # r3: B = [2,1,0,0] -> instance 2
    assert B == [2, 1, 1, 0]
    assert all(m[r] in P[r] for r in range(len(P)))


def test_place_hand_traced():
    # 2 nodes x 2 instances, Bucket: <=10 tokens -> 1, else 2;  K = [0, 8, 2, 2], B = [1, 0, 0, 0], K_max = 20
    nodes = [[0, 1], [2, 3]]
    K, B = [0, 8, 2, 2], [1, 0, 0, 0]
    out = ref.place(nodes, K, B, 20, [10, 10 ** 9], [1, 2], [6, 12, 30])
    # r0 (6 tok): node 1 (B^(1)=0 < 1); k=1; m=2; split [6]            -> K=[0,8,8,2] B=[1,0,1,0]
    assert out[0] == {"scheduled": True, "node": 1, "m": 2, "P": [2], "split": [6]}
    # r1 (12 tok): node loads 1,1 -> node 0; k=2; m = instance 1 (B=0); other = 0; WaterFill(K=[8,0],12) -> level 10: [2,10]
    assert out[1] == {"scheduled": True, "node": 0, "m": 1, "P": [1, 0], "split": [2, 10]}
    # r2 (30 tok): node loads 2,1 -> node 1; m=3; P=[3,2]; K=[2,8]: level 20 -> [18,12]; 20 <= K_max -> fits
    assert out[2] == {"scheduled": True, "node": 1, "m": 3, "P": [3, 2], "split": [18, 12]}
    assert K == [10, 10, 20, 20] and B == [1, 1, 1, 1]
    # a request that cannot fit is left in the queue and changes nothing
    out2 = ref.place(nodes, K, B, 20, [10, 10 ** 9], [1, 2], [25])
    assert out2[0]["scheduled"] is False and K == [10, 10, 20, 20] and B == [1, 1, 1, 1]


def test_place_invariants_random():
    rng = np.random.default_rng(11)
    for _ in range(20):
        per_node = rng.integers(1, 9, size=int(rng.integers(1, 5))).tolist()
        nodes, s = [], 0
        for c in per_node:
            nodes.append(list(range(s, s + c)))
            s += c
        K0 = rng.integers(0, 5000, size=s).tolist()
        B0 = rng.integers(0, 5, size=s).tolist()
        K, B = list(K0), list(B0)
        lengths = rng.integers(1, 20000, size=30).tolist()
        out = ref.place(nodes, K, B, 12000, [1000, 4000, 10 ** 9], [1, 2, 8], lengths)
        addK, addB = [0] * s, [0] * s
        for d, L in zip(out, lengths):
            assert sum(d["split"]) == L and d["m"] == d["P"][0] and len(set(d["P"])) == len(d["P"])
            assert set(d["P"]) <= set(nodes[d["node"]])
            assert len(d["P"]) == min(ref.bucket_degree([1000, 4000, 10 ** 9], [1, 2, 8], L), len(nodes[d["node"]]))
            if d["scheduled"]:
                for p, t in zip(d["P"], d["split"]):
                    addK[p] += t
                addB[d["m"]] += 1
        assert K == [a + b for a, b in zip(K0, addK)] and B == [a + b for a, b in zip(B0, addB)]
        assert max(K) <= max(12000, max(K0))


# ---------------------------------------------------------------- the C++ library against the statement

def test_sched_symbols_exported():
    hdr = open(os.path.join(ROOT, "include", "nanocp_sched.h")).read()
    declared = sorted(set(re.findall(r"\b(nanocp_sched_[a-z_]+)\s*\(", hdr)))
    assert set(declared) == set(nanocp.SCHED_EXPORTS)
    lib = ctypes.CDLL(nanocp.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name)
    assert ctypes.sizeof(nanocp.SchedDecision) == 16 + 32 + 64


@pytest.mark.parametrize("seed", range(8))
def test_library_matches_statement(seed):
    rng = np.random.default_rng(100 + seed)
    per_node = rng.integers(1, 9, size=int(rng.integers(1, 6))).tolist()
    nodes, s = [], 0
    for c in per_node:
        nodes.append(list(range(s, s + c)))
        s += c
    blen, bdeg = [2048, 32768, 65536, 10 ** 12], [1, 2, 4, 8]
    kmax = int(rng.integers(50_000, 400_000))
    sch = nanocp.Scheduler(per_node, kmax, blen, bdeg)
    # active requests with participant sets inside one node
    active = []
    for _ in range(int(rng.integers(0, 200))):
        n = int(rng.integers(0, len(nodes)))
        k = int(rng.integers(1, len(nodes[n]) + 1))
        active.append(sorted(rng.choice(nodes[n], size=k, replace=False).tolist()))
    m_lib = sch.rebalance(active)
    m_ref, B_ref = ref.rebalance(s, active)
    assert m_lib.tolist() == m_ref and sch.moe_load.tolist() == B_ref
    K = rng.integers(0, kmax // 2, size=s).tolist()
    sch.kv_load[:] = K
    B = list(B_ref)
    lengths = np.clip(np.rint(np.exp(rng.normal(np.log(2048), 1.6, 300))), 16, 1_048_576).astype(np.int64).tolist()
    out_lib = sch.place(lengths)
    out_ref = ref.place(nodes, K, B, kmax, blen, bdeg, lengths)
    assert out_lib == out_ref
    assert sch.kv_load.tolist() == K and sch.moe_load.tolist() == B
    for L in [0, 1, 17, 99999]:
        loads = rng.integers(0, 1000, size=int(rng.integers(1, 9))).tolist()
        assert nanocp.nanocp_sched_water_fill(loads, L) == ref.water_fill(loads, L)


def test_sched_argument_errors():
    with pytest.raises(nanocp.NanocpError) as e:
        nanocp.Scheduler([2, 2], 100, [10, 5], [1, 2]).place([3])             # bucket bounds not increasing
    assert e.value.status == nanocp.EINVAL
    with pytest.raises(nanocp.NanocpError) as e:
        nanocp.Scheduler([2, 2], 100, [10], [9]).place([3])                   # degree beyond the CP cap
    assert e.value.status == nanocp.EINVAL
    with pytest.raises(nanocp.NanocpError) as e:
        nanocp.Scheduler([2, 2], 100, [10], [1]).rebalance([[0, 7]])          # instance id out of range
    assert e.value.status == nanocp.EBOUNDS
    with pytest.raises(nanocp.NanocpError) as e:
        nanocp.Scheduler([2, 2], 100, [10], [1]).place([-4])
    assert e.value.status == nanocp.EINVAL


def test_micro_benchmark_split_is_what_the_scheduler_gives():
    """Workload 6 hands each GPU an even 1/8 slice of every long request; that is the scheduler's own split
    for the paper's micro-benchmark node (8 instances, each holding 64 x 2048 short tokens)."""
    import workloads as W
    sch = nanocp.Scheduler([8], 10 ** 9, [32768, 10 ** 12], [1, 8])
    sch.kv_load[:] = 64 * 2048
    out = sch.place([524288] * 3)
    for d in out:
        assert d["scheduled"] and sorted(d["P"]) == list(range(8)) and d["split"] == [65536] * 8
    assert [e - b for b, e in W.even_split(524288, 8)] == [65536] * 8
