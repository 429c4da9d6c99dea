"""Pins for the oracle's Algorithm 1 (Constrained LPT Load Balancing, Sec. 6).

None of these re-types the oracle's loop (a scan over the workers per item): they check it
against hand traces, exhaustive search, an independent formulation with a priority queue from
which full workers are taken out and put back (the library's heapq), Graham's theorem for the
unconstrained special case and structural invariants.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from paper_2507_13833_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "lpt_worked_examples.txt")


def members(b: oracle.Balance):
    return [b.perm[b.shard_seq_off[k]:b.shard_seq_off[k + 1]].tolist() for k in range(len(b.shard_load))]


def test_hand_traces():
    n = 0
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        parts = [p.strip() for p in line.split("|")]
        S = [int(x) for x in parts[0].split(",")]
        K = int(parts[1])
        want = [[int(x) for x in grp.split(",")] for grp in parts[2].split(";")]
        loads = [int(x) for x in parts[3].split(",")]
        cap = int(parts[4].split("=")[1]) if len(parts) > 4 else 0
        b = oracle.balance(S, K, cap)
        assert members(b) == want, line
        assert b.shard_load.tolist() == loads, line
        n += 1
    assert n >= 4


def queue_lpt(S, K, C):
    """Independent formulation: a priority queue of (load, k) pairs (the library's binary heap).
    The smallest pair is taken out until it belongs to a worker that is not full; that worker
    takes the item and goes back with its new load, and so do the full ones taken out on the
    way.  Selects the lexicographically smallest (load, k) among the workers that are not full."""
    import heapq
    order = sorted(range(len(S)), key=lambda i: (-S[i], i))
    queue = [(0, k) for k in range(K)]
    heapq.heapify(queue)
    mem = [[] for _ in range(K)]
    for u in order:
        aside = []
        while True:
            load, k = heapq.heappop(queue)
            if len(mem[k]) < C:
                break
            aside.append((load, k))
        mem[k].append(u)
        heapq.heappush(queue, (load + S[u], k))
        for x in aside:
            heapq.heappush(queue, x)
    return mem, [sum(S[u] for u in m) for m in mem]


@pytest.mark.parametrize("seed", range(6))
def test_scan_equals_priority_queue(seed):
    rng = np.random.default_rng(seed)
    for _ in range(150):
        K = int(rng.integers(1, 9))
        C = int(rng.integers(1, 9))
        hi = int(rng.choice([3, 10, 1000]))            # small ranges force many ties
        S = rng.integers(1, hi + 1, K * C).tolist()
        b = oracle.balance(S, K)
        mem, load = queue_lpt(S, K, C)
        assert members(b) == mem
        assert b.shard_load.tolist() == load
        # textbook LPT: constraint vacuous
        b2 = oracle.balance(S, K, cap=len(S))
        mem2, load2 = queue_lpt(S, K, len(S))
        assert members(b2) == mem2 and b2.shard_load.tolist() == load2


def opt_makespan(S, K, C=None):
    """Exhaustive optimum makespan (optionally with exactly C items per worker)."""
    S = sorted(S, reverse=True)
    best = [sum(S)]
    load = [0] * K
    cnt = [0] * K

    def rec(i):
        if i == len(S):
            best[0] = min(best[0], max(load))
            return
        seen = set()
        for k in range(K):
            if C is not None and cnt[k] >= C:
                continue
            key = (load[k], cnt[k])
            if key in seen:                             # symmetric workers
                continue
            seen.add(key)
            if load[k] + S[i] >= best[0]:
                continue
            load[k] += S[i]; cnt[k] += 1
            rec(i + 1)
            load[k] -= S[i]; cnt[k] -= 1

    rec(0)
    return best[0]


def test_opt_bruteforce_is_a_bruteforce():
    # the pruned search agrees with plain enumeration on a tiny case
    S = [7, 5, 4, 4, 3, 2]
    K = 3
    plain = min(max(sum(S[i] for i in range(6) if a[i] == k) for k in range(K))
                for a in itertools.product(range(K), repeat=6))
    assert opt_makespan(S, K) == plain
    plainc = min(max(sum(S[i] for i in range(6) if a[i] == k) for k in range(K))
                 for a in itertools.product(range(K), repeat=6)
                 if all(a.count(k) == 2 for k in range(K)))
    assert opt_makespan(S, K, 2) == plainc


@pytest.mark.parametrize("K,N", [(2, 8), (2, 12), (3, 9), (3, 12), (4, 12), (6, 12)])
def test_graham_bound_unconstrained(K, N):
    """cap = N: Algorithm 1 is textbook LPT, so makespan <= (4/3 - 1/(3K)) OPT (Graham 1969)."""
    rng = np.random.default_rng(100 * K + N)
    for _ in range(40):
        hi = int(rng.choice([4, 20, 200]))
        S = rng.integers(1, hi + 1, N).tolist()
        b = oracle.balance(S, K, cap=N)
        opt = opt_makespan(S, K)
        assert int(b.shard_load.max()) * 3 * K <= (4 * K - 1) * opt
        assert int(b.shard_load.max()) >= opt


@pytest.mark.parametrize("K,N", [(2, 8), (2, 12), (3, 9), (3, 12), (4, 12)])
def test_constrained_vs_constrained_opt(K, N):
    """cap = N/K: exactly C per worker; compared with the optimum under the SAME constraint
    (the constrained heuristic can exceed the unconstrained optimum's Graham bound)."""
    rng = np.random.default_rng(7 * K + N)
    for _ in range(40):
        hi = int(rng.choice([4, 20, 200]))
        S = rng.integers(1, hi + 1, N).tolist()
        b = oracle.balance(S, K)
        assert np.diff(b.shard_seq_off).tolist() == [N // K] * K
        opt = opt_makespan(S, K, N // K)
        ms = int(b.shard_load.max())
        assert ms >= opt
        assert ms * 3 * K <= (4 * K - 1) * opt


def test_constraint_changes_the_answer():
    # constrained LPT against the unconstrained optimum breaks Graham's ratio (K = 3)
    S = [8, 8, 13, 52, 8, 9, 8, 14, 12, 8, 10, 10]
    b = oracle.balance(S, 3)
    assert int(b.shard_load.max()) == 76
    assert opt_makespan(S, 3) == 54


def test_structure_on_all_workloads():
    for cfg in (1, 2, 3, 4, 5):
        w = workloads.make_workload(cfg, prompts={1: 64, 2: 64, 3: 64, 4: 64, 5: 128}[cfg])
        b = oracle.balance(w.seq_len, w.n_shards)
        N, K = w.n_seq, w.n_shards
        assert sorted(b.perm.tolist()) == list(range(N))
        assert np.diff(b.shard_seq_off).tolist() == [N // K] * K
        assert int(b.shard_load.sum()) == int(w.seq_len.astype(np.int64).sum())
        for k in range(K):
            m = b.perm[b.shard_seq_off[k]:b.shard_seq_off[k + 1]]
            assert np.all(b.shard_of_seq[m] == k)
            assert int(w.seq_len[m].astype(np.int64).sum()) == int(b.shard_load[k])
            # insertion order = descending length, ties by index
            keys = list(zip((-w.seq_len[m]).tolist(), m.tolist()))
            assert keys == sorted(keys)
        assert b.shard_load.max() <= b.shard_load.mean() * 1.25


def test_errors():
    with pytest.raises(oracle.OracleError) as e:
        oracle.balance([3, 2, 1], 2)
    assert e.value.code == 2
    with pytest.raises(oracle.OracleError) as e:
        oracle.balance([3, 0, 1, 1], 2)
    assert e.value.code == 4
    with pytest.raises(oracle.OracleError):
        oracle.balance([3, 2, 1, 1], 2, cap=1)
    b = oracle.balance([], 3)
    assert b.shard_seq_off.tolist() == [0, 0, 0, 0]
