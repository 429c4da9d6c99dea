"""Pins for the oracle's packed-layout plan and gather (Sec. 6 "Distributed Databuffer":
re-partitioning of stage outputs when the DP size changes)."""
import numpy as np
import pytest

import oracle
from paper_2507_13833_amd import workloads


def rederive_plan(S, perm, shard_seq_off, budget, align):
    """Second derivation, array-style: prefix sums + a search for each micro-batch end
    (the oracle walks slot by slot with a running counter)."""
    S = np.asarray(S, np.int64)
    K = len(shard_seq_off) - 1
    dst = np.zeros(len(S) + 1, np.int64)
    shard_tok = [0]
    mbs = []                                             # (first slot, end slot)
    shard_mb = [0]
    for p in range(K):
        a, b = int(shard_seq_off[p]), int(shard_seq_off[p + 1])
        lens = S[perm[a:b]]
        cs = np.concatenate([[0], np.cumsum(lens)])
        dst[a:b] = shard_tok[-1] + cs[:-1]
        j = 0
        while j < b - a:
            # largest e with cs[e] - cs[j] <= budget
            e = int(np.searchsorted(cs, cs[j] + budget, side="right")) - 1
            assert e > j
            mbs.append((a + j, a + e))
            j = e
        shard_mb.append(len(mbs))
        end = shard_tok[-1] + int(cs[-1])
        shard_tok.append(-(-end // align) * align)
    dst[len(S)] = shard_tok[-1]
    cu = []
    for (a, e) in mbs:
        cu.extend(np.concatenate([[0], np.cumsum(S[perm[a:e]])]).tolist())
    mb_seq_off = [a for a, _ in mbs] + [len(S)]
    return dst, shard_tok, shard_mb, mb_seq_off, cu


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("align", [1, 64])
def test_plan_matches_rederivation(cfg, align):
    w = workloads.make_workload(cfg, prompts={1: 64, 2: 64, 3: 96, 4: 96, 5: 128}[cfg])
    b = oracle.balance(w.seq_len, w.n_shards)
    p = oracle.plan(w.seq_len, b.perm, b.shard_seq_off, w.token_budget, align)
    dst, shard_tok, shard_mb, mb_seq_off, cu = rederive_plan(w.seq_len, b.perm, b.shard_seq_off,
                                                              w.token_budget, align)
    assert p.dst_tok_off.tolist() == dst.tolist()
    assert p.shard_tok_off.tolist() == shard_tok
    assert p.shard_mb_off.tolist() == shard_mb
    assert p.mb_seq_off.tolist() == mb_seq_off
    assert p.cu_seqlens.tolist() == cu
    assert p.n_mb == len(mb_seq_off) - 1


def test_plan_hand_example():
    # two shards, budget 10, align 4; slots: shard 0 = lens 6,4,3 ; shard 1 = lens 9,2
    S = np.array([4, 9, 6, 2, 3], np.int32)
    perm = np.array([2, 0, 4, 1, 3], np.int32)
    p = oracle.plan(S, perm, [0, 3, 5], 10, 4)
    # shard 0: tokens 0..12, micro-batches {6,4} and {3}; rounded up to 16
    # shard 1: tokens 16..26, micro-batches {9} (9+2 > 10) and {2}; rounded up to 28
    assert p.dst_tok_off.tolist() == [0, 6, 10, 16, 25, 28]
    assert p.shard_tok_off.tolist() == [0, 16, 28]
    assert p.shard_mb_off.tolist() == [0, 2, 4]
    assert p.mb_seq_off.tolist() == [0, 2, 3, 4, 5]
    assert p.cu_seqlens.tolist() == [0, 6, 10, 0, 3, 0, 9, 0, 2]
    assert p.n_mb == 4


def test_next_fit_properties():
    for cfg in (1, 2, 3, 5):
        w = workloads.make_workload(cfg, prompts=128)
        b = oracle.balance(w.seq_len, w.n_shards)
        p = oracle.plan(w.seq_len, b.perm, b.shard_seq_off, w.token_budget)
        lens = w.seq_len[b.perm].astype(np.int64)
        tot = np.array([lens[p.mb_seq_off[m]:p.mb_seq_off[m + 1]].sum() for m in range(p.n_mb)])
        assert np.all(tot <= w.token_budget) and np.all(tot > 0)
        for k in range(w.n_shards):
            m0, m1 = p.shard_mb_off[k], p.shard_mb_off[k + 1]
            assert p.mb_seq_off[m0] == b.shard_seq_off[k]          # never spans shards
            assert tot[m0:m1].sum() == b.shard_load[k]
            # next-fit: the slot that opened micro-batch m+1 did not fit into m
            for m in range(m0, m1 - 1):
                assert tot[m] + lens[p.mb_seq_off[m + 1]] > w.token_budget
        for m in range(p.n_mb):
            a, e = p.mb_seq_off[m], p.mb_seq_off[m + 1]
            sl = p.cu_seqlens[a + m: e + m + 1]
            assert sl[0] == 0 and sl[-1] == tot[m]
            assert np.array_equal(np.diff(sl), lens[a:e])
        assert len(p.cu_seqlens) == w.n_seq + p.n_mb


def test_plan_errors():
    with pytest.raises(oracle.OracleError) as e:
        oracle.plan([5, 11], [0, 1], [0, 2], 10)
    assert e.value.code == 3


def _token_index_fields(w):
    """int32 field whose value is the global source token index."""
    base = np.concatenate([[0], np.cumsum(w.src_shard_tokens)])
    return [np.arange(base[s], base[s + 1], dtype=np.int32) for s in range(w.n_src_shards)]


@pytest.mark.parametrize("cfg", [1, 2, 4, 5])
@pytest.mark.parametrize("align", [1, 16])
def test_every_token_exactly_once_and_inverse(cfg, align):
    w = workloads.make_workload(cfg, prompts=64)
    b = oracle.balance(w.seq_len, w.n_shards)
    p = oracle.plan(w.seq_len, b.perm, b.shard_seq_off, w.token_budget, align)
    T = w.total_tokens
    arena = int(p.shard_tok_off[-1])
    SENT = -7
    out = oracle.gather(w.seq_len, b.perm, w.src_tok_off, w.src_shard_seq_off, _token_index_fields(w),
                        p.dst_tok_off, arena, fill=SENT)
    valid = np.zeros(arena, bool)
    for k in range(w.n_shards):
        valid[p.shard_tok_off[k]: p.shard_tok_off[k] + b.shard_load[k]] = True
    assert not np.any(out[valid] == SENT)
    assert np.all(out[~valid] == SENT)                     # padding is never written
    assert np.array_equal(np.sort(out[valid]), np.arange(T, dtype=np.int32))
    # each slot holds its sequence's consecutive source tokens
    base = np.concatenate([[0], np.cumsum(w.src_shard_tokens)])
    shard_of = np.searchsorted(w.src_shard_seq_off, np.arange(w.n_seq), side="right") - 1
    for j in np.random.default_rng(0).integers(0, w.n_seq, 50):
        i = b.perm[j]
        g0 = base[shard_of[i]] + w.src_tok_off[i]
        seg = out[p.dst_tok_off[j]: p.dst_tok_off[j] + w.seq_len[i]]
        assert np.array_equal(seg, np.arange(g0, g0 + w.seq_len[i], dtype=np.int32))
    # scatter back through the plan reproduces every payload field bit for bit
    for f in w.fields:
        o = oracle.gather(w.seq_len, b.perm, w.src_tok_off, w.src_shard_seq_off, f.shards, p.dst_tok_off, arena)
        back = np.concatenate(f.shards).copy()
        back[:] = 0
        back[out[valid]] = o[valid]
        assert np.array_equal(back, np.concatenate(f.shards))


def test_identity_case():
    # one shard, lengths already descending: the packed output is the input
    rng = np.random.default_rng(2)
    S = np.sort(rng.integers(1, 50, 40).astype(np.int32))[::-1].copy()
    b = oracle.balance(S, 1)
    assert b.perm.tolist() == list(range(40))
    off = np.concatenate([[0], np.cumsum(S)]).astype(np.int64)
    p = oracle.plan(S, b.perm, b.shard_seq_off, 1000)
    assert p.dst_tok_off.tolist() == off.tolist()
    for dt in (np.uint8, np.uint16, np.float32):
        x = rng.integers(0, 250, int(off[-1])).astype(dt)
        o = oracle.gather(S, b.perm, off[:-1], [0, 40], [x], p.dst_tok_off, int(off[-1]))
        assert np.array_equal(o, x)


def test_gather_preserves_nan_payload_bits():
    S = np.array([2, 3], np.int32)
    bits = np.array([0x7FC00001, 0x80000000, 0xFFC12345, 0x7F800000, 0x00000001], np.uint32)
    x = bits.view(np.float32)
    o = oracle.gather(S, [1, 0], [0, 2], [0, 2], [x], [0, 3, 5], 5)
    assert o.view(np.uint32).tolist() == [0xFFC12345, 0x7F800000, 0x00000001, 0x7FC00001, 0x80000000]


# ---------------------------------------------------------------- reverse path (scatter)
def _scatter_case(seed, n=60, K=4, n_src=3, pad=7):
    """Small rollout batch with gaps between sequences (padded rows) in several rollout shards."""
    rng = np.random.default_rng(seed)
    n = n // (K * n_src) * (K * n_src)
    S = rng.integers(1, 40, n).astype(np.int32)
    per = n // n_src
    sso = (np.arange(n_src + 1) * per).astype(np.int32)
    sto = np.zeros(n, np.int64)
    stk = np.zeros(n_src, np.int64)
    for s in range(n_src):
        pos = int(rng.integers(0, pad))
        for i in range(sso[s], sso[s + 1]):
            sto[i] = pos
            pos += int(S[i]) + int(rng.integers(0, pad))
        stk[s] = pos
    bal = oracle.balance(S, K)
    pl = oracle.plan(S, bal.perm, bal.shard_seq_off, 100)
    return S, sso, sto, stk, bal, pl


@pytest.mark.parametrize("dtype", [np.uint8, np.uint16, np.int32])
def test_scatter_undoes_gather(dtype):
    S, sso, sto, stk, bal, pl = _scatter_case(3)
    rng = np.random.default_rng(5)
    src = [rng.integers(1, 200, int(t)).astype(dtype) for t in stk]
    arena = oracle.gather(S, bal.perm, sto, sso, src, pl.dst_tok_off, int(pl.shard_tok_off[-1]))
    blank = [np.full(int(t), 255, dtype) for t in stk]
    back = oracle.scatter(S, bal.perm, sto, sso, arena, pl.dst_tok_off, blank)
    for s in range(len(stk)):
        valid = np.zeros(int(stk[s]), bool)
        for i in range(sso[s], sso[s + 1]):
            valid[sto[i]: sto[i] + S[i]] = True
        assert np.array_equal(back[s][valid], src[s][valid])       # every token back where it came from
        assert np.all(back[s][~valid] == 255)                      # gaps between sequences untouched


def test_scatter_against_index_formulation():
    # independent formulation: build the token-level map arena index -> (shard, rollout index) with
    # NumPy and apply it with fancy indexing
    S, sso, sto, stk, bal, pl = _scatter_case(9, n=96, K=8, n_src=2)
    T = int(pl.shard_tok_off[-1])
    arena = np.arange(T, dtype=np.int32) * 3 + 1
    blank = [np.full(int(t), -1, np.int32) for t in stk]
    got = oracle.scatter(S, bal.perm, sto, sso, arena, pl.dst_tok_off, blank)
    want = [b.copy() for b in blank]
    shard_of = np.searchsorted(sso, np.arange(len(S)), side="right") - 1
    for j, i in enumerate(bal.perm):
        idx = np.arange(S[i])
        want[shard_of[i]][sto[i] + idx] = arena[pl.dst_tok_off[j] + idx]
    for a, b in zip(got, want):
        assert np.array_equal(a, b)


def test_scatter_hand_example():
    # S = [2, 3], one shard, perm = [1, 0] (longest first): arena = [b0 b1 b2 | a0 a1]
    S = np.array([2, 3], np.int32)
    arena = np.array([10, 11, 12, 20, 21], np.int32)
    out = oracle.scatter(S, [1, 0], [1, 4], [0, 2], arena, [0, 3, 5], [np.zeros(8, np.int32)])[0]
    assert out.tolist() == [0, 20, 21, 0, 10, 11, 12, 0]


def test_gather_by_slot_ranges_equals_gather():
    """gather_slots over disjoint slot ranges (what the benchmark's threaded CPU leg calls) fills
    the same arena as one gather call."""
    w = workloads.make_workload(1)
    bal = oracle.balance(w.seq_len, w.n_shards)
    pl = oracle.plan(w.seq_len, bal.perm, bal.shard_seq_off, w.token_budget)
    arena = int(pl.shard_tok_off[-1])
    for f in w.fields:
        want = oracle.gather(w.seq_len, bal.perm, w.src_tok_off, w.src_shard_seq_off, f.shards, pl.dst_tok_off, arena)
        got = np.zeros(arena, want.dtype)
        cuts = [0, 1, 7, w.n_seq // 2, w.n_seq]
        for a, b in zip(cuts[:-1], cuts[1:]):
            oracle.gather_slots(w.seq_len, bal.perm, w.src_tok_off, w.src_shard_seq_off, f.shards, pl.dst_tok_off,
                                got, a, b)
        assert np.array_equal(got, want), f.name
