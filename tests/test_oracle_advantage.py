"""Pins for the oracle's group-relative advantage (GRPO; the paper names the stage in
App. B Table 2 and lists advantages among the payloads in Sec. 1, the formula is the
standard one: reward minus group mean over group std plus eps)."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2507_13833_amd import workloads

EPS = 1e-6


def test_closed_form_binary_rewards():
    """k ones among G zeros/ones: mean k/G, sample variance k(G-k)/(G(G-1)),
    population variance k(G-k)/G^2."""
    for G in (2, 3, 8, 16, 33):
        for k in range(0, G + 1):
            r = np.zeros(G, np.float32)
            r[:k] = 1.0
            for ddof in (0, 1):
                a = oracle.group_advantage(r, [0, G], EPS, ddof)
                if k in (0, G):
                    assert np.all(a == 0.0)
                    continue
                var = Fraction(k * (G - k), G * (G - ddof))
                sd = math.sqrt(var)
                one = (1 - k / G) / (sd + EPS)
                zero = (0 - k / G) / (sd + EPS)
                np.testing.assert_allclose(a[:k], np.float32(one), rtol=3e-7, atol=0)
                np.testing.assert_allclose(a[k:], np.float32(zero), rtol=3e-7, atol=0)


def test_printed_value_g8_k1():
    # G=8, one success, sample std: sd = sqrt(7/56) = 0.35355339..., A(1) = 0.875/(sd+1e-6)
    r = np.array([1, 0, 0, 0, 0, 0, 0, 0], np.float32)
    a = oracle.group_advantage(r, [0, 8], EPS, 1)
    assert abs(float(a[0]) - 2.474867) < 2e-6
    assert abs(float(a[1]) + 0.353552) < 2e-6


@pytest.mark.parametrize("ddof", [0, 1])
def test_reduces_to_library_std(ddof):
    rng = np.random.default_rng(5)
    sizes = rng.integers(2, 40, 50)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    r = rng.standard_normal(int(off[-1])).astype(np.float32)
    a = oracle.group_advantage(r, off, EPS, ddof)
    for g in range(len(sizes)):
        x = r[off[g]:off[g + 1]].astype(np.float64)
        want = (x - np.mean(x)) / (np.std(x, ddof=ddof) + EPS)
        np.testing.assert_allclose(a[off[g]:off[g + 1]], want, rtol=2e-7, atol=1e-12)


def test_group_sum_zero_and_identical_groups():
    for cfg in (1, 2, 3, 4, 5):
        w = workloads.make_workload(cfg, prompts=64)
        a = oracle.group_advantage(w.reward, w.group_off, w.eps, w.ddof)
        A = a.reshape(-1, w.group_size).astype(np.float64)
        R = w.reward.reshape(-1, w.group_size)
        assert np.all(np.abs(A.sum(axis=1)) < 1e-5)
        same = np.all(R == R[:, :1], axis=1)
        assert np.all(A[same] == 0.0)
        assert np.all(np.any(A[~same] != 0.0, axis=1))
        if cfg == 4:
            assert same[np.arange(len(same)) % 8 < 3].all()
        # within a group the advantage is monotone in the reward
        for g in np.flatnonzero(~same)[:20]:
            o = np.argsort(R[g], kind="stable")
            assert np.all(np.diff(A[g][o]) >= 0)


def test_identical_rewards_any_group_size():
    # identical rewards give exactly +0 by rule, not by cancellation: with eps = 0 the formula alone is 0 / 0
    for G in (1, 2, 3, 5, 7, 10, 16, 100):
        r = np.full(G, 0.1, np.float32)
        for ddof in (0, 1):
            for eps in (EPS, 0.0):
                a = oracle.group_advantage(r, [0, G], eps, ddof)
                assert np.all(a == 0.0) and not np.any(np.signbit(a))


def test_singleton_group_and_empty_group():
    a = oracle.group_advantage(np.array([3.0, 1.0, 2.0], np.float32), [0, 1, 1, 3], EPS, 1)
    assert a[0] == 0.0
    sd = math.sqrt(0.5)
    np.testing.assert_allclose(a[1:], [-0.5 / (sd + EPS), 0.5 / (sd + EPS)], rtol=2e-7)


def test_shift_scale_invariance_and_permutation():
    rng = np.random.default_rng(11)
    G = 16
    r = rng.standard_normal(G * 30).astype(np.float32)
    # powers of two keep the transformed rewards exact in fp32
    off = np.arange(0, len(r) + 1, G, dtype=np.int32)
    a0 = oracle.group_advantage(r, off, 0.0, 1)
    a1 = oracle.group_advantage(r * np.float32(4.0), off, 0.0, 1)
    np.testing.assert_allclose(a1, a0, rtol=3e-7, atol=1e-7)
    r_small = (np.rint(r * 64) / 64).astype(np.float32)
    b0 = oracle.group_advantage(r_small, off, 0.0, 1)
    b1 = oracle.group_advantage(r_small + np.float32(8.0), off, 0.0, 1)
    np.testing.assert_allclose(b1, b0, rtol=1e-6, atol=1e-6)
    # eps shrinks magnitudes: |A_eps| < |A_0|, same sign
    ae = oracle.group_advantage(r, off, 1e-2, 1)
    assert np.all(np.abs(ae) <= np.abs(a0)) and np.all(np.sign(ae) == np.sign(a0))
    # permuting a group's members permutes its advantages
    p = rng.permutation(G)
    rp = r.reshape(-1, G)[:, p].reshape(-1).copy()
    ap = oracle.group_advantage(rp, off, EPS, 1)
    aa = oracle.group_advantage(r, off, EPS, 1)
    np.testing.assert_allclose(ap.reshape(-1, G), aa.reshape(-1, G)[:, p], rtol=1e-6, atol=1e-7)


def test_unit_sample_variance():
    # with eps = 0 the advantages of a group have sample variance exactly 1 (ddof=1)
    rng = np.random.default_rng(3)
    r = rng.random(16 * 20).astype(np.float32)
    off = np.arange(0, len(r) + 1, 16, dtype=np.int32)
    for ddof in (0, 1):
        a = oracle.group_advantage(r, off, 0.0, ddof).reshape(-1, 16).astype(np.float64)
        np.testing.assert_allclose(a.var(axis=1, ddof=ddof), 1.0, rtol=1e-5)


def test_broadcast_selects_on_mask():
    for cfg in (1, 4, 5):
        w = workloads.make_workload(cfg, prompts=16)
        a = oracle.group_advantage(w.reward, w.group_off, w.eps, w.ddof)
        mask = w.field_by_name("mask").shards
        toks = oracle.adv_broadcast(a, w.seq_len, w.src_tok_off, w.src_shard_seq_off, w.src_shard_tokens, mask)
        for s in range(w.n_src_shards):
            lo, hi = w.src_shard_seq_off[s], w.src_shard_seq_off[s + 1]
            # per-token sequence id by repetition (library routine), then select
            sid = np.repeat(np.arange(lo, hi), w.seq_len[lo:hi])
            want = np.where(mask[s] != 0, a[sid], np.float32(0.0))
            assert toks[s].dtype == np.float32
            assert np.array_equal(toks[s].view(np.uint32), want.view(np.uint32))
            # prompt tokens never carry an advantage
            first = w.src_tok_off[lo:hi]
            assert np.all(toks[s][first] == 0.0)
