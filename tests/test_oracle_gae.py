"""Pins for the oracle's generalized advantage estimation (the PPO counterpart of the
group-relative advantage; Sec. 7.1 evaluates PPO with a critic, the estimator itself is
Schulman et al. 2016, arXiv 1506.02438, eqs. 11-16): closed forms, the estimator written as
the explicit double sum of eq. 16, special cases, a hand-worked example, and the rule that
tokens without loss are transparent."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "gae_hand_example.txt")


def one_seq(values, reward, gamma, lam, mask=None, kl_coef=0.0, logp=None, ref=None):
    v = np.asarray(values, np.float32)
    L = len(v)
    m = np.ones(L, np.uint8) if mask is None else np.asarray(mask, np.uint8)
    adv, ret = oracle.gae(np.array([reward], np.float32), [L], [0], [0, 1], [L], [v], [m], gamma, lam, kl_coef,
                          None if logp is None else [np.asarray(logp, np.float32)],
                          None if ref is None else [np.asarray(ref, np.float32)])
    return adv[0], ret[0]


def test_hand_worked_example():
    """tests/golden/gae_hand_example.txt: V = (1, 2, 3), score 10, gamma = lambda = 1/2, worked by hand."""
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    vals = {r[0]: [float(x) for x in r[1:]] for r in rows}
    adv, ret = one_seq(vals["V"], vals["score"][0], vals["gamma"][0], vals["lambda"][0])
    assert adv.tolist() == vals["A"]          # all values are exact in binary floating point
    assert ret.tolist() == vals["ret"]


def test_lambda_one_gamma_one_gives_the_score_as_every_return():
    """lambda = gamma = 1: A_t = (sum of later rewards) - V_t, so ret_t = score for every t."""
    rng = np.random.default_rng(3)
    v = rng.normal(size=257)
    adv, ret = one_seq(v, 2.5, 1.0, 1.0)
    np.testing.assert_allclose(ret, 2.5, rtol=1e-6)
    np.testing.assert_allclose(adv, 2.5 - v.astype(np.float32).astype(np.float64), rtol=1e-6, atol=1e-6)


def test_lambda_zero_is_the_td_residual():
    """lambda = 0: A_t = delta_t = r_t + gamma V_{t+1} - V_t (eq. 17)."""
    rng = np.random.default_rng(4)
    v = rng.normal(size=100).astype(np.float32).astype(np.float64)
    adv, ret = one_seq(v, -1.25, 0.9, 0.0)
    nxt = np.append(v[1:], 0.0)
    r = np.zeros(100); r[-1] = -1.25
    np.testing.assert_allclose(adv, r + 0.9 * nxt - v, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(ret, r + 0.9 * nxt, rtol=1e-6, atol=1e-7)


def test_zero_values_give_a_geometric_tail():
    """V = 0: delta_t = r_t, A_t = (gamma lambda)^(L-1-t) * score."""
    L, g, lam = 64, 0.99, 0.95
    adv, ret = one_seq(np.zeros(L), 3.0, g, lam)
    want = 3.0 * (g * lam) ** (L - 1 - np.arange(L))
    np.testing.assert_allclose(adv, want, rtol=2e-7)
    np.testing.assert_array_equal(adv, ret)


def test_constant_values_gamma_one():
    """V = v everywhere, gamma = 1: every residual but the last vanishes, A_t = lambda^(L-1-t) (score - v)."""
    L, lam, v, R = 50, 0.9, 0.75, 2.0
    adv, _ = one_seq(np.full(L, v), R, 1.0, lam)
    np.testing.assert_allclose(adv, lam ** (L - 1 - np.arange(L)) * (R - v), rtol=1e-6)


def test_explicit_double_sum_with_kl_penalty():
    """Eq. 16 written out: A_t = sum_l (gamma lambda)^l delta_{t+l}; rewards carry the KL penalty."""
    rng = np.random.default_rng(5)
    for L in (1, 2, 7, 40):
        v = rng.normal(size=L).astype(np.float32).astype(np.float64)
        lp = (-np.abs(rng.normal(size=L))).astype(np.float32).astype(np.float64)
        rf = (-np.abs(rng.normal(size=L))).astype(np.float32).astype(np.float64)
        g, lam, beta, R = 0.97, 0.8, 0.05, 1.5
        adv, ret = one_seq(v, R, g, lam, kl_coef=beta, logp=lp, ref=rf)
        r = -beta * (lp - rf)
        r[-1] += R
        delta = r + g * np.append(v[1:], 0.0) - v
        want = np.array([sum((g * lam) ** l * delta[t + l] for l in range(L - t)) for t in range(L)])
        np.testing.assert_allclose(adv, want, rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(ret, want + v, rtol=1e-6, atol=1e-7)


def test_tokens_without_loss_are_transparent():
    """Inserting masked tokens changes nothing at the loss-bearing ones and yields +0 at the inserted ones."""
    rng = np.random.default_rng(6)
    L = 300
    v = rng.normal(size=L).astype(np.float32)
    m = (rng.random(L) < 0.6).astype(np.uint8)
    m[:40] = 0                                     # a prompt
    m[-5:] = 0                                     # the score must land on the last loss-bearing token, not the last token
    adv, ret = one_seq(v, 0.7, 0.98, 0.9, mask=m)
    keep = m != 0
    adv_c, ret_c = one_seq(v[keep], 0.7, 0.98, 0.9)
    np.testing.assert_array_equal(adv[keep], adv_c)
    np.testing.assert_array_equal(ret[keep], ret_c)
    assert not adv[~keep].any() and not ret[~keep].any()
    assert not np.signbit(adv[~keep]).any()


def test_all_masked_sequence_and_sequence_independence():
    rng = np.random.default_rng(7)
    lens = np.array([5, 1, 33, 8], np.int32)
    off = np.array([0, 5, 6, 39], np.int64)
    v = rng.normal(size=47).astype(np.float32)
    m = np.ones(47, np.uint8)
    m[5:6] = 0                                     # sequence 1 has no loss-bearing token at all
    R = np.array([1.0, 9.0, -2.0, 0.5], np.float32)
    adv, ret = oracle.gae(R, lens, off, [0, 4], [47], [v], [m], 0.95, 0.9)
    assert adv[0][5] == 0 and ret[0][5] == 0
    for i in (0, 2, 3):
        a, r_ = one_seq(v[off[i]:off[i] + lens[i]], R[i], 0.95, 0.9)
        np.testing.assert_array_equal(adv[0][off[i]:off[i] + lens[i]], a)
        np.testing.assert_array_equal(ret[0][off[i]:off[i] + lens[i]], r_)


def test_two_rollout_shards_and_padded_rows():
    """Offsets restart in every rollout shard; elements between sequences are left alone (0 from allocation)."""
    rng = np.random.default_rng(8)
    lens = np.array([4, 6, 3, 5], np.int32)
    off = np.array([2, 10, 0, 7], np.int64)        # shard 0: seqs 0, 1 in 20 elements; shard 1: seqs 2, 3 in 16
    vs = [rng.normal(size=20).astype(np.float32), rng.normal(size=16).astype(np.float32)]
    ms = [np.ones(20, np.uint8), np.ones(16, np.uint8)]
    R = np.array([1, 2, 3, 4], np.float32)
    adv, ret = oracle.gae(R, lens, off, [0, 2, 4], [20, 16], vs, ms, 1.0, 1.0)
    for i, s in ((0, 0), (1, 0), (2, 1), (3, 1)):
        np.testing.assert_allclose(ret[s][off[i]:off[i] + lens[i]], R[i], rtol=1e-6)
    used = np.zeros(20, bool); used[2:6] = True; used[10:16] = True
    assert not adv[0][~used].any()


def test_kl_needs_both_logprob_fields():
    with pytest.raises(oracle.OracleError):
        one_seq([0.0, 1.0], 1.0, 1.0, 1.0, kl_coef=0.1)
