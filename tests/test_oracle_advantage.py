"""Pins for the oracle's group advantages and token broadcast (CPU only).

GRPO: Sec. 3.1 (mean/std normalisation, zero when the std is zero).
RLOO: Sec. 4 / App. E (leave-one-out baseline).  Broadcast: the advantage has
no token dependence (Sec. 3.1).
"""
import numpy as np
import pytest


def random_groups(rng, n_groups, lo=1, hi=40):
    sizes = rng.integers(lo, hi + 1, n_groups)
    off = np.zeros(n_groups + 1, dtype=np.int64)
    np.cumsum(sizes, out=off[1:])
    return sizes, off


def test_grpo_binary_closed_form(oracle):
    # k ones among G rewards, eps = 0, population std:
    # A(1) = sqrt((G-k)/k), A(0) = -sqrt(k/(G-k))
    for G in (2, 3, 8, 17, 64):
        for k in range(1, G):
            r = np.zeros(G)
            r[np.random.default_rng(G * 100 + k).permutation(G)[:k]] = 1.0
            adv = oracle.group_advantage(np.array([0, G]), r, "grpo", eps=0.0)
            np.testing.assert_allclose(adv[r == 1], np.sqrt((G - k) / k), rtol=1e-14)
            np.testing.assert_allclose(adv[r == 0], -np.sqrt(k / (G - k)), rtol=1e-14)


def test_grpo_matches_numpy_standardisation(oracle):
    rng = np.random.default_rng(0)
    sizes, off = random_groups(rng, 300, lo=2)
    r = rng.normal(size=off[-1])
    for ddof in (0, 1):
        for eps in (0.0, 1e-6, 0.3):
            adv = oracle.group_advantage(off, r, "grpo", eps=eps, ddof=ddof)
            for g in range(len(sizes)):
                x = r[off[g]:off[g + 1]]
                want = (x - x.mean()) / (x.std(ddof=ddof) + eps)
                np.testing.assert_allclose(adv[off[g]:off[g + 1]], want, rtol=1e-12, atol=1e-14)
    adv = oracle.group_advantage(off, r, "grpo", eps=0.0)
    for g in range(len(sizes)):
        x = adv[off[g]:off[g + 1]]
        assert abs(x.mean()) < 1e-13
        assert x.var() == pytest.approx(1.0, rel=1e-12)


def test_grpo_zero_variance_groups_are_exactly_zero(oracle):
    # 0.1 * 3 / 3 != 0.1 in binary64: the rule must not rely on R - mean being 0.
    r = np.array([0.1, 0.1, 0.1, 1.0, 1.0, 0.0, 0.0, 0.0, 0.0, 0.5])
    off = np.array([0, 3, 5, 9, 10])
    for eps in (0.0, 1e-6):
        for ddof in (0, 1):
            adv = oracle.group_advantage(off, r, "grpo", eps=eps, ddof=ddof)
            assert np.all(adv == 0.0) and not np.signbit(adv).any()


def test_grpo_half_rewards(oracle):
    # training reward (fmt + acc)/2 takes values 0, 1/2, 1 (Sec. 4)
    r = np.array([0.0, 0.5, 0.5, 1.0, 1.0, 0.5, 0.0, 1.0])
    adv = oracle.group_advantage(np.array([0, 8]), r, "grpo", eps=1e-6)
    mean = r.sum() / 8
    sd = np.sqrt(((r - mean) ** 2).sum() / 8)
    np.testing.assert_allclose(adv, (r - mean) / (sd + 1e-6), rtol=1e-14)


def test_rloo_closed_forms(oracle):
    for G in (2, 5, 16, 33):
        for k in range(0, G + 1):
            r = np.zeros(G)
            r[:k] = 1.0
            adv = oracle.group_advantage(np.array([0, G]), r, "rloo")
            np.testing.assert_allclose(adv[:k], (G - k) / (G - 1), rtol=1e-15)
            np.testing.assert_allclose(adv[k:], -k / (G - 1), rtol=1e-15)
    rng = np.random.default_rng(1)
    sizes, off = random_groups(rng, 200, lo=1)
    r = rng.normal(size=off[-1])
    adv = oracle.group_advantage(off, r, "rloo")
    for g, G in enumerate(sizes):
        x, a = r[off[g]:off[g + 1]], adv[off[g]:off[g + 1]]
        if G == 1:
            assert a[0] == 0.0
            continue
        loo = np.array([np.delete(x, j).mean() for j in range(G)])       # definition
        np.testing.assert_allclose(a, x - loo, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(a, G / (G - 1) * (x - x.mean()), rtol=1e-11, atol=1e-13)
        assert abs(a.sum()) < 1e-12 * G


def test_empty_and_single_groups(oracle):
    off = np.array([0, 0, 1, 1, 3])
    r = np.array([1.0, 0.0, 1.0])
    assert oracle.group_advantage(off, r, "grpo", eps=1e-6).tolist() == [0.0, 1.0 / (0.5 + 1e-6) * -0.5, 1.0 / (0.5 + 1e-6) * 0.5]
    assert oracle.group_advantage(off, r, "rloo").tolist() == [0.0, -1.0, 1.0]
    assert oracle.group_advantage(np.array([0, 1]), np.array([1.0]), "grpo", ddof=1).tolist() == [0.0]


def test_token_broadcast_is_repeat(oracle):
    rng = np.random.default_rng(2)
    lengths = rng.integers(0, 50, 400)
    lengths[[3, 4, 5, 399]] = 0
    off = np.zeros(401, dtype=np.int64)
    np.cumsum(lengths, out=off[1:])
    adv = rng.normal(size=400)
    out = np.full(off[-1] + 7, np.nan)
    oracle.token_broadcast(adv, off, out=out)
    assert np.array_equal(out[:off[-1]], np.repeat(adv, lengths))
    assert np.isnan(out[off[-1]:]).all()
    assert out[:off[-1]].sum() == pytest.approx(np.dot(adv, lengths), rel=1e-10)
    with pytest.raises(oracle.OracleError):
        oracle.token_broadcast(adv[:2], np.array([0, 5, 3]))
