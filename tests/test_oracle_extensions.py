"""Pins for the oracle's functions beyond the main path (CPU only): centred advantage,
loss weights with variable-size groups (Sec. 3.1 objective, Sec. 3.2 "Training objective
with variable-size groups"), the baseline allocation rules of Sec. 5 / Table 2, and the
Pass@K estimator of Sec. 4, Eq. 6."""
from fractions import Fraction
from itertools import combinations

import numpy as np
import pytest


def random_groups(rng, n_groups, lo=1, hi=40):
    sizes = rng.integers(lo, hi + 1, n_groups)
    off = np.zeros(n_groups + 1, dtype=np.int64)
    np.cumsum(sizes, out=off[1:])
    return sizes, off


# ---- centred advantage -------------------------------------------------------------------
def test_centred_advantage_is_reward_minus_group_mean(oracle):
    rng = np.random.default_rng(5)
    sizes, off = random_groups(rng, 200)
    r = rng.normal(size=off[-1])
    adv = oracle.group_advantage(off, r, "center")
    rloo = oracle.group_advantage(off, r, "rloo")
    for g, size in enumerate(sizes):
        x = r[off[g]:off[g + 1]]
        np.testing.assert_allclose(adv[off[g]:off[g + 1]], x - x.mean(), rtol=0, atol=1e-14)
        if size > 1:   # leave-one-out baseline = G/(G-1) times the centred reward
            np.testing.assert_allclose(rloo[off[g]:off[g + 1]], size / (size - 1) * (x - x.mean()), rtol=0, atol=1e-13)
    # equal rewards give exactly zero although mean(0.1, 0.1, 0.1) != 0.1 in binary64
    assert np.all(oracle.group_advantage([0, 3, 4], [0.1, 0.1, 0.1, 7.0], "center") == 0.0)


# ---- loss weights ------------------------------------------------------------------------
def test_token_weights_give_every_prompt_the_same_total(oracle):
    """With w_j = 1/(G_i |o_j|) the tokens of prompt i carry total weight sum_j |o_j| w_j = 1,
    whatever G_i is: the reason the paper replaces 1/G by 1/G_i."""
    rng = np.random.default_rng(6)
    sizes, goff = random_groups(rng, 100, lo=1, hi=70)
    lens = rng.integers(1, 3000, goff[-1])
    toff = np.concatenate(([0], np.cumsum(lens))).astype(np.int64)
    w = oracle.response_weights(goff, toff)
    for g, size in enumerate(sizes):
        sl = slice(goff[g], goff[g + 1])
        assert float(np.dot(w[sl], lens[sl])) == pytest.approx(1.0, rel=1e-13)
        for j in range(goff[g], goff[g + 1]):   # exactly the correctly rounded quotient
            assert w[j] == float(Fraction(1, int(size) * int(lens[j])))


def test_constant_length_weights_and_empty_responses(oracle):
    goff = np.array([0, 3, 5], dtype=np.int64)
    toff = np.array([0, 10, 10, 40, 50, 80], dtype=np.int64)      # response 1 is empty
    w = oracle.response_weights(goff, toff)
    assert w.tolist() == [1 / 30, 0.0, 1 / 90, 1 / 20, 1 / 60]
    w = oracle.response_weights(goff, toff, length_const=2048.0)
    assert w.tolist() == [1 / (3 * 2048.0), 0.0, 1 / (3 * 2048.0), 1 / 4096.0, 1 / 4096.0]
    # constant normalisation: a prompt's total is its mean response length over the constant
    lens = np.diff(toff)
    assert float(np.dot(w[:3], lens[:3])) == pytest.approx(lens[:3].sum() / 3 / 2048.0, rel=1e-14)


# ---- baseline allocation rules -----------------------------------------------------------
def test_uniform_rule_closed_form(oracle):
    for n, budget in ((7, 0), (7, 7), (7, 23), (1, 5), (1000, 24000), (1000, 24017)):
        c = np.random.default_rng(n + budget).integers(0, 9, n).astype(np.int32)
        delta = oracle.allocate_baseline(c, budget, "uniform")
        want = budget // n + (np.arange(n) < budget % n)
        assert np.array_equal(delta, want)


def test_hard_first_rule(oracle):
    rng = np.random.default_rng(9)
    for trial in range(50):
        n = int(rng.integers(1, 40))
        c = rng.integers(0, 4, n).astype(np.int32)
        budget = int(rng.integers(0, 200))
        delta = oracle.allocate_baseline(c, budget, "hard_first")
        assert delta.sum() == budget and (delta >= 0).all()
        hard = c == 0
        if hard.any():
            assert (delta[~hard] == 0).all()                      # only prompts with c_i = 0 receive rollouts
            d = delta[hard]
            assert d.max() - d.min() <= 1 and (np.diff(d) <= 0).all()   # even split, lower indices first
        else:                                                     # reading: no hard prompt -> uniform
            assert np.array_equal(delta, oracle.allocate_baseline(c, budget, "uniform"))


def test_baseline_rules_respect_the_cap(oracle):
    c = np.array([0, 1, 0, 2], dtype=np.int32)
    assert oracle.allocate_baseline(c, 6, "hard_first", delta_max=3).tolist() == [3, 0, 3, 0]
    with pytest.raises(oracle.OracleError):
        oracle.allocate_baseline(c, 7, "hard_first", delta_max=3)
    with pytest.raises(oracle.OracleError):
        oracle.allocate_baseline(c, 13, "uniform", delta_max=3)
    assert oracle.allocate_baseline(c, 12, "uniform", delta_max=3).tolist() == [3, 3, 3, 3]


# ---- Pass@K ------------------------------------------------------------------------------
def test_pass_at_k_is_the_chance_that_k_of_the_n_samples_hold_a_correct_one(oracle):
    """Brute force over all K-subsets of the sample pool (tiny pools)."""
    for n in (1, 2, 5, 7):
        for c in range(n + 1):
            correct = [1] * c + [0] * (n - c)
            for k in range(1, n + 1):
                subsets = list(combinations(range(n), k))
                hit = sum(any(correct[j] for j in s) for s in subsets)
                per, mean = oracle.pass_at_k([n], [c], [k])
                assert per[0, 0] == float(Fraction(hit, len(subsets)))
                assert mean[0] == per[0, 0]


def test_pass_at_k_special_cases_and_mean(oracle):
    n = np.array([256, 256, 1024, 1024, 16])
    c = np.array([0, 3, 1, 1020, 16])
    per, mean = oracle.pass_at_k(n, c, [1, 8, 16])
    assert np.array_equal(per[0], c / n)                      # K = 1: the plain success rate
    assert (per[:, 0] == 0).all()                              # no correct sample
    assert per[1, 3] == 1.0 and per[2, 4] == 1.0               # fewer than K wrong samples
    assert per[1, 2] == 8 / 1024                               # c = 1: K / N
    assert (np.diff(per, axis=0) >= 0).all()                   # non-decreasing in K
    np.testing.assert_allclose(mean, per.mean(axis=1), rtol=1e-15)
    # product form 1 - prod_{i<c} (N-K-i)/(N-i)
    want = 1 - np.prod([(256 - 8 - i) / (256 - i) for i in range(3)])
    assert per[1, 1] == pytest.approx(want, rel=1e-14)
    with pytest.raises(oracle.OracleError):
        oracle.pass_at_k([8], [9], [1])
    with pytest.raises(oracle.OracleError):
        oracle.pass_at_k([8], [1], [9])
