"""The synthetic input recipes are deterministic and have the stated shape."""
import numpy as np

from paper_2605_07114_amd import workloads as wl


def test_phase_a_is_deterministic_and_in_range():
    for w in (wl.TINY, wl.SMALL, wl.scaled(wl.SKEWED, 4096)):
        a, b = wl.phase_a(w), wl.phase_a(w)
        assert np.array_equal(a.c, b.c) and np.array_equal(a.p, b.p)
        assert a.c.dtype == np.int32 and a.c.min() >= 0 and a.c.max() <= w.g0
        assert np.array_equal(a.c, a.pre.sum(axis=1))


def test_mixture_shapes():
    a = wl.phase_a(wl.scaled(wl.SKEWED, 65536))
    assert 0.55 < (a.p == 0).mean() < 0.65
    assert 0.70 < (a.c == 0).mean() < 0.82          # hard prompts dominate
    a = wl.phase_a(wl.scaled(wl.LARGE_ALLOC, 1 << 16))
    frac0, frac4 = (a.c == 0).mean(), (a.c == 4).mean()
    assert abs(frac0 - 0.2734) < 0.01 and abs(frac4 - 0.2734) < 0.01   # C(8,4)/2^8 each


def test_phase_b_layout():
    w = wl.TINY
    a = wl.phase_a(w)
    delta = np.arange(w.n) % 5
    b = wl.phase_b(w, a, delta)
    assert b.group_off[-1] == w.n * w.g0 + delta.sum() == b.reward.size
    assert np.array_equal(np.diff(b.group_off), w.g0 + delta)
    # pre-rollout rewards come first and reproduce c
    for i in (0, 1, 17, w.n - 1):
        lo = b.group_off[i]
        assert b.reward[lo:lo + w.g0].sum() == a.c[i]
    assert set(np.unique(b.reward)) <= {0.0, 1.0}
    assert b.lengths.min() >= 64 and b.lengths.max() <= 512
    assert b.tok_off[0] == 0 and np.array_equal(np.diff(b.tok_off), b.lengths)
    h = wl.phase_b(w, a, delta, half_rewards=True)
    assert set(np.unique(h.reward)) <= {0.0, 0.5, 1.0}


def test_lognormal_lengths_clip():
    rng = np.random.Generator(np.random.PCG64(0))
    x = wl.draw_lengths(("lognormal", 2048.0, 0.7, 128, 16384), 200000, rng)
    assert x.min() >= 128 and x.max() <= 16384
    assert 1900 < np.median(x) < 2200
