"""Randomized parity of the whole path against the CPU oracle, through the C ABI: many small
seeded cases (sizes around the kernels' tile and workgroup limits, priors, caps, budgets from
nothing to many rollouts per prompt, ragged shards, length mixes), every entry point of the
path on each of them.  Integers bit for bit, binary64 within 1e-12."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2605_07114_amd import hora
    assert torch.cuda.is_available(), "these tests need the MI355X"
    hora.load_library()
    return hora.Session("cuda:0"), torch, hora


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def allocation_matches(got, want, util, off):
    return (np.array_equal(got.delta.cpu().numpy().astype(np.int64), want)
            and np.array_equal(got.group_off.cpu().numpy(), off)
            and np.allclose(got.util.cpu().numpy(), util, rtol=1e-12, atol=0))


@pytest.mark.parametrize("seed", [101, 102, 103])
def test_random_batches(gpu, oracle, seed):
    sess, torch, hora = gpu
    rng = np.random.default_rng(seed)
    for case in range(60):
        n = int(rng.choice([1, 2, 7, 60, 255, 1000, 2047, 2048, 2049, 5000, 20000, 70000])) + int(rng.integers(0, 4))
        g0 = int(rng.choice([0, 1, 2, 4, 8, 16, 33]))
        c = rng.binomial(g0, rng.beta(0.5, 0.5, n)).astype(np.int32) if g0 > 0 else np.zeros(n, dtype=np.int32)
        cap = int(rng.choice([0, 0, 0, 3, 8, 56]))
        budget = int(float(rng.choice([0.0, 0.3, 1.0, 4.0, 8.0, 20.0])) * n)
        if cap > 0:
            budget = min(budget, n * cap)
        a0, b0 = (1.0, 1.0) if rng.random() < 0.6 else (float(rng.uniform(0.2, 4)), float(rng.uniform(0.2, 4)))
        tag = f"seed {seed} case {case}: n={n} g0={g0} budget={budget} cap={cap} prior=({a0:.3f}, {b0:.3f})"
        print(tag, flush=True)
        want = oracle.allocate(c, g0, budget, delta_max=cap, alpha0=a0, beta0=b0)
        alpha, beta = oracle.posterior(c, g0, a0, b0)
        util = oracle.utilities(alpha, beta, want)
        off = oracle.group_offsets(want, g0)
        dc = dev(torch, c)
        for method in (hora.ALLOC_CLASS, hora.ALLOC_BISECT):
            got = sess.allocate(dc, g0, budget, alpha0=a0, beta0=b0, delta_max=cap, method=method)
            assert sess.status() == 0 and allocation_matches(got, want, util, off), (tag, method)
        got = sess.allocate_posterior(dev(torch, alpha), dev(torch, beta), g0, budget, delta_max=cap)
        assert sess.status() == 0 and allocation_matches(got, want, util, off), (tag, "posterior")

        # the same prompts in ragged shards
        n_sh = int(rng.integers(1, min(n, 300) + 1))
        cuts = np.sort(rng.integers(0, n + 1, n_sh - 1))
        bounds = np.concatenate(([0], cuts, [n])).astype(np.int64)
        sizes = np.diff(bounds)
        sb = np.floor(sizes * rng.choice([0.0, 0.5, 2.0, 6.0, 12.0], n_sh)).astype(np.int64)
        if cap > 0:
            sb = np.minimum(sb, sizes * cap)
        want_sh = oracle.allocate_sharded(c, g0, bounds, sb, delta_max=cap, alpha0=a0, beta0=b0)
        got = sess.allocate_sharded(dc, g0, dev(torch, bounds), dev(torch, sb), alpha0=a0, beta0=b0, delta_max=cap)
        assert sess.status() == 0, tag
        assert allocation_matches(got, want_sh, oracle.utilities(alpha, beta, want_sh),
                                  oracle.group_offsets(want_sh, g0)), (tag, "sharded", n_sh)

        # advantages and token broadcast over the groups of the unsharded allocation
        n_resp = int(off[-1])
        if n_resp == 0 or n_resp > 2_000_000:
            continue
        reward = rng.integers(0, 2, n_resp).astype(np.float64) if rng.random() < 0.7 else rng.normal(size=n_resp)
        adv = None
        for mode, m in (("grpo", hora.ADV_GRPO), ("rloo", hora.ADV_RLOO)):
            adv = oracle.group_advantage(off, reward, mode, eps=1e-6)
            got_adv = sess.group_advantage(dev(torch, off), dev(torch, reward), m, eps=1e-6)
            assert sess.status() == 0, tag
            np.testing.assert_allclose(got_adv.cpu().numpy(), adv, rtol=1e-12, atol=1e-12, err_msg=tag)
        lens = rng.integers(0, int(rng.choice([2, 30, 400, 3000])) + 1, n_resp).astype(np.int64)
        if lens.sum() > 40_000_000:
            lens = np.minimum(lens, 20)
        tok_off = np.concatenate(([0], np.cumsum(lens))).astype(np.int64)
        total = int(tok_off[-1])
        as_float = rng.random() < 0.5
        vals = adv.astype(np.float32) if as_float else adv
        skew = int(rng.integers(0, 4)) if as_float else int(rng.integers(0, 2))
        buf = torch.full((total + skew + 3,), float("nan"), dtype=torch.float32 if as_float else torch.float64,
                         device="cuda:0")
        sess.token_broadcast(dev(torch, vals), dev(torch, tok_off if rng.random() < 0.5 else tok_off.astype(np.int32)),
                             total, out=buf[skew:skew + total])
        assert sess.status() == 0, tag
        host = buf.cpu().numpy()
        assert np.array_equal(host[skew:skew + total], oracle.token_broadcast(vals.astype(np.float64), tok_off).astype(vals.dtype)), tag
        assert np.isnan(host[:skew]).all() and np.isnan(host[skew + total:]).all(), tag


@pytest.mark.parametrize("seed", [201, 202])
def test_random_posteriors(gpu, oracle, seed):
    """Per-prompt posteriors of four kinds (learned priors; a few slowly decaying gain sequences
    among fast ones; a shared prior written per prompt; blocks of very different prompts), with
    budgets from a tenth of a unit to 150 units per prompt and caps: walks of very different
    length inside a wavefront and inside a batch.  Allocation and offsets bit for bit, utilities
    within 1e-12."""
    sess, torch, hora = gpu
    rng = np.random.default_rng(seed)
    for case in range(70):
        # (a third of the cases around and below one tile of 4096 prompts, down to the size where one workgroup searches alone)
        n = int(rng.integers(300, 4500)) if case % 3 == 0 else int(rng.integers(2049, 50000))
        g0 = int(rng.choice([2, 4, 8]))
        kind = int(rng.integers(0, 4))
        if kind == 0:
            s = rng.uniform(0.25, 16.0, n)
            p = rng.uniform(0.02, 0.98, n)
            c = rng.binomial(g0, p)
            alpha, beta = s * p + c, s * (1 - p) + g0 - c
        elif kind == 1:
            alpha, beta = rng.uniform(4.0, 9.0, n), rng.uniform(0.3, 1.0, n)
            slow = rng.random(n) < rng.uniform(0.005, 0.1)
            alpha[slow] = rng.uniform(0.1, 0.7, int(slow.sum()))
            beta[slow] = rng.uniform(1.0, 4.0, int(slow.sum()))
        elif kind == 2:
            c = rng.binomial(g0, rng.beta(0.5, 0.5, n))
            alpha, beta = 1.0 + c, 1.0 + g0 - c.astype(np.float64)
        else:
            alpha = np.repeat(rng.uniform(0.1, 9.0, (n + 999) // 1000), 1000)[:n] + rng.uniform(0, 0.01, n)
            beta = np.repeat(rng.uniform(0.3, 9.0, (n + 999) // 1000), 1000)[:n] + rng.uniform(0, 0.01, n)
        budget = int(min(float(rng.choice([0.1, 0.7, 2.0, 5.0, 9.0, 20.0, 30.0, 60.0, 150.0])) * n, 600000))
        cap = int(rng.choice([0, 0, 0, 3, 17, 60]))
        if cap > 0:
            budget = min(budget, cap * n)
        tag = f"seed {seed} case {case}: n={n} g0={g0} kind={kind} budget={budget} cap={cap}"
        print(tag, flush=True)
        want = oracle.allocate_posterior(alpha, beta, budget, delta_max=cap)
        got = sess.allocate_posterior(dev(torch, alpha), dev(torch, beta), g0, budget, delta_max=cap)
        assert sess.status() == 0, tag
        assert allocation_matches(got, want, oracle.utilities(alpha, beta, want), oracle.group_offsets(want, g0)), tag
