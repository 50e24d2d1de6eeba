"""GPU parity: hora_marginal_gains / hora_allocate / hora_allocate_posterior against the
CPU oracle, through the C ABI.  Integers must match bit for bit; utilities within
1e-12 relative (Sec. 3.2 Eq. 2-5, Alg. 1, Prop. 1)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

UTIL_RTOL = 1e-12


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2605_07114_amd import hora
    assert torch.cuda.is_available(), "these tests need the MI355X"
    hora.load_library()
    return hora.Session("cuda:0"), torch, hora


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def summary_fields(alloc):
    s = alloc.summary.cpu().numpy()
    tau = s[:1].view(np.float64)[0]
    return tau, int(s[1]), int(s[2]), int(s[3])


def check_allocation(gpu, oracle, c, g0, budget, delta_max=0, methods=None, alpha0=1.0, beta0=1.0,
                     off_dtype="i64"):
    sess, torch, hora = gpu
    methods = methods or (hora.ALLOC_CLASS, hora.ALLOC_BISECT)
    want = oracle.allocate(c, g0, budget, delta_max=delta_max, alpha0=alpha0, beta0=beta0)
    alpha, beta = oracle.posterior(c, g0, alpha0, beta0)
    want_util = oracle.utilities(alpha, beta, want) if c.size <= 20000 else None
    want_off = oracle.group_offsets(want, g0)
    tdt = {"i32": torch.int32, "i64": torch.int64}[off_dtype]
    for method in methods:
        print(f"allocate n={c.size} g0={g0} budget={budget} cap={delta_max} method={method}", flush=True)
        got = sess.allocate(dev(torch, c), g0, budget, alpha0=alpha0, beta0=beta0, delta_max=delta_max,
                            method=method, off_dtype=tdt)
        assert sess.status() == 0
        delta = got.delta.cpu().numpy()
        assert delta.dtype == np.int32
        assert np.array_equal(delta.astype(np.int64), want), (method, np.flatnonzero(delta != want)[:10])
        assert np.array_equal(got.group_off.cpu().numpy().astype(np.int64), want_off)
        util = got.util.cpu().numpy()
        if want_util is not None:
            np.testing.assert_allclose(util, want_util, rtol=UTIL_RTOL, atol=0)
        else:   # large inputs: the utility depends on (c, delta) only -- compare per distinct pair
            key = c.astype(np.int64) * (int(want.max()) + 1) + want
            uniq, first = np.unique(key, return_index=True)
            ref = oracle.utilities(alpha[first], beta[first], want[first])
            np.testing.assert_allclose(util[first], ref, rtol=UTIL_RTOL, atol=0)
            lut = dict(zip(uniq.tolist(), util[first].tolist()))
            assert np.array_equal(util, np.array([lut[k] for k in uniq])[np.searchsorted(uniq, key)])
        tau, count_gt, tie_units, tie_prompts = summary_fields(got)
        assert count_gt + tie_units == budget
        assert 0 <= tie_units <= max(tie_prompts, 0)
        if budget > 0:
            # tau is the smallest gain that was selected
            sel = np.flatnonzero(want > 0)
            classes = np.unique(c[sel])
            smallest = min(oracle.marginal_gains(alpha0 + k, beta0 + g0 - k, int(want[c == k].max()))[-1]
                           for k in classes)
            assert tau == smallest
    return want


@pytest.mark.parametrize("g0", [1, 2, 4, 8, 16])
def test_gain_and_utility_tables_are_bit_identical(gpu, oracle, g0):
    sess, torch, hora = gpu
    count = 4096
    rng = np.random.default_rng(g0)
    alpha = np.concatenate([1.0 + np.arange(g0 + 1), rng.uniform(0.02, 30, 300)])
    beta = np.concatenate([1.0 + g0 - np.arange(g0 + 1), rng.uniform(0.02, 30, 300)])
    n = alpha.size
    gains = torch.empty(count * n, dtype=torch.float64, device="cuda:0")
    util = torch.empty(count * n, dtype=torch.float64, device="cuda:0")
    hora.hora_marginal_gains(dev(torch, alpha), dev(torch, beta), count, gains, util)
    gains = gains.cpu().numpy().reshape(count, n)
    util = util.cpu().numpy().reshape(count, n)
    for i in range(n):
        want = oracle.marginal_gains(alpha[i], beta[i], count)
        assert np.array_equal(gains[:, i].view(np.int64), want.view(np.int64)), (i, alpha[i], beta[i])
    for i in range(0, n, 7):
        for l in (0, 1, 2, 5, 33, 1000, 4095):
            assert util[l, i] == oracle.hit_utility(alpha[i], beta[i], l)


def test_worked_example(gpu, oracle):
    c = np.array([0, 2, 4], dtype=np.int32)
    for budget in range(13):
        check_allocation(gpu, oracle, c, 4, budget)


@pytest.mark.parametrize("name", ["tiny", "small", "skewed", "large_bcast", "large_alloc"])
def test_allocation_parity_on_the_workloads(gpu, oracle, name):
    from paper_2605_07114_amd import workloads as wl
    w = wl.WORKLOADS[name]
    a = wl.phase_a(w)
    check_allocation(gpu, oracle, a.c, w.g0, w.budget, delta_max=w.delta_max,
                     off_dtype=w.group_off_type)


def test_ragged_sizes_and_budgets(gpu, oracle):
    rng = np.random.default_rng(17)
    for n in (1, 2, 3, 5, 63, 64, 65, 255, 1023, 1024, 1025, 4097, 70001):
        g0 = int(rng.choice([2, 4, 8]))
        c = rng.integers(0, g0 + 1, n).astype(np.int32)
        for budget in {0, 1, n - 1 if n > 1 else 1, n, 3 * n + 1}:
            check_allocation(gpu, oracle, c, g0, budget)


def test_degenerate_inputs(gpu, oracle):
    # all prompts equal: budget splits evenly, the remainder goes to the lowest indices
    for c0, g0 in ((0, 4), (4, 4), (3, 8)):
        c = np.full(3000, c0, dtype=np.int32)
        for budget in (0, 1, 2999, 3000, 3001, 10007):
            want = check_allocation(gpu, oracle, c, g0, budget)
            assert want.max() - want.min() <= 1 and np.all(np.diff(want) <= 0)
    # one prompt takes everything
    check_allocation(gpu, oracle, np.array([2], dtype=np.int32), 4, 777)
    # G0 = 0: no evidence, every prompt has the prior
    check_allocation(gpu, oracle, np.zeros(100, dtype=np.int32), 0, 250)
    # other priors, including a non-integer one
    rng = np.random.default_rng(3)
    c = rng.integers(0, 9, 5000).astype(np.int32)
    check_allocation(gpu, oracle, c, 8, 40000, alpha0=0.5, beta0=0.5)
    check_allocation(gpu, oracle, c, 8, 40000, alpha0=2.0, beta0=3.25)


def test_cap(gpu, oracle):
    c = np.zeros(4, dtype=np.int32)
    assert check_allocation(gpu, oracle, c, 4, 12, delta_max=3).tolist() == [3, 3, 3, 3]
    assert check_allocation(gpu, oracle, c, 4, 13, delta_max=4).tolist() == [4, 3, 3, 3]
    rng = np.random.default_rng(5)
    c = rng.integers(0, 9, 6000).astype(np.int32)
    for cap, budget in ((1, 6000), (1, 4321), (2, 9000), (5, 30000), (5, 29999), (56, 48000)):
        want = check_allocation(gpu, oracle, c, 8, budget, delta_max=cap)
        assert want.max() <= cap
    # a cap that binds for the hard prompts only
    c = np.array([0, 8, 8, 0, 8], dtype=np.int32)
    want = check_allocation(gpu, oracle, c, 8, 20, delta_max=6)
    assert want[0] == 6 and want[3] == 6


def test_large_g0_uses_every_class_lane(gpu, oracle):
    rng = np.random.default_rng(8)
    for g0 in (31, 63):
        c = rng.integers(0, g0 + 1, 20000).astype(np.int32)
        check_allocation(gpu, oracle, c, g0, 60000)
    # beyond the class method's limit AUTO falls back to bisection
    sess, torch, hora = gpu
    c = rng.integers(0, 101, 5000).astype(np.int32)
    check_allocation(gpu, oracle, c, 100, 15000, methods=(hora.ALLOC_AUTO,))


def test_unaligned_buffers(gpu, oracle):
    sess, torch, hora = gpu
    rng = np.random.default_rng(9)
    n, g0, budget = 5003, 4, 17011
    c = rng.integers(0, g0 + 1, n).astype(np.int32)
    want = oracle.allocate(c, g0, budget)
    for method in (hora.ALLOC_CLASS, hora.ALLOC_BISECT):
        cbuf = torch.zeros(n + 8, dtype=torch.int32, device="cuda:0")
        dbuf = torch.full((n + 8,), -7, dtype=torch.int32, device="cuda:0")
        ubuf = torch.full((n + 8,), -7.0, dtype=torch.float64, device="cuda:0")
        obuf = torch.full((n + 9,), -7, dtype=torch.int32, device="cuda:0")
        cbuf[1:n + 1] = dev(torch, c)
        hora.hora_allocate(cbuf[1:n + 1], g0, budget, dbuf[3:n + 3], sess.dev_status, sess.workspace(n, g0),
                           method=method, util=ubuf[1:n + 1], group_off=obuf[1:n + 2])
        assert sess.status() == 0
        d = dbuf.cpu().numpy()
        assert np.array_equal(d[3:n + 3], want) and np.all(d[:3] == -7) and np.all(d[n + 3:] == -7)
        o = obuf.cpu().numpy()
        assert np.array_equal(o[1:n + 2], oracle.group_offsets(want, g0)) and o[0] == -7 and np.all(o[n + 2:] == -7)
        u = ubuf.cpu().numpy()
        assert u[0] == -7.0 and np.all(u[n + 1:] == -7.0) and np.all((u[1:n + 1] >= 0) & (u[1:n + 1] < 1))


def test_data_errors_are_reported_not_fatal(gpu, oracle):
    sess, torch, hora = gpu
    c = np.array([0, 1, 9, 2, -3, 4] * 500, dtype=np.int32)
    for method in (hora.ALLOC_CLASS, hora.ALLOC_BISECT):
        got = sess.allocate(dev(torch, c), 4, 6000, method=method)
        assert sess.status() == hora.ERR_RANGE
        sess.dev_status.zero_()
        d = got.delta.cpu().numpy()
        assert d.min() >= 0 and d.sum() == 6000      # still a placement of the budget
    with pytest.raises(hora.HoraError) as e:
        sess.allocate(dev(torch, c[:4]), 4, 50, delta_max=3)
    assert e.value.status == hora.ERR_INFEASIBLE
    # empty batch
    got = sess.allocate(torch.zeros(0, dtype=torch.int32, device="cuda:0"), 4, 0)
    assert got.group_off.cpu().tolist() == [0] and sess.status() == 0


def test_repeated_calls_reuse_the_workspace(gpu, oracle):
    sess, torch, hora = gpu
    rng = np.random.default_rng(12)
    c = rng.integers(0, 5, 30000).astype(np.int32)
    want = oracle.allocate(c, 4, 90001)
    cd = dev(torch, c)
    for rep in range(4):
        for method in (hora.ALLOC_BISECT, hora.ALLOC_CLASS):
            got = sess.allocate(cd, 4, 90001, method=method)
            assert np.array_equal(got.delta.cpu().numpy(), want)
    assert sess.status() == 0


def learned_prior(rng, n, g0):
    """Posterior of App. D: alpha = s p + c, beta = s (1 - p) + G0 - c, s in [0.25, 16]."""
    s = rng.uniform(0.25, 16.0, n)
    p = rng.uniform(0.02, 0.98, n)
    c = rng.binomial(g0, p)
    return s * p + c, s * (1 - p) + g0 - c, c.astype(np.int32)


def test_per_prompt_posteriors(gpu, oracle):
    sess, torch, hora = gpu
    rng = np.random.default_rng(21)
    for n, g0, budget, cap in ((1, 8, 9, 0), (777, 8, 5000, 0), (20000, 8, 160000, 0), (20000, 4, 70000, 5),
                               (300000, 8, 2400000, 0)):
        alpha, beta, _ = learned_prior(rng, n, g0)
        want = oracle.allocate_posterior(alpha, beta, budget, delta_max=cap)
        print(f"allocate_posterior n={n} budget={budget} cap={cap}", flush=True)
        got = sess.allocate_posterior(dev(torch, alpha), dev(torch, beta), g0, budget, delta_max=cap)
        assert sess.status() == 0
        assert np.array_equal(got.delta.cpu().numpy().astype(np.int64), want)
        assert np.array_equal(got.group_off.cpu().numpy(), oracle.group_offsets(want, g0))
        idx = rng.integers(0, n, min(n, 3000))
        np.testing.assert_allclose(got.util.cpu().numpy()[idx], oracle.utilities(alpha[idx], beta[idx], want[idx]),
                                   rtol=UTIL_RTOL, atol=0)


def test_posteriors_whose_contested_gains_sit_in_one_workgroup(gpu, oracle):
    """The search sets the gains of a narrow bracket aside, one list per workgroup.  Here all
    gains near the threshold belong to prompts of one workgroup's share (the others are hopeless
    prompts that get nothing), so its list overflows at first and the search has to carry on
    without it."""
    sess, torch, hora = gpu
    rng = np.random.default_rng(23)
    n, g0 = 200000, 8
    alpha = np.full(n, 0.01)
    beta = np.full(n, 60.0)
    good = slice(5 * 1024, 6 * 1024)                  # one tile of 1024 prompts
    alpha[good] = rng.uniform(0.5, 9.0, 1024)
    beta[good] = rng.uniform(0.5, 9.0, 1024)
    for budget in (1024 * 40, 1024 * 3, 1024 * 300):
        want = oracle.allocate_posterior(alpha, beta, budget)
        if budget <= 1024 * 40:
            assert want[good].sum() == budget        # nothing goes to the hopeless prompts
        print(f"allocate_posterior one-tile contest n={n} budget={budget}", flush=True)
        got = sess.allocate_posterior(dev(torch, alpha), dev(torch, beta), g0, budget)
        assert sess.status() == 0
        assert np.array_equal(got.delta.cpu().numpy().astype(np.int64), want)
        np.testing.assert_allclose(got.util.cpu().numpy()[good], oracle.utilities(alpha[good], beta[good], want[good]),
                                   rtol=UTIL_RTOL, atol=0)


def test_depth_estimate_from_an_unrepresentative_sample(gpu, oracle):
    """The threshold search takes the depth of its first walk from 512 prompts spread evenly
    over the batch (prompt floor(q n / 512), q < 512).  The estimate only steers the work: with
    a sample that is nothing like the batch (the sampled prompts all eager, the rest reluctant;
    the reverse; prompts sorted, so that the tiles differ as much as they can) the allocation
    must still be the oracle's."""
    sess, torch, hora = gpu
    rng = np.random.default_rng(29)
    n, g0 = 300000, 8
    sampled = (np.arange(512, dtype=np.int64) * n) // 512
    cases = {}
    for name, (c_sample, c_rest) in {"sample decays fast": (g0, 0), "sample decays slowly": (0, g0)}.items():
        c = np.full(n, c_rest, dtype=np.int32)
        c[sampled] = c_sample
        cases[name] = c
    cases["sorted"] = np.sort(rng.binomial(g0, rng.beta(0.5, 0.5, n)).astype(np.int32))
    cases["sorted descending"] = cases["sorted"][::-1].copy()
    for name, c in cases.items():
        for budget in (4 * n, n // 3, 40 * n):
            print(f"allocate (threshold search) {name} n={n} budget={budget}", flush=True)
            check_allocation(gpu, oracle, c, g0, budget, methods=(hora.ALLOC_BISECT,))
    # the same through per-prompt posteriors, with a cap that some prompts reach
    alpha = np.where(np.isin(np.arange(n), sampled), 9.0, 0.4) + rng.uniform(0.0, 0.05, n)
    beta = np.where(np.isin(np.arange(n), sampled), 0.5, 7.0) + rng.uniform(0.0, 0.05, n)
    for budget, cap in ((4 * n, 0), (6 * n, 9)):
        want = oracle.allocate_posterior(alpha, beta, budget, delta_max=cap)
        print(f"allocate_posterior unrepresentative sample n={n} budget={budget} cap={cap}", flush=True)
        got = sess.allocate_posterior(dev(torch, alpha), dev(torch, beta), g0, budget, delta_max=cap)
        assert sess.status() == 0
        assert np.array_equal(got.delta.cpu().numpy().astype(np.int64), want)


def test_deep_budgets_with_walks_of_very_different_length(gpu, oracle):
    """With a deep budget and prompts whose gain sequences decay at very different rates the
    threshold search hands a wavefront's prompts to its lanes one by one instead of walking them
    in lockstep (coarse count and survival products).  Same allocation, same utilities; also when
    half of the tiles hold nothing but reluctant prompts, so that they end the pooled walk short
    of their share and are walked again octave by octave."""
    sess, torch, hora = gpu
    rng = np.random.default_rng(31)
    n, g0 = 40000, 8
    alpha, beta, _ = learned_prior(rng, n, g0)
    cases = {"mixed": (alpha, beta)}
    a2, b2 = alpha.copy(), beta.copy()
    a2[n // 2:] = 0.02 + rng.uniform(0.0, 0.01, n - n // 2)       # hopeless prompts: gains ~ 1e-3 and below
    b2[n // 2:] = 30.0 + rng.uniform(0.0, 1.0, n - n // 2)
    cases["half of the tiles reluctant"] = (a2, b2)
    for name, (al, be) in cases.items():
        for budget, cap in ((100 * n, 0), (150 * n, 400)):
            want = oracle.allocate_posterior(al, be, budget, delta_max=cap)
            print(f"allocate_posterior deep, {name}: n={n} budget={budget} cap={cap} deepest={int(want.max())} "
                  f"mean={want.mean():.0f}", flush=True)
            got = sess.allocate_posterior(dev(torch, al), dev(torch, be), g0, budget, delta_max=cap)
            assert sess.status() == 0
            assert np.array_equal(got.delta.cpu().numpy().astype(np.int64), want)
            idx = rng.integers(0, n, 2000)
            np.testing.assert_allclose(got.util.cpu().numpy()[idx], oracle.utilities(al[idx], be[idx], want[idx]),
                                       rtol=UTIL_RTOL, atol=0)


def test_a_few_deep_walks_in_every_wavefront(gpu, oracle):
    """While the coarse count walks, a wavefront whose active walks would fit fewer items per
    lane permutes its 256 walks across its lanes, and permutes the kept walk states back before
    they are stored.  Here every block of 256 prompts holds a handful of prompts whose gains
    decay slowly among prompts that are done after a step or two (so the regrouping goes from
    four items per lane to one early), the batch ends in a ragged tile, and a cap stops the
    deepest walks.  Allocation and offsets bit for bit, utilities within 1e-12."""
    sess, torch, hora = gpu
    rng = np.random.default_rng(37)
    n, g0 = 5 * 4096 + 777, 8
    alpha = rng.uniform(6.0, 9.0, n)            # fast decay: a gain or two above any threshold of interest
    beta = rng.uniform(0.3, 1.0, n)
    deep = np.zeros(n, dtype=bool)
    for start in range(0, n, 256):
        pick = start + rng.choice(min(256, n - start), size=min(5, n - start), replace=False)
        deep[pick] = True
    alpha[deep] = rng.uniform(0.2, 0.6, int(deep.sum()))     # slow decay: dozens of gains in the same range
    beta[deep] = rng.uniform(1.0, 3.0, int(deep.sum()))
    for budget, cap in ((3 * n, 0), (4 * n, 30), (6 * n, 0)):
        want = oracle.allocate_posterior(alpha, beta, budget, delta_max=cap)
        print(f"allocate_posterior few deep walks n={n} budget={budget} cap={cap} deepest={int(want.max())} "
              f"median={int(np.median(want))}", flush=True)
        got = sess.allocate_posterior(dev(torch, alpha), dev(torch, beta), g0, budget, delta_max=cap)
        assert sess.status() == 0
        assert np.array_equal(got.delta.cpu().numpy().astype(np.int64), want)
        assert np.array_equal(got.group_off.cpu().numpy(), oracle.group_offsets(want, g0))
        np.testing.assert_allclose(got.util.cpu().numpy(), oracle.utilities(alpha, beta, want), rtol=UTIL_RTOL, atol=0)


@pytest.mark.parametrize("n,g0,per", [(3 * (1 << 20) + 5, 4, 3), ((1 << 21) + 4097, 0, 2)])
def test_offsets_over_several_tiles_per_workgroup(gpu, oracle, n, g0, per):
    """Beyond 2^20 prompts a workgroup handles several tiles and carries its running sums from
    tile to tile; 32-bit offsets are formed in 32-bit arithmetic, 64-bit ones in 64-bit.  Both
    methods, both offset types, G0 = 0 included (the offsets are then the prefix sums of delta)."""
    sess, torch, hora = gpu
    rng = np.random.default_rng(n % 1000)
    c = rng.binomial(g0, rng.beta(0.5, 0.5, n)).astype(np.int32) if g0 else np.zeros(n, dtype=np.int32)
    budget = per * n
    want = oracle.allocate(c, g0, budget)
    off = oracle.group_offsets(want, g0)
    dc = dev(torch, c)
    for method in (hora.ALLOC_CLASS, hora.ALLOC_BISECT):
        for dt in (torch.int32, torch.int64):
            print(f"allocate n={n} g0={g0} budget={budget} method={method} offsets={dt}", flush=True)
            got = sess.allocate(dc, g0, budget, method=method, off_dtype=dt)
            assert sess.status() == 0
            assert np.array_equal(got.delta.cpu().numpy().astype(np.int64), want)
            assert np.array_equal(got.group_off.cpu().numpy().astype(np.int64), off)


@pytest.mark.parametrize("n", [1, 60, 511, 512, 513, 4095, 4096, 4097])
def test_posteriors_around_the_sizes_where_the_method_changes(gpu, oracle, n):
    """Per-prompt posteriors at the sizes of one training step and at the batch sizes where the
    library changes its way of working: one workgroup that searches alone (up to 512 prompts),
    one tile whose steps run in a single launch (up to 4096), the launches of the general path.
    Learned-prior posteriors (App. D), 8 and 24 units per prompt, one run with a cap that binds.
    Allocation and offsets bit for bit, utilities within 1e-12."""
    sess, torch, hora = gpu
    rng = np.random.default_rng(1000 + n)
    g0 = 8
    s = rng.uniform(0.25, 16.0, n)
    p = rng.uniform(0.02, 0.98, n)
    c = rng.binomial(g0, p)
    alpha, beta = s * p + c, s * (1 - p) + g0 - c
    for budget, cap in ((8 * n, 0), (24 * n, 0), (24 * n, 40), (1, 0)):
        want = oracle.allocate_posterior(alpha, beta, budget, delta_max=cap)
        print(f"allocate_posterior n={n} budget={budget} cap={cap} deepest={int(want.max())}", flush=True)
        got = sess.allocate_posterior(dev(torch, alpha), dev(torch, beta), g0, budget, delta_max=cap)
        assert sess.status() == 0
        assert np.array_equal(got.delta.cpu().numpy().astype(np.int64), want)
        assert np.array_equal(got.group_off.cpu().numpy(), oracle.group_offsets(want, g0))
        np.testing.assert_allclose(got.util.cpu().numpy(), oracle.utilities(alpha, beta, want), rtol=UTIL_RTOL, atol=0)


def test_posteriors_beyond_a_million_prompts(gpu, oracle):
    """More tiles than the first narrowing pass keeps in registers when it adds up the tiles'
    coarse counts (256 tiles of 4096 prompts): learned-prior posteriors (App. D) in a batch of
    385 tiles, the last one ragged.  Allocation and offsets bit for bit, utilities within 1e-12."""
    sess, torch, hora = gpu
    rng = np.random.default_rng(41)
    n, g0 = (1 << 20) + (1 << 19) + 777, 8
    s = rng.uniform(0.25, 16.0, n)
    p = rng.uniform(0.02, 0.98, n)
    c = rng.binomial(g0, p)
    alpha, beta = s * p + c, s * (1 - p) + g0 - c
    budget = 3 * n
    want = oracle.allocate_posterior(alpha, beta, budget)
    print(f"allocate_posterior n={n} budget={budget} deepest={int(want.max())}", flush=True)
    got = sess.allocate_posterior(dev(torch, alpha), dev(torch, beta), g0, budget)
    assert sess.status() == 0
    assert np.array_equal(got.delta.cpu().numpy().astype(np.int64), want)
    assert np.array_equal(got.group_off.cpu().numpy(), oracle.group_offsets(want, g0))
    np.testing.assert_allclose(got.util.cpu().numpy(), oracle.utilities(alpha, beta, want), rtol=UTIL_RTOL, atol=0)


def test_learned_prior_collapses_to_the_uniform_prior(gpu, oracle):
    # App. D: s = 2, p = 1/2 gives alpha = 1 + c, beta = 1 + G0 - c
    sess, torch, hora = gpu
    rng = np.random.default_rng(22)
    g0, n, budget = 8, 50000, 400000
    c = rng.integers(0, g0 + 1, n).astype(np.int32)
    alpha = 2.0 * 0.5 + c
    beta = 2.0 * (1 - 0.5) + g0 - c
    want = oracle.allocate(c, g0, budget)
    got = sess.allocate_posterior(dev(torch, alpha), dev(torch, beta), g0, budget)
    assert np.array_equal(got.delta.cpu().numpy(), want)
    got2 = sess.allocate(dev(torch, c), g0, budget)
    assert torch.equal(got.delta, got2.delta)
    # (the two calls evaluate E(k) differently: a table of the product recurrence, the closed-form
    # ratio of App. A from the last gain)
    np.testing.assert_allclose(got.util.cpu().numpy(), got2.util.cpu().numpy(), rtol=UTIL_RTOL, atol=0)
    np.testing.assert_allclose(got.util.cpu().numpy(), oracle.utilities(alpha, beta, want), rtol=UTIL_RTOL, atol=0)
    assert sess.status() == 0
    bad = alpha.copy()
    bad[17] = -1.0
    sess.allocate_posterior(dev(torch, bad), dev(torch, beta), g0, budget)
    assert sess.status() == hora.ERR_RANGE
    sess.dev_status.zero_()


def test_exchange_condition_on_the_large_workload(gpu, oracle):
    """Optimality certificate of App. A on the GPU result itself, at N = 2^20."""
    from fractions import Fraction
    from test_oracle_gains import exact_gain
    from paper_2605_07114_amd import workloads as wl
    sess, torch, hora = gpu
    w = wl.LARGE_ALLOC
    a = wl.phase_a(w)
    got = sess.allocate(dev(torch, a.c), w.g0, w.budget)
    delta = got.delta.cpu().numpy()
    assert delta.sum() == w.budget and delta.min() >= 0
    taken, avail = [], []
    for k in range(w.g0 + 1):
        d = delta[a.c == k]
        fa, fb = Fraction(1 + k), Fraction(1 + w.g0 - k)
        if d.max() > 0:
            taken.append(exact_gain(fa, fb, int(d.max()) - 1))
        avail.append(exact_gain(fa, fb, int(d.min())))
        assert d.max() - d.min() <= 1 and np.all(np.diff(d) <= 0)
    assert min(taken) >= max(avail)
