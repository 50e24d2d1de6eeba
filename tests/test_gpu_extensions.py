"""GPU parity, through the C ABI, of the entry points beyond the main path: centred
advantages, loss weights for variable-size groups (Sec. 3.1 / 3.2), the baseline allocation
rules of Sec. 5 Table 2, and the Pass@K estimator of Sec. 4 Eq. 6."""
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


def random_groups(rng, n_groups, lo=1, hi=40):
    sizes = rng.integers(lo, hi + 1, n_groups)
    off = np.zeros(n_groups + 1, dtype=np.int64)
    np.cumsum(sizes, out=off[1:])
    return sizes, off


def test_centred_advantage(gpu, oracle):
    sess, torch, hora = gpu
    rng = np.random.default_rng(41)
    sizes, off = random_groups(rng, 5000, lo=1, hi=70)
    r = rng.normal(size=off[-1])
    r[off[10]:off[11]] = 0.1                                  # an all-equal group
    want = oracle.group_advantage(off, r, "center")
    got = sess.group_advantage(dev(torch, off), dev(torch, r), hora.ADV_CENTER).cpu().numpy()
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    assert (got[off[10]:off[11]] == 0).all()
    r32 = r.astype(np.float32)
    want32 = oracle.group_advantage(off, r32.astype(np.float64), "center")
    got32 = sess.group_advantage(dev(torch, off.astype(np.int32)), dev(torch, r32), hora.ADV_CENTER).cpu().numpy()
    np.testing.assert_allclose(got32, want32, rtol=1e-6, atol=1e-6)
    assert sess.status() == 0


@pytest.mark.parametrize("name", ["tiny", "small", "large_bcast"])
def test_response_weights_and_their_broadcast(gpu, oracle, name):
    from paper_2605_07114_amd import workloads as wl
    sess, torch, hora = gpu
    w = wl.WORKLOADS[name]
    a = wl.phase_a(w)
    delta = oracle.allocate(a.c, w.g0, w.budget, delta_max=w.delta_max)
    b = wl.phase_b(w, a, delta)
    goff = dev(torch, b.group_off.astype(wl.np_int(w.group_off_type)))
    toff = dev(torch, b.tok_off.astype(wl.np_int(w.tok_off_type)))
    n_resp = b.reward.size
    for length_const in (0.0, 2048.0):
        want = oracle.response_weights(b.group_off, b.tok_off, length_const)
        w64 = torch.empty(n_resp, dtype=torch.float64, device="cuda:0")
        hora.hora_response_weights(goff, toff, w64, sess.dev_status, length_const=length_const)
        assert np.array_equal(w64.cpu().numpy(), want)                       # same two operations: bit-equal
        w32 = torch.empty(n_resp, dtype=torch.float32, device="cuda:0")
        hora.hora_response_weights(goff, toff, w32, sess.dev_status, length_const=length_const)
        assert np.array_equal(w32.cpu().numpy(), want.astype(np.float32))   # rounded once
    # the weight of every token: the broadcast of the per-response weights (here the last ones computed)
    total = int(b.tok_off[-1])
    if total < 5e7:
        tokw = sess.token_broadcast(w64, toff, total, out_dtype=torch.float64)
        want_tok = oracle.token_broadcast(oracle.response_weights(b.group_off, b.tok_off, 2048.0), b.tok_off)
        assert np.array_equal(tokw.cpu().numpy(), want_tok)
    assert sess.status() == 0


def test_response_weights_edges(gpu, oracle):
    sess, torch, hora = gpu
    goff = np.array([0, 3, 3, 5], dtype=np.int64)                 # an empty group
    toff = np.array([0, 10, 10, 40, 50, 80], dtype=np.int64)     # an empty response
    want = oracle.response_weights(goff, toff)
    out = torch.empty(5, dtype=torch.float64, device="cuda:0")
    hora.hora_response_weights(dev(torch, goff), dev(torch, toff), out, sess.dev_status)
    assert np.array_equal(out.cpu().numpy(), want) and sess.status() == 0
    bad = np.array([0, 10, 5, 40, 50, 80], dtype=np.int64)       # decreasing token offsets
    hora.hora_response_weights(dev(torch, goff), dev(torch, bad), out, sess.dev_status)
    assert sess.status() == hora.ERR_RANGE
    sess.dev_status.zero_()


@pytest.mark.parametrize("name", ["tiny", "small", "skewed", "large_alloc"])
@pytest.mark.parametrize("rule", ["uniform", "hard_first"])
def test_baseline_rules_on_the_workloads(gpu, oracle, name, rule):
    from paper_2605_07114_amd import workloads as wl
    sess, torch, hora = gpu
    w = wl.WORKLOADS[name]
    a = wl.phase_a(w)
    budget = w.budget + 3                                         # a remainder to hand out by index
    want = oracle.allocate_baseline(a.c, budget, rule)
    code = {"uniform": hora.RULE_UNIFORM, "hard_first": hora.RULE_HARD_FIRST}[rule]
    got = sess.allocate_baseline(dev(torch, a.c), w.g0, budget, code)
    assert sess.status() == 0
    delta = got.delta.cpu().numpy().astype(np.int64)
    assert np.array_equal(delta, want)
    assert np.array_equal(got.group_off.cpu().numpy(), oracle.group_offsets(want, w.g0))
    # hit utility of what the rule hands out: one value per (c, delta) pair
    alpha, beta = oracle.posterior(a.c, w.g0)
    key = a.c.astype(np.int64) * (int(want.max()) + 1) + want
    uniq, first = np.unique(key, return_index=True)
    util = got.util.cpu().numpy()
    np.testing.assert_allclose(util[first], oracle.utilities(alpha[first], beta[first], want[first]), rtol=1e-12, atol=0)
    assert np.array_equal(util, util[first][np.searchsorted(uniq, key)])
    # Prop. 1: no rule beats the hit-utility allocation on the objective of Eq. 4
    best = sess.allocate(dev(torch, a.c), w.g0, budget)
    assert float(best.util.sum()) >= float(got.util.sum()) - 1e-9 * w.n


def test_baseline_rules_edges(gpu, oracle):
    sess, torch, hora = gpu
    c = np.array([1, 2, 3, 4, 2], dtype=np.int32)                 # no prompt with c = 0: hard-first falls back
    for budget in (0, 3, 12):
        want = oracle.allocate_baseline(c, budget, "hard_first")
        got = sess.allocate_baseline(dev(torch, c), 4, budget, hora.RULE_HARD_FIRST)
        assert np.array_equal(got.delta.cpu().numpy().astype(np.int64), want)
    c = np.array([0, 1, 0, 2], dtype=np.int32)
    got = sess.allocate_baseline(dev(torch, c), 4, 6, hora.RULE_HARD_FIRST, delta_max=3)
    assert got.delta.cpu().numpy().tolist() == [3, 0, 3, 0] and sess.status() == 0
    sess.allocate_baseline(dev(torch, c), 4, 7, hora.RULE_HARD_FIRST, delta_max=3)   # two prompts cannot take 7
    assert sess.status() == hora.ERR_INFEASIBLE
    sess.dev_status.zero_()
    with pytest.raises(hora.HoraError):
        sess.allocate_baseline(dev(torch, c), 4, 13, hora.RULE_UNIFORM, delta_max=3)  # 13 > 4 * 3: host check


def test_pass_at_k(gpu, oracle):
    sess, torch, hora = gpu
    rng = np.random.default_rng(17)
    for n_pool, ks, n_problems in ((256, [1, 8, 16, 32, 64, 128, 256], 500),
                                   (1024, [1, 8, 16, 32, 64, 128, 256, 512, 1024], 60),
                                   (16, [1, 2, 16], 3000)):
        p = rng.beta(0.3, 0.6, n_problems)
        p[rng.random(n_problems) < 0.3] = 0.0
        c = rng.binomial(n_pool, p).astype(np.int32)
        n = np.full(n_problems, n_pool, dtype=np.int32)
        if n_pool == 16:
            n = rng.integers(16, 40, n_problems).astype(np.int32)   # mixed pool sizes
            c = np.minimum(c, n)
        want_per, want_mean = oracle.pass_at_k(n, c, ks)
        per = torch.empty(len(ks) * n_problems, dtype=torch.float64, device="cuda:0")
        mean = torch.empty(len(ks), dtype=torch.float64, device="cuda:0")
        ws = torch.empty(hora.hora_pass_at_k_workspace_bytes(n_problems, len(ks)), dtype=torch.uint8, device="cuda:0")
        hora.hora_pass_at_k(dev(torch, n), dev(torch, c), ks, mean, sess.dev_status, ws, per_problem=per)
        assert sess.status() == 0
        got = per.cpu().numpy().reshape(len(ks), n_problems)
        np.testing.assert_allclose(got, want_per, rtol=1e-12, atol=0)
        assert (got[want_per == 0] == 0).all() and (got[want_per == 1] == 1).all()
        np.testing.assert_allclose(mean.cpu().numpy(), want_mean, rtol=1e-12, atol=0)
    # a K larger than a pool, and c > n: reported, the value counts as 0
    n = np.array([8, 8], dtype=np.int32)
    mean = torch.empty(1, dtype=torch.float64, device="cuda:0")
    ws = torch.empty(hora.hora_pass_at_k_workspace_bytes(2, 1), dtype=torch.uint8, device="cuda:0")
    hora.hora_pass_at_k(dev(torch, n), dev(torch, np.array([1, 9], dtype=np.int32)), [4], mean, sess.dev_status, ws)
    assert sess.status() == hora.ERR_RANGE
    sess.dev_status.zero_()


def test_allocation_shares_per_class(gpu, oracle):
    """Sec. 4, allocation dynamics: prompts and Phase-B budget per value of c, against np.bincount on the
    oracle's allocation (integers, exact), for the batch and the sharded call."""
    from paper_2605_07114_amd import workloads as wl
    sess, torch, hora = gpu
    for w in (wl.TINY, wl.SMALL, wl.SKEWED, wl.LARGE_ALLOC, wl.PAPER_STEP):
        a = wl.phase_a(w)
        if w is wl.PAPER_STEP:
            bounds, budgets = wl.equal_shards(w.n, wl.PAPER_STEP_SHARDS, w.budget)
            want = oracle.allocate_sharded(a.c, w.g0, bounds, budgets)
            got = sess.allocate_sharded(dev(torch, a.c), w.g0, dev(torch, bounds), dev(torch, budgets))
        else:
            want = oracle.allocate(a.c, w.g0, w.budget, delta_max=w.delta_max)
            got = sess.allocate(dev(torch, a.c), w.g0, w.budget, delta_max=w.delta_max)
        count = torch.full((w.g0 + 1,), -1, dtype=torch.int64, device="cuda:0")
        budget = torch.full((w.g0 + 1,), -1, dtype=torch.int64, device="cuda:0")
        print(f"allocation_shares {w.name} n={w.n}", flush=True)
        hora.hora_allocation_shares(dev(torch, a.c), got.delta, w.g0, count, budget, sess.dev_status)
        assert sess.status() == 0
        assert np.array_equal(count.cpu().numpy(), np.bincount(a.c, minlength=w.g0 + 1))
        assert np.array_equal(budget.cpu().numpy(),
                              np.bincount(a.c, weights=want, minlength=w.g0 + 1).astype(np.int64))
        assert int(budget.sum()) == w.budget
    # nothing to count; data out of range is reported and left out
    count = torch.full((5,), -1, dtype=torch.int64, device="cuda:0")
    budget = torch.full((5,), -1, dtype=torch.int64, device="cuda:0")
    empty = torch.zeros(0, dtype=torch.int32, device="cuda:0")
    hora.hora_allocation_shares(empty, empty, 4, count, budget, sess.dev_status)
    assert sess.status() == 0 and not count.any() and not budget.any()
    c = dev(torch, np.array([0, 4, 9, 2, -1, 4], dtype=np.int32))
    d = dev(torch, np.array([3, 1, 5, 0, 2, 7], dtype=np.int32))
    hora.hora_allocation_shares(c, d, 4, count, budget, sess.dev_status)
    assert sess.status() == hora.ERR_RANGE
    sess.dev_status.zero_()
    assert count.cpu().tolist() == [1, 0, 1, 0, 2] and budget.cpu().tolist() == [3, 0, 0, 0, 8]
