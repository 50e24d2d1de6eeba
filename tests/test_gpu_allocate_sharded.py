"""GPU parity of hora_allocate_sharded (App. C: Phase B on independent shards) against the
CPU oracle, through the C ABI: delta and group offsets bit for bit, utilities within 1e-12."""
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


def check_sharded(gpu, oracle, c, g0, bounds, budgets, delta_max=0, off_dtype="i64", check_util=True):
    sess, torch, hora = gpu
    print(f"sharded n={c.size} g0={g0} shards={budgets.size} budget={int(budgets.sum())} cap={delta_max}", flush=True)
    want = oracle.allocate_sharded(c, g0, bounds, budgets, delta_max=delta_max)
    tdt = {"i32": torch.int32, "i64": torch.int64}[off_dtype]
    got = sess.allocate_sharded(dev(torch, c), g0, dev(torch, bounds), dev(torch, budgets), delta_max=delta_max,
                                off_dtype=tdt)
    assert sess.status() == 0
    delta = got.delta.cpu().numpy().astype(np.int64)
    assert np.array_equal(delta, want), np.flatnonzero(delta != want)[:10]
    assert np.array_equal(got.group_off.cpu().numpy().astype(np.int64), oracle.group_offsets(want, g0))
    if check_util:
        alpha, beta = oracle.posterior(c, g0)
        np.testing.assert_allclose(got.util.cpu().numpy(), oracle.utilities(alpha, beta, want),
                                   rtol=UTIL_RTOL, atol=0)
    summ = got.summary.cpu().numpy().reshape(-1, 4)
    assert np.array_equal(summ[:, 1] + summ[:, 2], budgets)          # count_gt + tie_units = budget
    assert ((summ[:, 2] >= 0) & (summ[:, 2] <= np.maximum(summ[:, 3], 0))).all()
    return want


def test_paper_step_four_shards(gpu, oracle):
    from paper_2605_07114_amd import workloads as wl
    w = wl.PAPER_STEP
    a = wl.phase_a(w)
    bounds, budgets = wl.equal_shards(w.n, wl.PAPER_STEP_SHARDS, w.budget)
    assert budgets.tolist() == [360] * 4
    check_sharded(gpu, oracle, a.c, w.g0, bounds, budgets, off_dtype="i32")


def test_one_shard_equals_the_unsharded_call(gpu, oracle):
    from paper_2605_07114_amd import workloads as wl
    sess, torch, hora = gpu
    w = wl.TINY
    a = wl.phase_a(w)
    want = check_sharded(gpu, oracle, a.c, w.g0, np.array([0, w.n], dtype=np.int64),
                         np.array([w.budget], dtype=np.int64))
    whole = sess.allocate(dev(torch, a.c), w.g0, w.budget)
    assert np.array_equal(whole.delta.cpu().numpy().astype(np.int64), want)


@pytest.mark.parametrize("g0,n,n_shards,mean", [(4, 3000, 37, 4.0), (8, 2000, 150, 20.0), (2, 5000, 9, 14.0),
                                                 (16, 700, 25, 9.0)])
def test_ragged_shards_with_empty_ones(gpu, oracle, g0, n, n_shards, mean):
    from paper_2605_07114_amd import workloads as wl
    rng = np.random.default_rng(g0 * 1000 + n)
    c = rng.integers(0, g0 + 1, n).astype(np.int32)
    bounds, budgets = wl.ragged_shards(n, n_shards, mean, seed=n)
    check_sharded(gpu, oracle, c, g0, bounds, budgets)


def test_shards_larger_than_a_workgroup_and_cap(gpu, oracle):
    from paper_2605_07114_amd import workloads as wl
    w = wl.SMALL
    a = wl.phase_a(w)
    bounds, budgets = wl.equal_shards(w.n, 5, w.budget)           # 1638-prompt shards, several tiles each
    check_sharded(gpu, oracle, a.c, w.g0, bounds, budgets, delta_max=w.delta_max, off_dtype="i32")
    # a cap that binds: every prompt of a shard ends at the cap, or one short of it
    c = np.zeros(40, dtype=np.int32)
    check_sharded(gpu, oracle, c, 4, np.array([0, 10, 40], dtype=np.int64), np.array([30, 85], dtype=np.int64),
                  delta_max=3)


def test_degenerate_shards(gpu, oracle):
    sess, torch, hora = gpu
    # zero budgets everywhere; single-prompt shards; all prompts in one class
    c = np.array([0, 4, 2, 2, 1], dtype=np.int32)
    check_sharded(gpu, oracle, c, 4, np.array([0, 1, 2, 5], dtype=np.int64), np.array([0, 0, 0], dtype=np.int64))
    check_sharded(gpu, oracle, c, 4, np.array([0, 1, 2, 3, 4, 5], dtype=np.int64),
                  np.array([3, 0, 7, 1, 2], dtype=np.int64))
    check_sharded(gpu, oracle, np.full(100, 3, dtype=np.int32), 8, np.array([0, 50, 100], dtype=np.int64),
                  np.array([75, 1], dtype=np.int64))
    # no prompts at all
    empty = sess.allocate_sharded(dev(torch, np.zeros(0, dtype=np.int32)), 4,
                                  dev(torch, np.zeros(1, dtype=np.int64)), dev(torch, np.zeros(0, dtype=np.int64)))
    assert sess.status() == 0 and empty.group_off.cpu().numpy().tolist() == [0]


def test_bad_shard_data_is_reported_not_fatal(gpu, oracle):
    sess, torch, hora = gpu
    c = dev(torch, np.zeros(8, dtype=np.int32))

    def status_of(bounds, budgets, cap=0):
        sess.dev_status.zero_()
        sess.allocate_sharded(c, 4, dev(torch, np.array(bounds, dtype=np.int64)),
                              dev(torch, np.array(budgets, dtype=np.int64)), delta_max=cap)
        s = sess.status()
        sess.dev_status.zero_()
        return s

    assert status_of([0, 4, 7], [1, 1]) == hora.ERR_RANGE            # does not end at n
    assert status_of([0, 5, 3, 8], [1, 1, 1]) == hora.ERR_RANGE      # decreasing
    assert status_of([0, 4, 8], [1, -1]) == hora.ERR_RANGE           # negative budget
    assert status_of([0, 4, 4, 8], [1, 1, 1]) == hora.ERR_INFEASIBLE  # budget on an empty shard
    assert status_of([0, 4, 8], [13, 1], cap=3) == hora.ERR_INFEASIBLE
    assert status_of([0, 4, 8], [12, 1], cap=3) == 0


def test_sharded_large_workload(gpu, oracle):
    """65 536 shards of 16 prompts (the benchmark's sharded workload): delta and offsets."""
    from paper_2605_07114_amd import workloads as wl
    w = wl.SHARDED_LARGE
    a = wl.phase_a(w)
    bounds, budgets = wl.equal_shards(w.n, wl.SHARDED_LARGE_SHARDS, w.budget)
    check_sharded(gpu, oracle, a.c, w.g0, bounds, budgets, off_dtype="i32", check_util=False)


def test_wavefront_path_edges(gpu, oracle):
    """Cases that steer between the wavefront-per-shard kernel and the workgroup-per-shard code
    that takes what it leaves over."""
    from paper_2605_07114_amd import workloads as wl
    sess, torch, hora = gpu
    rng = np.random.default_rng(77)
    # a cap that is not a power of two: 9 * 56 table levels, the last block of levels is short
    w = wl.SMALL
    a = wl.phase_a(w)
    bounds, budgets = wl.equal_shards(w.n, 512, w.budget)
    check_sharded(gpu, oracle, a.c, w.g0, bounds, budgets, delta_max=w.delta_max, off_dtype="i32")
    # one shard far larger than a wavefront handles among many tiny ones (it goes on the left-over list)
    sizes = np.concatenate((np.full(50, 10), [2000], np.full(50, 10)))
    bounds = np.concatenate(([0], np.cumsum(sizes))).astype(np.int64)
    c = rng.integers(0, 9, int(bounds[-1])).astype(np.int32)
    budgets = (sizes * 12).astype(np.int64)
    check_sharded(gpu, oracle, c, 8, bounds, budgets)
    # allocations deeper than the table: two hard prompts take 1500 rollouts
    c = np.array([0, 0, 8, 8, 3, 0, 1], dtype=np.int32)
    check_sharded(gpu, oracle, c, 8, np.array([0, 4, 7], dtype=np.int64), np.array([1500, 40], dtype=np.int64))
    # budget of one unit, budget equal to the number of prompts, all prompts tied
    c = np.full(64, 2, dtype=np.int32)
    check_sharded(gpu, oracle, c, 4, np.array([0, 1, 33, 64], dtype=np.int64), np.array([1, 32, 5], dtype=np.int64))


def test_tables_follow_the_prior_between_calls(gpu, oracle):
    """The workspace keeps the gain tables of the last call: a change of prior, G0 or cap must rebuild them."""
    sess, torch, hora = gpu
    rng = np.random.default_rng(78)
    c = rng.integers(0, 5, 600).astype(np.int32)
    bounds = np.arange(0, 601, 20, dtype=np.int64)
    budgets = np.full(30, 70, dtype=np.int64)
    for alpha0, beta0, cap in ((1.0, 1.0, 0), (0.5, 2.0, 0), (1.0, 1.0, 0), (1.0, 1.0, 9), (3.0, 0.25, 9)):
        want = oracle.allocate_sharded(c, 4, bounds, budgets, delta_max=cap, alpha0=alpha0, beta0=beta0)
        got = sess.allocate_sharded(dev(torch, c), 4, dev(torch, bounds), dev(torch, budgets), alpha0=alpha0,
                                    beta0=beta0, delta_max=cap)
        assert sess.status() == 0
        assert np.array_equal(got.delta.cpu().numpy().astype(np.int64), want), (alpha0, beta0, cap)
        alpha, beta = oracle.posterior(c, 4, alpha0, beta0)
        np.testing.assert_allclose(got.util.cpu().numpy(), oracle.utilities(alpha, beta, want), rtol=UTIL_RTOL, atol=0)


def test_int32_offsets_that_overflow_are_reported(gpu):
    """With 32-bit offsets the total n*g0 + sum of budgets must stay below 2^31; the budgets are
    device data, so the overflow is found on the device and reported through dev_status."""
    sess, torch, hora = gpu
    n, g0, n_shards = 1 << 24, 63, 1 << 16
    rng = np.random.default_rng(79)
    c = dev(torch, rng.integers(0, g0 + 1, n).astype(np.int32))
    bounds = dev(torch, np.arange(0, n + 1, n // n_shards, dtype=np.int64))
    for per_shard, want_status in ((16000, 0), (16896, hora.ERR_RANGE)):
        total = n * g0 + n_shards * per_shard
        assert (total >= 1 << 31) == (want_status != 0)
        print(f"sharded int32 offsets: total {total}", flush=True)
        sess.dev_status.zero_()
        got = sess.allocate_sharded(c, g0, bounds, dev(torch, np.full(n_shards, per_shard, dtype=np.int64)),
                                    want_util=False, off_dtype=torch.int32, want_summary=False)
        assert sess.status() == want_status
        sess.dev_status.zero_()
        if want_status == 0:
            assert int(got.group_off[-1]) == total
            assert int(got.delta.sum(dtype=torch.int64)) == n_shards * per_shard
            widths = got.group_off[1:].to(torch.int64) - got.group_off[:-1].to(torch.int64)
            assert bool((widths == got.delta.to(torch.int64) + g0).all())


def test_prepared_call_repeats_the_paper_step(gpu, oracle):
    """hora.prepared marshals once; every call of what it returns is the same library call:
    outputs against the oracle after each of two calls (the second on changed counts in the
    same buffer), and an error status still raises."""
    from paper_2605_07114_amd import workloads as wl
    sess, torch, hora = gpu
    w = wl.PAPER_STEP
    a = wl.phase_a(w)
    bounds, budgets = wl.equal_shards(w.n, wl.PAPER_STEP_SHARDS, w.budget)
    c = dev(torch, a.c)
    so, sb = dev(torch, bounds), dev(torch, budgets)
    delta = torch.full((w.n,), -7, dtype=torch.int32, device="cuda:0")
    util = torch.full((w.n,), float("nan"), dtype=torch.float64, device="cuda:0")
    goff = torch.full((w.n + 1,), -7, dtype=torch.int32, device="cuda:0")
    ws = torch.zeros(hora.hora_allocate_sharded_workspace_bytes(budgets.size), dtype=torch.uint8, device="cuda:0")
    run = hora.prepared(hora.hora_allocate_sharded, c, w.g0, so, sb, delta, sess.dev_status, ws, util=util,
                        group_off=goff)
    torch.cuda.synchronize()
    assert int(delta[0].item()) == -7          # preparing launches nothing
    counts = a.c
    for call in range(2):
        print(f"prepared paper_step call {call}", flush=True)
        run()
        torch.cuda.synchronize()
        assert sess.status() == 0
        want = oracle.allocate_sharded(counts, w.g0, bounds, budgets)
        assert np.array_equal(delta.cpu().numpy().astype(np.int64), want)
        assert np.array_equal(goff.cpu().numpy().astype(np.int64), oracle.group_offsets(want, w.g0))
        alpha, beta = oracle.posterior(counts, w.g0)
        np.testing.assert_allclose(util.cpu().numpy(), oracle.utilities(alpha, beta, want), rtol=UTIL_RTOL, atol=0)
        counts = (w.g0 - counts).astype(np.int32)   # new Phase-A outcomes in the same device buffer
        c.copy_(dev(torch, counts))
    # a prepared call whose arguments the library rejects raises like the plain binding
    bad = hora.prepared(hora.hora_allocate_sharded, c, w.g0, so, sb, delta, sess.dev_status, ws[:256], util=util,
                        group_off=goff)
    with pytest.raises(hora.HoraError):
        bad()
