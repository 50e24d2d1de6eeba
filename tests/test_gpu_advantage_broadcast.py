"""GPU parity: hora_group_advantage and hora_token_broadcast against the CPU oracle,
through the C ABI (Sec. 3.1; Sec. 4 / App. E).  Tolerances: 1e-12 relative for binary64
outputs, 1e-6 for float outputs; the broadcast is a copy and must be bit-exact."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

RTOL64, RTOL32 = 1e-12, 1e-6


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2605_07114_amd import hora
    assert torch.cuda.is_available(), "these tests need the MI355X"
    hora.load_library()
    return hora.Session("cuda:0"), torch, hora


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def check_advantage(gpu, oracle, group_off, reward64, ftype, itype, mode, eps=0.0, ddof=0):
    sess, torch, hora = gpu
    fdt = {"f32": np.float32, "f64": np.float64}[ftype]
    idt = {"i32": np.int32, "i64": np.int64}[itype]
    reward = reward64.astype(fdt)
    want = oracle.group_advantage(group_off, reward.astype(np.float64), mode, eps=eps, ddof=ddof)
    m = {"grpo": hora.ADV_GRPO, "rloo": hora.ADV_RLOO, "center": hora.ADV_CENTER}[mode]
    print(f"group_advantage groups={group_off.size - 1} resp={reward.size} {ftype} {itype} {mode}", flush=True)
    got = sess.group_advantage(dev(torch, group_off.astype(idt)), dev(torch, reward), m, eps=eps, ddof=ddof)
    assert sess.status() == 0
    got = got.cpu().numpy()
    assert got.dtype == fdt
    if ftype == "f64":
        np.testing.assert_allclose(got, want, rtol=RTOL64, atol=RTOL64)   # |x-y| <= tol * max(1, |y|)
    else:
        np.testing.assert_allclose(got, want.astype(np.float32), rtol=RTOL32, atol=RTOL32)
    if mode == "grpo":
        assert np.array_equal(got == 0, want == 0)      # zero-variance groups are exactly zero
    else:
        assert np.all(got[want == 0] == 0)              # an exact zero of the definition stays one
        sizes = np.diff(group_off)
        first = reward[np.minimum(group_off[:-1], reward.size - 1)] if reward.size else reward
        gid = np.repeat(np.arange(sizes.size), sizes)
        flat = np.zeros(sizes.size, dtype=bool)
        if reward.size:
            flat = np.bincount(gid, weights=(reward != first[gid]), minlength=sizes.size) == 0
            assert np.all(got[flat[gid]] == 0)          # all-equal groups carry no advantage
    return got, want


@pytest.mark.parametrize("name", ["tiny", "small", "skewed", "large_bcast"])
def test_advantage_parity_on_the_workloads(gpu, oracle, name):
    from paper_2605_07114_amd import workloads as wl
    w = wl.WORKLOADS[name]
    a = wl.phase_a(w)
    delta = oracle.allocate(a.c, w.g0, w.budget, delta_max=w.delta_max)
    b = wl.phase_b(w, a, delta, with_tokens=False)
    # parity, then invariants on the GPU result (RLOO sums to zero per group; GRPO has zero group mean)
    sizes = np.diff(b.group_off)
    gid = np.repeat(np.arange(w.n), sizes)
    tol = 1e-5 if w.float_type == "f32" else 1e-11
    for mode in w.modes:
        got, _ = check_advantage(gpu, oracle, b.group_off, b.reward, w.float_type, w.group_off_type, mode,
                                 eps=w.eps)
        sums = np.bincount(gid, weights=got.astype(np.float64), minlength=w.n)
        assert np.abs(sums).max() <= tol * sizes.max()


def test_advantage_general_rewards_modes_and_types(gpu, oracle):
    rng = np.random.default_rng(31)
    # (mean sizes that take 1, 2, 4, 8, 16, 32 and 64 lanes per group: every cross-lane path of the kernel)
    for n_groups, lo, hi in ((1, 1, 1), (1, 700, 700), (257, 1, 3), (900, 2, 9), (5000, 1, 40), (400, 20, 80),
                             (300, 60, 160), (300, 30, 900), (6, 3000, 9000)):
        sizes = rng.integers(lo, hi + 1, n_groups)
        off = np.zeros(n_groups + 1, dtype=np.int64)
        np.cumsum(sizes, out=off[1:])
        reward = rng.normal(size=off[-1])
        for ftype in ("f64", "f32"):
            for itype in ("i32", "i64"):
                check_advantage(gpu, oracle, off, reward, ftype, itype, "rloo")
                for ddof in (0, 1):
                    for eps in (0.0, 1e-6):
                        check_advantage(gpu, oracle, off, reward, ftype, itype, "grpo", eps=eps, ddof=ddof)


def test_advantage_few_large_groups_among_small_ones(gpu, oracle):
    """The lanes per group follow the mean size; groups far above it take the path that re-reads
    what a lane's registers do not hold (one lane per group here, groups of up to 700)."""
    rng = np.random.default_rng(32)
    sizes = rng.integers(1, 4, 4000)
    sizes[[5, 1999, 3999]] = (700, 9, 130)
    off = np.zeros(sizes.size + 1, dtype=np.int64)
    np.cumsum(sizes, out=off[1:])
    reward = rng.integers(0, 2, off[-1]).astype(np.float64)
    for ftype in ("f64", "f32"):
        for mode in ("grpo", "rloo", "center"):
            check_advantage(gpu, oracle, off, reward, ftype, "i32", mode, eps=1e-6)


def test_advantage_edge_groups(gpu, oracle):
    # empty groups, singletons, zero-variance groups whose mean is not representable,
    # rewards in {0, 1/2, 1}
    off = np.array([0, 0, 1, 1, 4, 6, 6, 10, 13, 13], dtype=np.int64)
    reward = np.array([1.0, 0.1, 0.1, 0.1, 1.0, 1.0, 0.0, 0.5, 1.0, 0.5, 0.3, 0.3, 0.3])
    for ftype in ("f64", "f32"):
        for mode in ("grpo", "rloo"):
            for eps in (0.0, 1e-6):
                got, want = check_advantage(gpu, oracle, off, reward, ftype, "i64", mode, eps=eps)
                if mode == "grpo":
                    assert np.all(got[[0, 1, 2, 3, 4, 5, 10, 11, 12]] == 0)
    from paper_2605_07114_amd import workloads as wl
    w = wl.TINY
    a = wl.phase_a(w)
    delta = oracle.allocate(a.c, w.g0, w.budget)
    b = wl.phase_b(w, a, delta, half_rewards=True, with_tokens=False)
    for mode in ("grpo", "rloo"):
        check_advantage(gpu, oracle, b.group_off, b.reward, "f64", "i64", mode, eps=1e-6)


def test_saturated_groups_are_exactly_zero_in_every_mode(gpu, oracle):
    """All-correct groups of sizes for which (G-1) * fl(1/(G-1)) != 1 in binary64 (50, 99, 104, ...):
    a leave-one-out advantage formed with the reciprocal would leave 1e-16 in every token."""
    sizes = np.array([50, 99, 104, 108, 162, 188, 2, 7, 50], dtype=np.int64)
    off = lengths_to_off(sizes)
    reward = np.ones(off[-1])
    reward[off[7]:off[8]] = 0.0          # an all-wrong group
    reward[off[8]:] = 0.3                # all equal, not representable
    for ftype in ("f64", "f32"):
        for mode in ("rloo", "grpo", "center"):
            got, _ = check_advantage(gpu, oracle, off, reward, ftype, "i64", mode, eps=1e-6)
            assert np.all(got == 0)


def test_advantage_bad_offsets_are_reported(gpu):
    sess, torch, hora = gpu
    reward = torch.ones(10, dtype=torch.float64, device="cuda:0")
    for off in ([0, 4, 3, 10], [1, 4, 6, 10], [0, 4, 6, 9], [0, 4, 60, 10]):
        sess.group_advantage(torch.tensor(off, dtype=torch.int64, device="cuda:0"), reward, hora.ADV_GRPO)
        assert sess.status() == hora.ERR_RANGE
        sess.dev_status.zero_()


# ---------------------------------------------------------------------------------
# token broadcast
# ---------------------------------------------------------------------------------
def run_broadcast(gpu, adv, tok_off, out_dtype, itype, skew=0):
    sess, torch, hora = gpu
    idt = {"i32": np.int32, "i64": np.int64}[itype]
    total = int(tok_off[-1])
    tdt = {"f32": torch.float32, "f64": torch.float64}[out_dtype]
    buf = torch.full((total + skew + 5,), float("nan"), dtype=tdt, device="cuda:0")
    out = buf[skew:skew + total]
    print(f"token_broadcast resp={adv.size} tokens={total} {adv.dtype}->{out_dtype} {itype} skew={skew}", flush=True)
    sess.token_broadcast(dev(torch, adv), dev(torch, tok_off.astype(idt)), total, out=out)
    assert sess.status() == 0
    return buf


def check_broadcast(gpu, oracle, adv, tok_off, out_dtype="f32", itype="i64", skew=0):
    buf = run_broadcast(gpu, adv, tok_off, out_dtype, itype, skew)
    total = int(tok_off[-1])
    host = buf.cpu().numpy()
    ndt = {"f32": np.float32, "f64": np.float64}[out_dtype]
    want = oracle.token_broadcast(adv.astype(np.float64), tok_off).astype(ndt)
    assert np.array_equal(host[skew:skew + total], want)
    assert np.isnan(host[:skew]).all() and np.isnan(host[skew + total:]).all()   # nothing outside


def lengths_to_off(lengths):
    off = np.zeros(lengths.size + 1, dtype=np.int64)
    np.cumsum(lengths, out=off[1:])
    return off


def test_broadcast_parity_tiny_and_small(gpu, oracle):
    from paper_2605_07114_amd import workloads as wl
    for w in (wl.TINY, wl.SMALL):
        a = wl.phase_a(w)
        delta = oracle.allocate(a.c, w.g0, w.budget, delta_max=w.delta_max)
        b = wl.phase_b(w, a, delta)
        for mode in w.modes:
            adv = oracle.group_advantage(b.group_off, b.reward, mode, eps=w.eps)
            adv = adv.astype(wl.np_float(w.float_type))
            check_broadcast(gpu, oracle, adv, b.tok_off, out_dtype=w.token_type, itype=w.tok_off_type)


def test_broadcast_shapes_and_edges(gpu, oracle):
    rng = np.random.default_rng(41)
    cases = {
        "one token": np.array([1]),
        "one long response": np.array([200001]),
        "zero-length runs": np.concatenate([np.zeros(5000, dtype=np.int64), [3], np.zeros(4000, dtype=np.int64),
                                            rng.integers(0, 3, 30000), [70000], np.zeros(17, dtype=np.int64)]),
        "all empty but one": np.concatenate([np.zeros(100, dtype=np.int64), [1]]),
        "tiny segments": rng.integers(1, 4, 200000),          # > 2048 responses per tile
        "ones": np.ones(100000, dtype=np.int64),
        "mixed": rng.integers(0, 40000, 300),
        "ragged tail": np.array([16384 * 3 + 1]),
        "exact tiles": np.array([16384, 16384, 8192, 8192]),
        # 2..6 responses per 4 KiB row: short descriptors, wide ones and the search, side by side
        "a few per row": rng.integers(170, 520, 6000),
        "short and long mixed": np.where(rng.random(4000) < 0.5, rng.integers(100, 300, 4000),
                                         rng.integers(3000, 9000, 4000)),
    }
    for name, lengths in cases.items():
        off = lengths_to_off(lengths.astype(np.int64))
        adv = rng.normal(size=lengths.size)
        print("case:", name, flush=True)
        check_broadcast(gpu, oracle, adv, off, "f64", "i64")
        check_broadcast(gpu, oracle, adv.astype(np.float32), off, "f32", "i32")
        check_broadcast(gpu, oracle, adv, off, "f32", "i64")       # rounded once to float
    # output buffers that do not start on a 16-byte boundary
    lengths = rng.integers(0, 3000, 500)
    off = lengths_to_off(lengths)
    adv = rng.normal(size=500)
    for skew in (1, 2, 3):
        check_broadcast(gpu, oracle, adv.astype(np.float32), off, "f32", "i64", skew=skew)
    check_broadcast(gpu, oracle, adv, off, "f64", "i64", skew=1)
    # nothing to write
    sess, torch, hora = gpu
    sess.token_broadcast(dev(torch, adv[:3].astype(np.float32)), torch.zeros(4, dtype=torch.int64, device="cuda:0"), 0)
    assert sess.status() == 0


def check_broadcast2(gpu, oracle, adv_a, adv_b, tok_off, out_dtype="f32", itype="i64", skew=0):
    """Two streams in one pass against two runs of the oracle, bit for bit, with canaries around both outputs."""
    sess, torch, hora = gpu
    idt = {"i32": np.int32, "i64": np.int64}[itype]
    ndt = {"f32": np.float32, "f64": np.float64}[out_dtype]
    tdt = {"f32": torch.float32, "f64": torch.float64}[out_dtype]
    total = int(tok_off[-1])
    step = 16 // np.dtype(ndt).itemsize
    bufs = [torch.full((total + skew + 5 + step,), float("nan"), dtype=tdt, device="cuda:0") for _ in range(2)]
    # both outputs at the same address modulo 16
    starts = [skew + (-(b.data_ptr() // b.element_size()) % step) for b in bufs]
    outs = [b[s0:s0 + total] for b, s0 in zip(bufs, starts)]
    assert outs[0].data_ptr() % 16 == outs[1].data_ptr() % 16
    print(f"token_broadcast2 resp={adv_a.size} tokens={total} {adv_a.dtype}->{out_dtype} {itype} skew={skew}", flush=True)
    sess.token_broadcast2(dev(torch, adv_a), dev(torch, adv_b), dev(torch, tok_off.astype(idt)), total, out=outs)
    assert sess.status() == 0
    for buf, s0, adv in zip(bufs, starts, (adv_a, adv_b)):
        host = buf.cpu().numpy()
        want = oracle.token_broadcast(adv.astype(np.float64), tok_off).astype(ndt)
        assert np.array_equal(host[s0:s0 + total], want)
        assert np.isnan(host[:s0]).all() and np.isnan(host[s0 + total:]).all()


def test_two_stream_broadcast_matches_two_broadcasts(gpu, oracle):
    from paper_2605_07114_amd import workloads as wl
    sess, torch, hora = gpu
    for w in (wl.TINY, wl.SMALL, wl.LARGE_BCAST):
        a = wl.phase_a(w)
        delta = oracle.allocate(a.c, w.g0, w.budget, delta_max=w.delta_max)
        b = wl.phase_b(w, a, delta)
        fdt = wl.np_float(w.float_type)
        rloo = oracle.group_advantage(b.group_off, b.reward, "rloo").astype(fdt)
        grpo = oracle.group_advantage(b.group_off, b.reward, "grpo", eps=w.eps).astype(fdt)
        check_broadcast2(gpu, oracle, rloo, grpo, b.tok_off, out_dtype=w.token_type, itype=w.tok_off_type)
        # the loss weights of Sec. 3.2 as the second stream
        wts = oracle.response_weights(b.group_off, b.tok_off).astype(fdt)
        check_broadcast2(gpu, oracle, grpo, wts, b.tok_off, out_dtype=w.token_type, itype=w.tok_off_type)
    rng = np.random.default_rng(47)
    cases = {
        "one token": np.array([1]),
        "zero-length runs": np.concatenate([np.zeros(5000, dtype=np.int64), [3], np.zeros(4000, dtype=np.int64),
                                            rng.integers(0, 3, 30000), [70000], np.zeros(17, dtype=np.int64)]),
        "tiny segments": rng.integers(1, 4, 100000),
        "a few per row": rng.integers(170, 520, 6000),
        "short and long mixed": np.where(rng.random(4000) < 0.5, rng.integers(100, 300, 4000),
                                         rng.integers(3000, 9000, 4000)),
        "ragged tail": np.array([16384 * 3 + 1]),
    }
    for name, lengths in cases.items():
        off = lengths_to_off(lengths.astype(np.int64))
        x, y = rng.normal(size=lengths.size), rng.normal(size=lengths.size)
        print("case:", name, flush=True)
        check_broadcast2(gpu, oracle, x, y, off, "f64", "i64")
        check_broadcast2(gpu, oracle, x.astype(np.float32), y.astype(np.float32), off, "f32", "i32")
        check_broadcast2(gpu, oracle, x, y, off, "f32", "i64")
    lengths = rng.integers(0, 3000, 500)
    off = lengths_to_off(lengths)
    x, y = rng.normal(size=500), rng.normal(size=500)
    for skew in (1, 2, 3):
        check_broadcast2(gpu, oracle, x.astype(np.float32), y.astype(np.float32), off, "f32", "i64", skew=skew)
    check_broadcast2(gpu, oracle, x, y, off, "f64", "i64", skew=1)
    # outputs that do not share their alignment are refused (they would need two row grids)
    out = torch.zeros(int(off[-1]) + 8, dtype=torch.float32, device="cuda:0")
    with pytest.raises(hora.HoraError) as e:
        hora.hora_token_broadcast2(dev(torch, x.astype(np.float32)), dev(torch, y.astype(np.float32)),
                                   dev(torch, off), out[:int(off[-1])], out[1:int(off[-1]) + 1], int(off[-1]),
                                   sess.dev_status, sess.broadcast_workspace(2 * int(off[-1]), torch.float32))
    assert e.value.status == hora.ERR_INVALID_ARG


def test_broadcast_bad_offsets_are_reported(gpu):
    sess, torch, hora = gpu
    adv = torch.ones(3, dtype=torch.float32, device="cuda:0")
    out = torch.zeros(100, dtype=torch.float32, device="cuda:0")
    for off in ([0, 50, 40, 100], [5, 50, 60, 100], [0, 50, 60, 90]):
        sess.token_broadcast(adv, torch.tensor(off, dtype=torch.int64, device="cuda:0"), 100, out=out)
        assert sess.status() == hora.ERR_RANGE
        sess.dev_status.zero_()


@pytest.mark.parametrize("name", ["large_bcast", "skewed"])
def test_broadcast_full_size_every_token(gpu, oracle, name):
    """Full-size runs in the launch shape the benchmark times: the whole output is compared
    with the oracle element by element, in chunks of consecutive responses (the oracle works in
    binary64, so a chunk of 2^25 tokens is 256 MiB on the host), plus the canary outside."""
    from paper_2605_07114_amd import workloads as wl
    sess, torch, hora = gpu
    w = wl.WORKLOADS[name]
    a = wl.phase_a(w)
    delta = oracle.allocate(a.c, w.g0, w.budget, delta_max=w.delta_max)
    b = wl.phase_b(w, a, delta)
    adv = oracle.group_advantage(b.group_off, b.reward, "rloo").astype(np.float32)
    total = int(b.tok_off[-1])
    buf = run_broadcast(gpu, adv, b.tok_off, "f32", w.tok_off_type)
    assert bool(torch.isnan(buf[total:]).all())                # nothing beyond the last token
    r = adv.size
    chunk_tokens = 1 << 25
    j0, compared = 0, 0
    while j0 < r:
        j1 = int(np.searchsorted(b.tok_off, b.tok_off[j0] + chunk_tokens, side="right")) - 1
        j1 = min(max(j1, j0 + 1), r)
        t0, t1 = int(b.tok_off[j0]), int(b.tok_off[j1])
        want = oracle.token_broadcast(adv[j0:j1].astype(np.float64), b.tok_off[j0:j1 + 1] - t0)
        got = buf[t0:t1].cpu().numpy()
        assert np.array_equal(got, want.astype(np.float32)), (name, j0, j1)
        compared += t1 - t0
        print(f"  {name}: responses [{j0}, {j1}) tokens [{t0}, {t1}) equal", flush=True)
        j0 = j1
    assert compared == total
