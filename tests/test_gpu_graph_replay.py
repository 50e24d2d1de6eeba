"""The entry points only enqueue kernels on the caller's stream (no allocation, no copy, no
synchronisation), so a caller may record them into a HIP graph.  Here the whole path is
captured once and replayed with new inputs written into the same buffers; every replay is
checked against the CPU oracle, with eager work and synchronisations in between."""
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


@pytest.mark.parametrize("per_prompt", [False, True])
def test_whole_path_replayed_from_a_graph(gpu, oracle, per_prompt):
    sess, torch, hora = gpu
    rng = np.random.default_rng(7 + int(per_prompt))
    n, g0 = 5000, 8
    budget = 8 * n
    n_resp = n * g0 + budget
    lengths = rng.integers(0, 600, n_resp).astype(np.int64)
    tok_off_h = np.concatenate(([0], np.cumsum(lengths))).astype(np.int64)
    total = int(tok_off_h[-1])

    i32, f64, dev = torch.int32, torch.float64, "cuda:0"
    c = torch.zeros(n, dtype=i32, device=dev)
    alpha = torch.ones(n, dtype=f64, device=dev)
    beta = torch.ones(n, dtype=f64, device=dev)
    reward = torch.zeros(n_resp, dtype=f64, device=dev)
    tok_off = torch.from_numpy(tok_off_h).to(dev)
    delta = torch.empty(n, dtype=i32, device=dev)
    util = torch.empty(n, dtype=f64, device=dev)
    goff = torch.empty(n + 1, dtype=torch.int64, device=dev)
    adv = torch.empty(n_resp, dtype=f64, device=dev)
    tok_adv = torch.empty(total, dtype=f64, device=dev)
    ws = sess.workspace(n, g0)
    bws = sess.broadcast_workspace(total, f64)
    status = sess.dev_status
    status.zero_()

    def path():
        if per_prompt:
            hora.hora_allocate_posterior(alpha, beta, g0, budget, delta, status, ws, util=util, group_off=goff)
        else:
            hora.hora_allocate(c, g0, budget, delta, status, ws, util=util, group_off=goff)
        hora.hora_group_advantage(goff, reward, adv, hora.ADV_GRPO, status, eps=1e-6)
        hora.hora_token_broadcast(adv, tok_off, tok_adv, total, status, bws)

    def new_inputs():
        c_h = rng.binomial(g0, rng.beta(0.5, 0.5, n)).astype(np.int32)
        if per_prompt:
            s, p = rng.uniform(0.25, 16.0, n), rng.uniform(0.02, 0.98, n)
            a_h, b_h = s * p + c_h, s * (1 - p) + g0 - c_h
        else:
            a_h, b_h = 1.0 + c_h, 1.0 + g0 - c_h
        r_h = rng.integers(0, 2, n_resp).astype(np.float64)
        c.copy_(torch.from_numpy(c_h))
        alpha.copy_(torch.from_numpy(a_h))
        beta.copy_(torch.from_numpy(b_h))
        reward.copy_(torch.from_numpy(r_h))
        return a_h, b_h, r_h

    def check(a_h, b_h, r_h, what):
        torch.cuda.synchronize()
        assert int(status.item()) == 0, what
        want = oracle.allocate_posterior(a_h, b_h, budget)
        assert np.array_equal(delta.cpu().numpy().astype(np.int64), want), what
        off = oracle.group_offsets(want, g0)
        assert np.array_equal(goff.cpu().numpy(), off), what
        np.testing.assert_allclose(util.cpu().numpy(), oracle.utilities(a_h, b_h, want), rtol=1e-12, atol=0)
        want_adv = oracle.group_advantage(off, r_h, "grpo", eps=1e-6)
        np.testing.assert_allclose(adv.cpu().numpy(), want_adv, rtol=1e-12, atol=1e-12)
        got_adv = adv.cpu().numpy()
        assert np.array_equal(tok_adv.cpu().numpy(), oracle.token_broadcast(got_adv, tok_off_h)), what

    inputs = new_inputs()
    path()                                   # eager, also warms everything up before the capture
    check(*inputs, "eager")
    graph = torch.cuda.CUDAGraph()
    print(f"capturing the path (per-prompt posteriors: {per_prompt})", flush=True)
    with torch.cuda.graph(graph):
        path()
    for replay in range(4):
        inputs = new_inputs()
        tok_adv.fill_(float("nan"))          # eager work between the replays
        delta.zero_()
        torch.cuda.synchronize()
        print(f"replay {replay}", flush=True)
        graph.replay()
        check(*inputs, f"replay {replay}")
