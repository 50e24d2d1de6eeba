"""Repeated calls on the same inputs must give bit-identical outputs: the kernels use integer
atomics only where the order cannot matter, and floating-point sums run in a fixed order."""
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


def test_outputs_do_not_change_between_runs(gpu, oracle):
    from paper_2605_07114_amd import workloads as wl
    sess, torch, hora = gpu
    w = wl.SMALL
    a = wl.phase_a(w)
    c = torch.from_numpy(a.c).to("cuda:0")
    delta0 = oracle.allocate(a.c, w.g0, w.budget, delta_max=w.delta_max)
    b = wl.phase_b(w, a, delta0)
    goff = torch.from_numpy(b.group_off.astype(np.int32)).to("cuda:0")
    reward = torch.from_numpy(b.reward.astype(np.float32) + 0.125 * (np.arange(b.reward.size) % 7).astype(np.float32)).to("cuda:0")
    toff = torch.from_numpy(b.tok_off.astype(np.int32)).to("cuda:0")
    total = int(b.tok_off[-1])
    bounds, budgets = wl.equal_shards(w.n, 300, w.budget)
    so, sb = torch.from_numpy(bounds).to("cuda:0"), torch.from_numpy(budgets).to("cuda:0")
    alpha = torch.from_numpy(0.7 + a.c.astype(np.float64) * 1.3).to("cuda:0")
    beta = torch.from_numpy(1.9 + (w.g0 - a.c).astype(np.float64) * 0.8).to("cuda:0")

    def one_run():
        out = []
        for method in (hora.ALLOC_CLASS, hora.ALLOC_BISECT):
            r = sess.allocate(c, w.g0, w.budget, delta_max=w.delta_max, method=method)
            out += [r.delta, r.util, r.group_off, r.summary]
        r = sess.allocate_posterior(alpha, beta, w.g0, w.budget)
        out += [r.delta, r.util, r.group_off]
        r = sess.allocate_sharded(c, w.g0, so, sb, delta_max=w.delta_max)
        out += [r.delta, r.util, r.group_off, r.summary]
        for mode in (hora.ADV_GRPO, hora.ADV_RLOO, hora.ADV_CENTER):
            adv = sess.group_advantage(goff, reward, mode, eps=1e-6)
            out.append(adv)
        out.append(sess.token_broadcast(adv, toff, total))
        return [t.cpu().numpy().copy() for t in out]

    first = one_run()
    for rep in range(9):
        again = one_run()
        for x, y in zip(first, again):
            assert x.tobytes() == y.tobytes()
    assert sess.status() == 0
