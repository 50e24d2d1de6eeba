"""hora_allocate_static (the entry point for callers that cannot allocate) against
hora_allocate, through the C ABI: two calls in a row on the library's own device buffer,
the second with a smaller input, both allocation methods, outputs bit for bit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2605_07114_amd import hora
    assert torch.cuda.is_available(), "these tests need the MI355X"
    hora.load_library()
    return torch, hora


def run_both(torch, hora, c_host, g0, budget, method, delta_max=0, alpha0=1.0, beta0=1.0):
    n = c_host.size
    c = torch.from_numpy(c_host).to("cuda:0")
    status = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    outs = []
    for static in (False, True):
        delta = torch.full((n,), -7, dtype=torch.int32, device="cuda:0")
        util = torch.full((n,), float("nan"), dtype=torch.float64, device="cuda:0")
        goff = torch.full((n + 1,), -7, dtype=torch.int64, device="cuda:0")
        summary = torch.full((4,), -7, dtype=torch.int64, device="cuda:0")
        print(f"n={n} g0={g0} budget={budget} method={method} static={static}", flush=True)
        if static:
            hora.hora_allocate_static(c, g0, budget, delta, status, alpha0=alpha0, beta0=beta0, delta_max=delta_max,
                                      method=method, util=util, group_off=goff, summary=summary)
        else:
            ws = torch.zeros(hora.hora_allocate_workspace_bytes(n, g0), dtype=torch.uint8, device="cuda:0")
            hora.hora_allocate(c, g0, budget, delta, status, ws, alpha0=alpha0, beta0=beta0, delta_max=delta_max,
                               method=method, util=util, group_off=goff, summary=summary)
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        outs.append([t.cpu().numpy() for t in (delta, util, goff, summary)])
    for want, got in zip(*outs):
        assert np.array_equal(want.view(np.uint8), got.view(np.uint8))
    return outs[1][0]


def test_static_entry_point_matches_hora_allocate_on_two_calls_in_a_row(gpu, oracle):
    torch, hora = gpu
    rng = np.random.default_rng(77)
    for method in (hora.ALLOC_CLASS, hora.ALLOC_BISECT):
        # a batch of several tiles with a ragged tail, then a smaller one on the same buffer,
        # then one that a single workgroup handles
        for n, g0, per_prompt, cap in ((300_001, 8, 6, 0), (5_000, 4, 9, 12), (100, 4, 3, 0)):
            c = rng.binomial(g0, rng.beta(0.5, 0.5, n)).astype(np.int32)
            delta = run_both(torch, hora, c, g0, per_prompt * n, method, delta_max=cap, alpha0=0.5, beta0=2.0)
            if n <= 5_000:
                want = oracle.allocate(c, g0, per_prompt * n, delta_max=cap, alpha0=0.5, beta0=2.0)
                assert np.array_equal(delta, want)


def test_static_entry_point_rejects_what_does_not_fit(gpu):
    torch, hora = gpu
    lib = hora.load_library()
    import ctypes
    fake, status = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x2000)
    too_many = (1 << 22) + 1
    assert lib.hora_allocate_static(too_many, 4, fake, 1.0, 1.0, 8, 0, 0, fake, None, None, 0, None, status,
                                    None) == hora.ERR_UNSUPPORTED
    assert lib.hora_allocate_static(-1, 4, fake, 1.0, 1.0, 8, 0, 0, fake, None, None, 0, None, status,
                                    None) == hora.ERR_INVALID_ARG
