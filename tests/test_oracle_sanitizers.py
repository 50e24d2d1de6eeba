"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

oracle/hora_oracle.c is built a second time with -fsanitize=address,undefined together with
oracle/sanitize_driver.c, which runs every oracle function on small seeded inputs whose
buffers have exactly the documented sizes.  The run must finish without a sanitizer report,
and what it prints must equal what the ordinary build returns for the same inputs."""
import os
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE_DIR = os.path.join(ROOT, "oracle")


class Lcg:
    def __init__(self):
        self.state = 0x9e3779b97f4a7c15

    def u32(self):
        self.state = (self.state * 6364136223846793005 + 1442695040888963407) & ((1 << 64) - 1)
        return self.state >> 33


def fmt_d(x):
    return " ".join(float(v).hex() for v in x)


def parse_d(tokens):
    return [float.fromhex(t) for t in tokens]


@pytest.fixture(scope="module")
def sanitizer_output(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fno-omit-frame-pointer",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           os.path.join(ORACLE_DIR, "hora_oracle.c"), os.path.join(ORACLE_DIR, "sanitize_driver.c"),
           "-o", exe, "-lm"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stderr[-4000:]
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-4000:]
    return run.stdout.splitlines()


def test_sanitizer_build_agrees_with_the_ordinary_build(oracle, sanitizer_output):
    lines = iter(sanitizer_output)
    rng = Lcg()

    def expect(tag):
        parts = next(lines).split()
        assert parts[0] == tag, (tag, parts[:3])
        return parts[1:]

    assert parse_d(expect("gains")) == oracle.marginal_gains(0.75, 3.25, 40).tolist()
    cases = [(0, 4, 0, 0, 1.0, 1.0), (1, 4, 0, 0, 1.0, 1.0), (1, 4, 9, 0, 1.0, 1.0), (7, 2, 30, 0, 0.5, 3.0),
             (12, 8, 40, 4, 2.0, 3.25), (12, 8, 48, 4, 1.0, 1.0), (5, 4, 21, 4, 1.0, 1.0), (33, 16, 100, 0, 1.0, 1.0)]
    for n, g0, budget, cap, a0, b0 in cases:
        c = np.array([rng.u32() % (g0 + 1) for _ in range(n)], dtype=np.int32)
        head = next(lines)
        assert head.startswith(f"case n={n} g0={g0} budget={budget} cap={cap} rc=0"), head
        status = next(lines)
        try:
            delta = oracle.allocate(c, g0, budget, delta_max=cap, alpha0=a0, beta0=b0)
        except oracle.OracleError as e:
            assert status == f"allocate rc={e.code} scan rc={e.code}"
            continue
        assert status == "allocate rc=0 scan rc=0"
        assert [int(t) for t in expect("delta")] == delta.tolist()
        assert [int(t) for t in expect("delta_scan")] == delta.tolist()
        alpha, beta = oracle.posterior(c, g0, a0, b0)
        assert parse_d(expect("util")) == oracle.utilities(alpha, beta, delta).tolist()
        first = int(delta[:n // 3].sum())
        assert next(lines) == "sharded rc=0"
        want = oracle.allocate_sharded(c, g0, [0, n // 3, n], [first, budget - first], delta_max=cap,
                                       alpha0=a0, beta0=b0)
        assert [int(t) for t in expect("delta_sharded")] == want.tolist()
        for rule, name in ((0, "uniform"), (1, "hard_first")):
            line = next(lines)
            try:
                want = oracle.allocate_baseline(c, budget, name, delta_max=cap)
            except oracle.OracleError as e:
                assert line == f"baseline rule={rule} rc={e.code}"
                continue
            assert line == f"baseline rule={rule} rc=0"
            assert [int(t) for t in expect("delta_rule")] == want.tolist()
        goff = oracle.group_offsets(delta, g0)
        assert [int(t) for t in expect("group_off")] == goff.tolist()
        r = int(goff[-1])
        reward = np.array([(rng.u32() % 3) * 0.5 for _ in range(r)])
        toff = np.concatenate(([0], np.cumsum([rng.u32() % 5 for _ in range(r)]))).astype(np.int64)
        adv = None
        for mode, name in enumerate(("grpo", "rloo", "center")):
            assert next(lines) == f"advantage mode={mode} rc=0"
            adv = oracle.group_advantage(goff, reward, name, eps=1e-6 if mode == 0 else 0.0)
            assert parse_d(expect("adv")) == adv.tolist()
        assert next(lines) == "broadcast rc=0"
        assert parse_d(expect("tok")) == oracle.token_broadcast(adv, toff).tolist()
        for const in (0.0, 2048.0):
            assert next(lines) == "weights rc=0"
            assert parse_d(expect("w")) == oracle.response_weights(goff, toff, const).tolist()
    assert next(lines, None) is None
