"""ctypes front end of the C test oracle (``hora_oracle.c``).

TEST INFRASTRUCTURE, not the product: only ``tests/``, the smoke check and the
benchmark's CPU-baseline leg may import this.  The functions marshal numpy
arrays and call the C code; the method's arithmetic lives in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hora_oracle.c")
_LIB = os.path.join(_HERE, "libhora_oracle.so")
CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC"]

_lib = None

OK, ERR_INVALID, ERR_INFEASIBLE, ERR_NOMEM, ERR_RANGE = 0, -1, -2, -3, -4


class OracleError(RuntimeError):
    def __init__(self, code: int):
        super().__init__(f"oracle status {code}")
        self.code = code


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (always when ``force``, else when stale)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.run(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        d, i64, i32, p = ctypes.c_double, ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
        _lib.hora_oracle_marginal_gains.argtypes = [d, d, i64, p]
        _lib.hora_oracle_marginal_gains.restype = None
        _lib.hora_oracle_hit_utility.argtypes = [d, d, i64]
        _lib.hora_oracle_hit_utility.restype = d
        _lib.hora_oracle_posterior.argtypes = [i64, i32, p, d, d, p, p]
        _lib.hora_oracle_posterior.restype = ctypes.c_int
        for f in (_lib.hora_oracle_allocate, _lib.hora_oracle_allocate_scan):
            f.argtypes = [i64, p, p, i64, i64, p]
            f.restype = ctypes.c_int
        _lib.hora_oracle_allocate_sharded.argtypes = [i64, p, p, i64, p, p, i64, p]
        _lib.hora_oracle_allocate_sharded.restype = ctypes.c_int
        _lib.hora_oracle_group_offsets.argtypes = [i64, i32, p, p]
        _lib.hora_oracle_group_offsets.restype = None
        _lib.hora_oracle_group_advantage.argtypes = [i64, p, p, p, i32, d, i32]
        _lib.hora_oracle_group_advantage.restype = ctypes.c_int
        _lib.hora_oracle_token_broadcast.argtypes = [i64, p, p, p]
        _lib.hora_oracle_token_broadcast.restype = ctypes.c_int
        _lib.hora_oracle_response_weights.argtypes = [i64, p, p, d, p]
        _lib.hora_oracle_response_weights.restype = ctypes.c_int
        _lib.hora_oracle_allocate_baseline.argtypes = [i64, p, i64, i64, i32, p]
        _lib.hora_oracle_allocate_baseline.restype = ctypes.c_int
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _check(code: int):
    if code != OK:
        raise OracleError(code)


def marginal_gains(alpha: float, beta: float, count: int) -> np.ndarray:
    out = np.empty(count, dtype=np.float64)
    lib().hora_oracle_marginal_gains(alpha, beta, count, _ptr(out))
    return out


def hit_utility(alpha: float, beta: float, delta: int) -> float:
    return float(lib().hora_oracle_hit_utility(alpha, beta, int(delta)))


def posterior(c: np.ndarray, g0: int, alpha0: float = 1.0, beta0: float = 1.0
              ) -> Tuple[np.ndarray, np.ndarray]:
    c = np.ascontiguousarray(c, dtype=np.int32)
    alpha = np.empty(c.size, dtype=np.float64)
    beta = np.empty(c.size, dtype=np.float64)
    _check(lib().hora_oracle_posterior(c.size, g0, _ptr(c), alpha0, beta0, _ptr(alpha), _ptr(beta)))
    return alpha, beta


def allocate_posterior(alpha: np.ndarray, beta: np.ndarray, budget: int, delta_max: int = 0,
                       scan: bool = False) -> np.ndarray:
    alpha = np.ascontiguousarray(alpha, dtype=np.float64)
    beta = np.ascontiguousarray(beta, dtype=np.float64)
    assert alpha.shape == beta.shape and alpha.ndim == 1
    delta = np.empty(alpha.size, dtype=np.int64)
    f = lib().hora_oracle_allocate_scan if scan else lib().hora_oracle_allocate
    _check(f(alpha.size, _ptr(alpha), _ptr(beta), int(budget), int(delta_max), _ptr(delta)))
    return delta


def allocate(c: np.ndarray, g0: int, budget: int, delta_max: int = 0, alpha0: float = 1.0,
             beta0: float = 1.0, scan: bool = False) -> np.ndarray:
    alpha, beta = posterior(c, g0, alpha0, beta0)
    return allocate_posterior(alpha, beta, budget, delta_max, scan=scan)


def allocate_sharded(c: np.ndarray, g0: int, shard_off: np.ndarray, shard_budget: np.ndarray,
                     delta_max: int = 0, alpha0: float = 1.0, beta0: float = 1.0) -> np.ndarray:
    alpha, beta = posterior(c, g0, alpha0, beta0)
    shard_off = np.ascontiguousarray(shard_off, dtype=np.int64)
    shard_budget = np.ascontiguousarray(shard_budget, dtype=np.int64)
    assert shard_off.size == shard_budget.size + 1
    delta = np.zeros(alpha.size, dtype=np.int64)
    _check(lib().hora_oracle_allocate_sharded(alpha.size, _ptr(alpha), _ptr(beta), shard_budget.size,
                                              _ptr(shard_off), _ptr(shard_budget), int(delta_max), _ptr(delta)))
    return delta


def utilities(alpha: np.ndarray, beta: np.ndarray, delta: np.ndarray) -> np.ndarray:
    f = lib().hora_oracle_hit_utility
    return np.array([f(float(a), float(b), int(d)) for a, b, d in zip(alpha, beta, delta)],
                    dtype=np.float64)


def group_offsets(delta: np.ndarray, g0: int) -> np.ndarray:
    delta = np.ascontiguousarray(delta, dtype=np.int64)
    off = np.empty(delta.size + 1, dtype=np.int64)
    lib().hora_oracle_group_offsets(delta.size, g0, _ptr(delta), _ptr(off))
    return off


def group_advantage(group_off: np.ndarray, reward: np.ndarray, mode: str, eps: float = 0.0,
                    ddof: int = 0) -> np.ndarray:
    group_off = np.ascontiguousarray(group_off, dtype=np.int64)
    reward = np.ascontiguousarray(reward, dtype=np.float64)
    adv = np.zeros(reward.size, dtype=np.float64)
    m = {"grpo": 0, "rloo": 1, "center": 2}[mode]
    _check(lib().hora_oracle_group_advantage(group_off.size - 1, _ptr(group_off), _ptr(reward),
                                             _ptr(adv), m, float(eps), int(ddof)))
    return adv


def token_broadcast(adv: np.ndarray, tok_off: np.ndarray, out: Optional[np.ndarray] = None
                    ) -> np.ndarray:
    adv = np.ascontiguousarray(adv, dtype=np.float64)
    tok_off = np.ascontiguousarray(tok_off, dtype=np.int64)
    total = int(tok_off[-1]) if tok_off.size else 0
    if out is None:
        out = np.empty(total, dtype=np.float64)
    assert out.dtype == np.float64 and out.size >= total
    _check(lib().hora_oracle_token_broadcast(adv.size, _ptr(adv), _ptr(tok_off), _ptr(out)))
    return out


def response_weights(group_off: np.ndarray, tok_off: np.ndarray, length_const: float = 0.0) -> np.ndarray:
    group_off = np.ascontiguousarray(group_off, dtype=np.int64)
    tok_off = np.ascontiguousarray(tok_off, dtype=np.int64)
    weight = np.zeros(tok_off.size - 1, dtype=np.float64)
    _check(lib().hora_oracle_response_weights(group_off.size - 1, _ptr(group_off), _ptr(tok_off),
                                              float(length_const), _ptr(weight)))
    return weight


def allocate_baseline(c: np.ndarray, budget: int, rule: str, delta_max: int = 0) -> np.ndarray:
    c = np.ascontiguousarray(c, dtype=np.int32)
    delta = np.zeros(c.size, dtype=np.int64)
    _check(lib().hora_oracle_allocate_baseline(c.size, _ptr(c), int(budget), int(delta_max),
                                               {"uniform": 0, "hard_first": 1}[rule], _ptr(delta)))
    return delta


def pass_at_k(n_samples: np.ndarray, c: np.ndarray, ks) -> Tuple[np.ndarray, np.ndarray]:
    """Unbiased Pass@K estimator of Sec. 4, Eq. 6, by its definition in exact integer
    arithmetic: per problem 1 - C(N - c, K) / C(N, K), rounded once to binary64; the
    benchmark value is the mean over the problems (math.fsum, exactly rounded).
    Returns (per_problem[len(ks), n], mean[len(ks)])."""
    import math
    from fractions import Fraction
    n_samples = np.asarray(n_samples, dtype=np.int64)
    c = np.asarray(c, dtype=np.int64)
    assert n_samples.shape == c.shape and c.ndim == 1
    memo = {}
    per = np.zeros((len(ks), c.size), dtype=np.float64)
    for a, k in enumerate(ks):
        for i, (nn, cc) in enumerate(zip(n_samples.tolist(), c.tolist())):
            if not (0 <= cc <= nn and 1 <= k <= nn):
                raise OracleError(ERR_RANGE)
            key = (nn, cc, k)
            if key not in memo:
                memo[key] = float(1 - Fraction(math.comb(nn - cc, k), math.comb(nn, k)))
            per[a, i] = memo[key]
    mean = np.array([math.fsum(row) / c.size if c.size else 0.0 for row in per], dtype=np.float64)
    return per, mean
