"""Seeded synthetic inputs for the HORA rollout-allocation path.

This module only draws random inputs (success probabilities, Phase-A correct
counts, rewards, response lengths) and packs them into arrays.  It holds none
of the method's arithmetic: no posterior, no gains, no allocation, no
advantages.  Both the test oracle and the HIP path are fed from here, so that
they see identical bytes.

The workloads have the shape of the paper's training step (Sec. 3.2, Alg. 1,
App. C): a batch of prompts with strongly bimodal per-prompt success rates,
G0 binary pre-rollout outcomes per prompt, binary accuracy rewards on the
pooled groups and bounded response lengths.  They stand in for the paper's
MATH12k / Qwen2.5 rollouts, which need model weights and a dataset.

Recipe (numpy ``Generator(PCG64(...))``, fixed draw order):

Phase A, stream ``PCG64(seed)``:
  1. ``u ~ U(0,1)^N`` picks the mixture component of every prompt;
  2. one full-length draw per Beta component, in the order the mixture lists
     them (point masses draw nothing); ``p_i`` is selected by the mask of 1;
  3. ``pre[N, G0] = (U(0,1) < p_i)``; ``c_i = sum_j pre[i, j]``.
Phase B, stream ``PCG64([seed, 0xB])`` (independent of how much Phase A drew),
given the allocation ``delta``:
  4. ``add = (U(0,1)^{sum delta} < p_i)`` repeated ``delta_i`` times per prompt,
     appended after the prompt's G0 pre-rollout rewards;
  5. one length per response, in response order.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Sequence, Tuple

import numpy as np

# Mixture components: ("point", value) or ("beta", a, b), each with a weight.
Component = Tuple


@dataclass(frozen=True)
class Workload:
    name: str
    n: int                      # prompts
    g0: int                     # pre-rollouts per prompt
    budget: int                 # Phase-B budget
    delta_max: int              # per-prompt cap, 0 = none
    mixture: Sequence[Tuple[float, Component]]
    lengths: Optional[Tuple]    # ("uniform", lo, hi) | ("lognormal", median, sigma, lo, hi) | None
    seed: int
    float_type: str = "f64"     # reward / advantage storage type
    token_type: str = "f32"     # per-token advantage type
    group_off_type: str = "i64"
    tok_off_type: str = "i64"
    modes: Tuple[str, ...] = ("grpo", "rloo")
    eps: float = 1e-6
    note: str = ""


_MIX_STD = ((0.30, ("point", 0.0)), (0.15, ("beta", 20.0, 1.0)), (0.55, ("beta", 0.5, 0.5)))
_MIX_SKEW = ((0.60, ("point", 0.0)), (0.40, ("beta", 0.3, 0.3)))
_MIX_ARCSINE = ((1.0, ("beta", 0.5, 0.5)),)

TINY = Workload("tiny", 512, 4, 2048, 0, _MIX_STD, ("uniform", 64, 512), 0,
                float_type="f64", token_type="f64", modes=("grpo", "rloo"))
SMALL = Workload("small", 8192, 8, 8 * 8192, 56, _MIX_STD,
                 ("lognormal", 800.0, 0.6, 32, 4096), 1,
                 float_type="f32", token_type="f32",
                 group_off_type="i32", tok_off_type="i32")
SKEWED = Workload("skewed", 65536, 2, 14 * 65536, 0, _MIX_SKEW, ("uniform", 16, 2048), 2,
                  float_type="f32", token_type="f32",
                  group_off_type="i32", tok_off_type="i32")
LARGE_ALLOC = Workload("large_alloc", 1 << 20, 4, 4 << 20, 0, _MIX_ARCSINE, None, 3,
                       group_off_type="i32")
LARGE_BCAST = Workload("large_bcast", 4096, 8, 8 * 4096, 0, _MIX_STD,
                       ("lognormal", 2048.0, 0.7, 128, 16384), 4,
                       float_type="f32", token_type="f32",
                       group_off_type="i32", tok_off_type="i64")

# The paper's own training step (App. C, Tables 3-5): 60 prompts, G0 = 8, G = 32, so a
# Phase-B budget of 60 * 24, allocated on four shards of 15 prompts.
PAPER_STEP = Workload("paper_step", 60, 8, 60 * 24, 0, _MIX_STD, ("lognormal", 800.0, 0.6, 32, 2048), 5,
                      float_type="f32", token_type="f32", group_off_type="i32", tok_off_type="i32",
                      note="4 shards of 15 prompts")
PAPER_STEP_SHARDS = 4
# The same shard shape at scale: 65 536 shards of 16 prompts, G0 = 8, 24 additional rollouts per prompt.
SHARDED_LARGE = Workload("sharded_large", 1 << 20, 8, 24 << 20, 0, _MIX_STD, None, 6, group_off_type="i32",
                         note="65536 shards of 16 prompts")
SHARDED_LARGE_SHARDS = 1 << 16

WORKLOADS = {w.name: w for w in (TINY, SMALL, SKEWED, LARGE_ALLOC, LARGE_BCAST, PAPER_STEP, SHARDED_LARGE)}


def equal_shards(n: int, n_shards: int, budget: int) -> Tuple[np.ndarray, np.ndarray]:
    """Consecutive shards of (almost) equal size with the budget split in proportion to
    the shard sizes (any remainder of the budget goes to the first shards, one unit each)."""
    bounds = (np.arange(n_shards + 1, dtype=np.int64) * n) // n_shards
    sizes = np.diff(bounds)
    per = budget // n if n else 0
    shard_budget = sizes * per
    rest = budget - int(shard_budget.sum())
    shard_budget[:rest] += 1
    return bounds, shard_budget.astype(np.int64)


def ragged_shards(n: int, n_shards: int, mean_per_prompt: float, seed: int
                  ) -> Tuple[np.ndarray, np.ndarray]:
    """Random consecutive shards (some empty) with random budgets; empty shards get none."""
    rng = np.random.Generator(np.random.PCG64([seed, 0x5A]))
    cuts = np.sort(rng.integers(0, n + 1, size=max(n_shards - 1, 0)))
    bounds = np.concatenate(([0], cuts, [n])).astype(np.int64)
    sizes = np.diff(bounds)
    shard_budget = rng.poisson(mean_per_prompt * sizes).astype(np.int64)
    shard_budget[sizes == 0] = 0
    return bounds, shard_budget


def scaled(w: Workload, n: int, name: Optional[str] = None) -> Workload:
    """Same recipe at ``n`` prompts, budget scaled in proportion."""
    per = w.budget // w.n
    return Workload(name or f"{w.name}_n{n}", n, w.g0, per * n, w.delta_max, w.mixture,
                    w.lengths, w.seed, w.float_type, w.token_type, w.group_off_type,
                    w.tok_off_type, w.modes, w.eps, w.note)


@dataclass
class PhaseA:
    p: np.ndarray       # float64 [N] true success probability (never shown to the method)
    pre: np.ndarray     # uint8 [N, G0] pre-rollout accuracy outcomes
    c: np.ndarray       # int32 [N] Phase-A correct counts


@dataclass
class PhaseB:
    group_off: np.ndarray   # int64 [N+1]
    reward: np.ndarray      # float64 [R], values in {0, 1} (or {0, .5, 1})
    lengths: Optional[np.ndarray]  # int64 [R]
    tok_off: Optional[np.ndarray]  # int64 [R+1]


def phase_a(w: Workload) -> PhaseA:
    rng = np.random.Generator(np.random.PCG64(w.seed))
    n = w.n
    u = rng.random(n)
    p = np.zeros(n, dtype=np.float64)
    lo = 0.0
    ncomp = len(w.mixture)
    for k, (weight, comp) in enumerate(w.mixture):
        hi = 1.0 if k == ncomp - 1 else lo + weight
        mask = (u >= lo) & (u < hi)
        if comp[0] == "point":
            vals = np.full(n, float(comp[1]))
        elif comp[0] == "beta":
            vals = rng.beta(comp[1], comp[2], n)
        else:
            raise ValueError(comp)
        p[mask] = vals[mask]
        lo = hi
    pre = (rng.random((n, w.g0)) < p[:, None]).astype(np.uint8)
    c = pre.sum(axis=1).astype(np.int32)
    return PhaseA(p=p, pre=pre, c=c)


def draw_lengths(spec: Tuple, count: int, rng: np.random.Generator) -> np.ndarray:
    if spec[0] == "uniform":
        _, lo, hi = spec
        return rng.integers(lo, hi + 1, size=count, dtype=np.int64)
    if spec[0] == "lognormal":
        _, median, sigma, lo, hi = spec
        x = rng.lognormal(np.log(median), sigma, size=count)
        return np.clip(np.rint(x), lo, hi).astype(np.int64)
    raise ValueError(spec)


def phase_b(w: Workload, a: PhaseA, delta: np.ndarray, *, half_rewards: bool = False,
            with_tokens: bool = True) -> PhaseB:
    """Rewards and lengths of the pooled groups for a given allocation.

    ``half_rewards`` draws a format bit as well and stores (fmt + acc) / 2, the
    training reward of Sec. 4 with values in {0, 1/2, 1}.
    """
    rng = np.random.Generator(np.random.PCG64([w.seed, 0xB]))
    delta = np.asarray(delta, dtype=np.int64)
    n, g0 = w.n, w.g0
    sizes = g0 + delta
    group_off = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(sizes, out=group_off[1:])
    r = int(group_off[-1])
    total_add = int(delta.sum())
    add = (rng.random(total_add) < np.repeat(a.p, delta)).astype(np.float64)
    reward = np.empty(r, dtype=np.float64)
    # position of every response inside its group
    gid = np.repeat(np.arange(n, dtype=np.int64), sizes)
    pos = np.arange(r, dtype=np.int64) - group_off[gid]
    is_pre = pos < g0
    reward[is_pre] = a.pre.reshape(-1).astype(np.float64)
    reward[~is_pre] = add
    if half_rewards:
        fmt = (rng.random(r) < 0.9).astype(np.float64)
        reward = (fmt + reward) / 2.0
    lengths = tok_off = None
    if with_tokens and w.lengths is not None:
        lengths = draw_lengths(w.lengths, r, rng)
        tok_off = np.zeros(r + 1, dtype=np.int64)
        np.cumsum(lengths, out=tok_off[1:])
    return PhaseB(group_off=group_off, reward=reward, lengths=lengths, tok_off=tok_off)


def np_float(t: str):
    return {"f32": np.float32, "f64": np.float64}[t]


def np_int(t: str):
    return {"i32": np.int32, "i64": np.int64}[t]
