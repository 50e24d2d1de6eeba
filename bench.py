#!/usr/bin/env python3
"""Benchmark of the HORA rollout path on one MI355X.

Metric: prompts allocated/s at N = 2^20 (workload "large_alloc": posterior -> gains ->
allocation -> utilities -> group offsets), and the per-token advantage broadcast in
GB/s against the HBM peak (workload "large_bcast": allocation -> RLOO and GRPO group
advantages -> token broadcast, whole path timed, broadcast kernel timed on its own).
Inputs are seeded synthetic arrays already resident in HBM when timing starts.

Prints one JSON line.  The CPU baseline is the test oracle, timed on this host.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published

# HBM bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE (KiB per dispatch, scaled by what
# the same counters read for a plain device copy of known size); the figures and the commands
# are in profiles/hbm_traffic_large_alloc_large_bcast.txt.  Set to None when a kernel named
# there changes.
TRAFFIC_BROADCAST_BYTES = 692395767     # k_row_desc + k_token_fill, large_bcast
TRAFFIC_ALLOCATE_BYTES = 25532911       # k_class_hist + k_class_write, large_alloc


def ensure_library():
    from paper_2605_07114_amd import build, hora
    if not os.path.exists(hora.LIB_PATH):
        build.build_library()
    return hora.load_library()


def timed(torch, fn, steps, warmup):
    """Wall-clock and HIP-event time of `steps` calls of fn on the current stream."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()
    for _ in range(steps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, start.elapsed_time(stop) * 1e-3


def per_launch_events(torch, fn, steps, warmup):
    """Average duration of one call of fn: HIP events around `steps` back-to-back calls,
    repeated a few times (mean and best of the repeats)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    means = []
    for _ in range(5):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(steps):
            fn()
        b.record()
        torch.cuda.synchronize()
        means.append(a.elapsed_time(b) / steps)
    return float(np.mean(means)) * 1e-3, float(np.min(means)) * 1e-3


def cpu_baseline(wl, oracle, w_alloc, a_alloc, bcast_inputs):
    """The oracle as it stands, single thread, on this host."""
    best = float("inf")
    reps = 2
    for _ in range(reps):
        t0 = time.perf_counter()
        oracle.allocate(a_alloc.c, w_alloc.g0, w_alloc.budget, delta_max=w_alloc.delta_max)
        best = min(best, time.perf_counter() - t0)
    out = {"value": w_alloc.n / best, "unit": "prompts/s", "cores": 1, "kind": "oracle",
           "sample": f"full {w_alloc.name} (N={w_alloc.n}, B={w_alloc.budget}): posterior + max-heap greedy, "
                     f"best of {reps}, {best:.3f} s per pass"}
    w_b, a_b = bcast_inputs                          # the oracle's own pass over the broadcast workload
    delta = oracle.allocate(a_b.c, w_b.g0, w_b.budget, delta_max=w_b.delta_max)
    b = wl.phase_b(w_b, a_b, delta)
    adv = oracle.group_advantage(b.group_off, b.reward, "rloo")
    n_resp = min(adv.size, 16384)                    # bounded sample of the broadcast workload
    sub_off = b.tok_off[:n_resp + 1]
    buf = np.empty(int(sub_off[-1]), dtype=np.float64)
    t0 = time.perf_counter()
    oracle.token_broadcast(adv[:n_resp], sub_off, out=buf)
    dt = time.perf_counter() - t0
    out["broadcast_GBps"] = buf.size * 8 / dt / 1e9
    out["broadcast_sample"] = f"first {n_resp} responses of large_bcast, {buf.size} tokens, binary64 stores"
    return out


def other_paths(torch, hora, wl, sess, a1, c1, w1, delta1, util1, goff1, ws, reps):
    """Timings of the entry points next to the headline path (HIP events, mean of `reps` calls)."""
    def mean_us(fn):
        return per_launch_events(torch, fn, reps, 2)[0] * 1e6

    out = {}
    # per-prompt posteriors (threshold search) on the large-allocation inputs
    alpha = torch.from_numpy(1.0 + a1.c.astype(np.float64)).to("cuda:0")
    beta = torch.from_numpy(1.0 + w1.g0 - a1.c.astype(np.float64)).to("cuda:0")
    us = mean_us(lambda: hora.hora_allocate_posterior(alpha, beta, w1.g0, w1.budget, delta1, sess.dev_status, ws,
                                                      util=util1, group_off=goff1))
    out["allocate_posterior_large_alloc"] = {"us_per_call": us, "prompts_per_s": w1.n / us * 1e6}
    # learned-prior posteriors (App. D: s in [0.25, 16], p in (0, 1), c ~ Binomial(8, p)), all distinct
    rng_p = np.random.Generator(np.random.PCG64(13))
    s_ = rng_p.uniform(0.25, 16.0, w1.n)
    p_ = rng_p.uniform(0.02, 0.98, w1.n)
    c_ = rng_p.binomial(8, p_)
    alpha_l = torch.from_numpy(s_ * p_ + c_).to("cuda:0")
    beta_l = torch.from_numpy(s_ * (1 - p_) + 8 - c_).to("cuda:0")
    us = mean_us(lambda: hora.hora_allocate_posterior(alpha_l, beta_l, 8, 8 * w1.n, delta1, sess.dev_status, ws,
                                                      util=util1, group_off=goff1))
    assert int(delta1.sum()) == 8 * w1.n
    out["allocate_posterior_learned_prior_2^20"] = {"budget": 8 * w1.n, "us_per_call": us,
                                                    "prompts_per_s": w1.n / us * 1e6}
    # the same posteriors at the sizes of one training step and up (B = 8N): one workgroup alone, one
    # tile in one launch, the six launches
    sweep = []
    for n_s in (60, 256, 1024, 4096, 1 << 16, 1 << 18):
        us = mean_us(lambda: hora.hora_allocate_posterior(alpha_l[:n_s], beta_l[:n_s], 8, 8 * n_s, delta1[:n_s],
                                                          sess.dev_status, ws, util=util1[:n_s],
                                                          group_off=goff1[:n_s + 1]))
        assert int(delta1[:n_s].sum()) == 8 * n_s
        sweep.append({"n": n_s, "us_per_call": us})
    out["allocate_posterior_learned_prior_sweep"] = sweep
    # a deep budget: 200 additional rollouts per prompt on average, 2^18 prompts
    n_deep = 1 << 18
    us = mean_us(lambda: hora.hora_allocate_posterior(alpha[:n_deep], beta[:n_deep], w1.g0, 200 * n_deep,
                                                      delta1[:n_deep], sess.dev_status, ws, util=util1[:n_deep],
                                                      group_off=goff1[:n_deep + 1]))
    out["allocate_posterior_deep_budget_2^18"] = {"budget": 200 * n_deep, "max_delta": int(delta1[:n_deep].max()),
                                                  "us_per_call": us, "prompts_per_s": n_deep / us * 1e6}
    del alpha_l, beta_l
    # sharded Phase B: the paper's own step (4 shards of 15 prompts) and the same shard shape at scale
    for w, n_shards in ((wl.PAPER_STEP, wl.PAPER_STEP_SHARDS), (wl.SHARDED_LARGE, wl.SHARDED_LARGE_SHARDS)):
        a = wl.phase_a(w)
        bounds, budgets = wl.equal_shards(w.n, n_shards, w.budget)
        c = torch.from_numpy(a.c).to("cuda:0")
        so, sb = torch.from_numpy(bounds).to("cuda:0"), torch.from_numpy(budgets).to("cuda:0")
        delta = torch.empty(w.n, dtype=torch.int32, device="cuda:0")
        util = torch.empty(w.n, dtype=torch.float64, device="cuda:0")
        goff = torch.empty(w.n + 1, dtype=torch.int32, device="cuda:0")
        sws = torch.zeros(hora.hora_allocate_sharded_workspace_bytes(n_shards), dtype=torch.uint8, device="cuda:0")
        us = mean_us(lambda: hora.hora_allocate_sharded(c, w.g0, so, sb, delta, sess.dev_status, sws, util=util,
                                                        group_off=goff))
        assert int(delta.sum()) == w.budget
        out[f"allocate_sharded_{w.name}"] = {"shards": n_shards, "prompts": w.n, "us_per_call": us,
                                             "prompts_per_s": w.n / us * 1e6}
        # the same call with the Python-side checks and conversions done once (hora.prepared): a
        # call on a few dozen prompts is bound by them, not by its one kernel
        run = hora.prepared(hora.hora_allocate_sharded, c, w.g0, so, sb, delta, sess.dev_status, sws, util=util,
                            group_off=goff)
        delta.zero_()
        us_p = mean_us(run)
        assert int(delta.sum()) == w.budget and sess.status() == 0
        out[f"allocate_sharded_{w.name}"]["us_per_prepared_call"] = us_p
        if w is wl.PAPER_STEP:
            # the step's batch as one shard (the unsharded optimum of the same 60 prompts), next to
            # hora_allocate on it: the sharded call keeps its gain tables from call to call and is one launch
            one_off = torch.tensor([0, w.n], dtype=torch.int64, device="cuda:0")
            one_bud = torch.tensor([w.budget], dtype=torch.int64, device="cuda:0")
            us_1 = mean_us(lambda: hora.hora_allocate_sharded(c, w.g0, one_off, one_bud, delta, sess.dev_status, sws,
                                                              util=util, group_off=goff))
            by_shard = delta.clone()
            ws_small = sess.workspace(w.n, w.g0)
            us_a = mean_us(lambda: hora.hora_allocate(c, w.g0, w.budget, delta, sess.dev_status, ws_small, util=util,
                                                      group_off=goff))
            assert torch.equal(by_shard, delta) and sess.status() == 0
            out["allocate_paper_step_as_one_batch"] = {"prompts": w.n, "us_per_call_sharded_one_shard": us_1,
                                                       "us_per_call_hora_allocate": us_a}
    # the helpers next to the path, on the large-broadcast shapes: loss weights, baseline rule, Pass@K
    w2 = wl.LARGE_BCAST
    a2 = wl.phase_a(w2)
    c2 = torch.from_numpy(a2.c).to("cuda:0")
    alloc2 = sess.allocate(c2, w2.g0, w2.budget, off_dtype=torch.int32, want_util=False, want_summary=False)
    b2 = wl.phase_b(w2, a2, alloc2.delta.cpu().numpy())
    toff2 = torch.from_numpy(b2.tok_off).to("cuda:0")
    wts = torch.empty(b2.reward.size, dtype=torch.float32, device="cuda:0")
    us = mean_us(lambda: hora.hora_response_weights(alloc2.group_off, toff2, wts, sess.dev_status))
    out["response_weights_large_bcast"] = {"responses": int(b2.reward.size), "us_per_call": us}
    # group advantages far beyond the paper's sizes: 2^20 groups of 8..24 responses, binary rewards
    rng_g = np.random.Generator(np.random.PCG64(11))
    sizes = rng_g.integers(8, 25, 1 << 20)
    goff_big = torch.from_numpy(np.concatenate(([0], np.cumsum(sizes))).astype(np.int32)).to("cuda:0")
    n_big = int(goff_big[-1])
    for dt, tag in ((torch.float32, ""), (torch.float64, "_f64")):
        rew_big = (torch.rand(n_big, device="cuda:0") < 0.4).to(dt)
        adv_big = torch.empty_like(rew_big)
        size = rew_big.element_size()
        for mode, name in ((hora.ADV_GRPO, "grpo"), (hora.ADV_RLOO, "rloo")):
            us = mean_us(lambda: hora.hora_group_advantage(goff_big, rew_big, adv_big, mode, sess.dev_status, eps=1e-6))
            gbps = (2 * size * n_big + 4 * (sizes.size + 1)) / us / 1e3
            out[f"group_advantage_{name}_2^20_groups{tag}"] = {"responses": n_big, "us_per_call": us, "GBps": gbps,
                                                               "frac_of_hbm_peak": gbps / 8000.0}
        us = mean_us(lambda: adv_big.copy_(rew_big))      # a plain copy of the same rewards, for comparison
        out[f"plain_copy_of_the_rewards{tag}"] = {"us_per_call": us, "GBps": 2 * size * n_big / us / 1e3}
        del rew_big, adv_big
    del goff_big
    us = mean_us(lambda: hora.hora_allocate_baseline(c1, w1.g0, w1.budget, hora.RULE_HARD_FIRST, delta1,
                                                     sess.dev_status, ws, util=util1, group_off=goff1))
    out["allocate_hard_first_large_alloc"] = {"us_per_call": us, "prompts_per_s": w1.n / us * 1e6}
    rng = np.random.Generator(np.random.PCG64(7))
    n_prob, pool, ks = 500, 256, [1, 8, 16, 32, 64, 128, 256]       # the paper's MATH500 evaluation shape
    corr = torch.from_numpy(rng.binomial(pool, rng.beta(0.5, 0.5, n_prob)).astype(np.int32)).to("cuda:0")
    pools = torch.full((n_prob,), pool, dtype=torch.int32, device="cuda:0")
    mean = torch.empty(len(ks), dtype=torch.float64, device="cuda:0")
    pws = torch.empty(hora.hora_pass_at_k_workspace_bytes(n_prob, len(ks)), dtype=torch.uint8, device="cuda:0")
    us = mean_us(lambda: hora.hora_pass_at_k(pools, corr, ks, mean, sess.dev_status, pws))
    out["pass_at_k_500_problems_256_samples_7_ks"] = {"us_per_call": us}
    assert sess.status() == 0
    return out


def allocation_sweep(torch, hora, sess, reps):
    """hora_allocate (delta, utility, int32 offsets) at growing batch sizes, next to a plain stream of the
    same shape: one elementwise kernel that reads 4 bytes and writes 16 per element (torch's int32 ->
    complex128 copy)."""
    rows = []
    rng = np.random.Generator(np.random.PCG64(17))
    for lg in (20, 22, 24, 26):
        n = 1 << lg
        c = torch.from_numpy(rng.binomial(4, rng.beta(0.5, 0.5, n)).astype(np.int32)).to("cuda:0")
        delta = torch.empty(n, dtype=torch.int32, device="cuda:0")
        util = torch.empty(n, dtype=torch.float64, device="cuda:0")
        goff = torch.empty(n + 1, dtype=torch.int32, device="cuda:0")
        plain = torch.empty(n, dtype=torch.complex128, device="cuda:0")
        ws = sess.workspace(n, 4)
        t = per_launch_events(torch, lambda: hora.hora_allocate(c, 4, 4 * n, delta, sess.dev_status, ws, util=util,
                                                                group_off=goff), reps, 3)[0]
        tp = per_launch_events(torch, lambda: plain.copy_(c), reps, 3)[0]
        rows.append({"n": n, "us_per_call": t * 1e6, "GBps": 20 * n / t / 1e9, "plain_stream_us": tp * 1e6,
                     "plain_stream_GBps": 20 * n / tp / 1e9, "frac_of_plain_stream": tp / t})
        del c, delta, util, goff, plain
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--skip-extras", action="store_true",
                    help="leave out the size sweep and the entry points next to the headline path (counter runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device copy of the token buffer (known size), for scaling HBM counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import torch
    if not torch.cuda.is_available():
        print("bench.py needs the GPU (there is no CPU fallback)", file=sys.stderr)
        return 2
    ensure_library()
    from paper_2605_07114_amd import hora, workloads as wl
    torch.cuda.set_device(0)
    sess = hora.Session("cuda:0")
    steps, warmup = args.steps, args.warmup

    # ---- workload 1: large allocation (N = 2^20, G0 = 4, B = 4N, no cap) -------------------
    w1 = wl.LARGE_ALLOC
    a1 = wl.phase_a(w1)
    c1 = torch.from_numpy(a1.c).to("cuda:0")
    delta1 = torch.empty(w1.n, dtype=torch.int32, device="cuda:0")
    util1 = torch.empty(w1.n, dtype=torch.float64, device="cuda:0")
    goff1 = torch.empty(w1.n + 1, dtype=torch.int32, device="cuda:0")
    ws = sess.workspace(w1.n, w1.g0)

    def step_alloc():
        hora.hora_allocate(c1, w1.g0, w1.budget, delta1, sess.dev_status, ws, util=util1, group_off=goff1)

    wall1, ev1 = timed(torch, step_alloc, steps, warmup)
    assert sess.status() == 0 and int(delta1.sum()) == w1.budget
    alloc_bytes = w1.n * (4 + 4 + 8 + 4)      # c in; delta, util, group_off out
    ms_alloc = wall1 / steps * 1e3

    # ---- workload 2: large broadcast (N = 4096, G0 = 8, B = 8N; ~1.7e8 tokens) ---------------
    w2 = wl.LARGE_BCAST
    a2 = wl.phase_a(w2)
    c2 = torch.from_numpy(a2.c).to("cuda:0")
    alloc2 = sess.allocate(c2, w2.g0, w2.budget, off_dtype=torch.int32, want_util=False, want_summary=False)
    b2 = wl.phase_b(w2, a2, alloc2.delta.cpu().numpy())
    n_resp, n_tok = b2.reward.size, int(b2.tok_off[-1])
    reward2 = torch.from_numpy(b2.reward.astype(np.float32)).to("cuda:0")
    tok_off2 = torch.from_numpy(b2.tok_off).to("cuda:0")                     # packed int64 offsets
    delta2 = torch.empty(w2.n, dtype=torch.int32, device="cuda:0")
    goff2 = torch.empty(w2.n + 1, dtype=torch.int32, device="cuda:0")
    adv_rloo = torch.empty(n_resp, dtype=torch.float32, device="cuda:0")
    adv_grpo = torch.empty(n_resp, dtype=torch.float32, device="cuda:0")
    tok_rloo = torch.empty(n_tok, dtype=torch.float32, device="cuda:0")
    tok_grpo = torch.empty(n_tok, dtype=torch.float32, device="cuda:0")
    bws = sess.broadcast_workspace(n_tok, torch.float32)
    bws2 = torch.empty(hora.hora_token_broadcast2_workspace_bytes(n_tok, torch.float32), dtype=torch.uint8,
                       device="cuda:0")

    def step_path():            # both estimators' token streams written in one pass over the offsets
        hora.hora_allocate(c2, w2.g0, w2.budget, delta2, sess.dev_status, ws, group_off=goff2)
        hora.hora_group_advantage(goff2, reward2, adv_rloo, hora.ADV_RLOO, sess.dev_status)
        hora.hora_group_advantage(goff2, reward2, adv_grpo, hora.ADV_GRPO, sess.dev_status, eps=w2.eps)
        hora.hora_token_broadcast2(adv_rloo, adv_grpo, tok_off2, tok_rloo, tok_grpo, n_tok, sess.dev_status, bws2)

    def step_path_two_calls():  # the same with one broadcast per estimator
        hora.hora_allocate(c2, w2.g0, w2.budget, delta2, sess.dev_status, ws, group_off=goff2)
        hora.hora_group_advantage(goff2, reward2, adv_rloo, hora.ADV_RLOO, sess.dev_status)
        hora.hora_group_advantage(goff2, reward2, adv_grpo, hora.ADV_GRPO, sess.dev_status, eps=w2.eps)
        hora.hora_token_broadcast(adv_rloo, tok_off2, tok_rloo, n_tok, sess.dev_status, bws)
        hora.hora_token_broadcast(adv_grpo, tok_off2, tok_grpo, n_tok, sess.dev_status, bws)

    steps2 = max(steps // 4, 10)
    wall2, ev2 = timed(torch, step_path, steps2, max(warmup // 4, 3))
    wall2b, _ = timed(torch, step_path_two_calls, steps2, max(warmup // 4, 3))
    assert sess.status() == 0

    def dual_broadcast():
        hora.hora_token_broadcast2(adv_rloo, adv_grpo, tok_off2, tok_rloo, tok_grpo, n_tok, sess.dev_status, bws2)

    dual_mean, dual_min = per_launch_events(torch, dual_broadcast, steps2, 3)
    dual_bytes = 8 * n_tok + n_resp * (8 + 4 + 4)    # two float streams out; offsets and two advantages in

    def one_broadcast():
        hora.hora_token_broadcast(adv_rloo, tok_off2, tok_rloo, n_tok, sess.dev_status, bws)

    bc_mean, bc_min = per_launch_events(torch, one_broadcast, steps2, 3)
    # what a plain fill of the same buffer reaches in the same run (torch's fill kernel)
    fill_mean, _ = per_launch_events(torch, lambda: tok_grpo.zero_(), steps2, 3)
    fill_gbs = 4 * n_tok / fill_mean / 1e9
    if args.calibrate_copy:          # reads and writes 4 * n_tok bytes each
        tok_grpo.copy_(tok_rloo)
        torch.cuda.synchronize()
    bcast_bytes = 4 * n_tok + n_resp * (8 + 4)       # float stores; offsets and advantages in
    bcast_gbs = bcast_bytes / bc_mean / 1e9

    # what a plain stream of the allocation's shape reaches in the same run: one elementwise kernel that
    # reads 4 bytes and writes 16 per prompt (torch's int32 -> complex128 copy)
    plain1 = torch.empty(w1.n, dtype=torch.complex128, device="cuda:0")
    plain_mean, _ = per_launch_events(torch, lambda: plain1.copy_(c1), steps, 3)
    alloc_mean, alloc_min = per_launch_events(torch, step_alloc, steps, 3)
    del plain1
    sweep, extras = None, None
    if not args.skip_extras:
        sweep = allocation_sweep(torch, hora, sess, max(steps // 10, 5))
        ws = sess.workspace(w1.n, w1.g0)
        extras = other_paths(torch, hora, wl, sess, a1, c1, w1, delta1, util1, goff1, ws, max(steps // 10, 5))

    result = {
        "metric": "prompts allocated/s at N=1M; advantage broadcast GB/s as % of HBM peak",
        "value": w1.n / (wall1 / steps),
        "unit": "prompts/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms_alloc,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": {
            "workload": f"large_alloc: N={w1.n} prompts, G0={w1.g0}, budget={w1.budget}, no cap, "
                        "c ~ Binomial(G0, p), p ~ Beta(0.5, 0.5); outputs int32 delta, f64 utility, int32 group offsets",
            "method": "class histogram + threshold solve + index-ordered tie pass",
            "event_ms_per_step": ev1 / steps * 1e3,
        },
        "broadcast": {
            "workload": f"large_bcast: N={w2.n}, G0={w2.g0}, budget={w2.budget}, {n_resp} responses, "
                        f"{n_tok} tokens, int64 packed offsets, f32 token advantages",
            "GBps": bcast_gbs,
            "pct_of_hbm_peak": 100.0 * bcast_gbs / HBM_PEAK_GBS,
            "plain_fill_GBps": fill_gbs,
            "pct_of_plain_fill": 100.0 * bcast_gbs / fill_gbs,
            "kernel_ms_mean": bc_mean * 1e3,
            "kernel_ms_min": bc_min * 1e3,
            "whole_path_ms_per_step": wall2 / steps2 * 1e3,
            "whole_path": "allocate + RLOO and GRPO group advantages + one two-stream token broadcast",
            "tokens_per_s_whole_path": 2 * n_tok / (wall2 / steps2),
            "whole_path_two_broadcast_calls_ms_per_step": wall2b / steps2 * 1e3,
            "two_stream": {
                "kernel_ms_mean": dual_mean * 1e3,
                "kernel_ms_min": dual_min * 1e3,
                "bytes_per_launch": dual_bytes,
                "GBps": dual_bytes / dual_mean / 1e9,
                "pct_of_hbm_peak": 100.0 * dual_bytes / dual_mean / 1e9 / HBM_PEAK_GBS,
                "pct_of_plain_fill": 100.0 * dual_bytes / dual_mean / 1e9 / fill_gbs,
            },
        },
        "roofline": {
            "kernel": "k_row_desc + k_token_fill<float,float,int64> (large_bcast)",
            "bound": "hbm",
            "achieved": bcast_gbs,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": bcast_gbs / HBM_PEAK_GBS,
            "traffic": TRAFFIC_BROADCAST_BYTES,
            "bytes_per_launch": bcast_bytes,
        },
        "roofline_allocate": {
            "kernel": "k_class_hist + k_class_write (large_alloc)",
            "bound": "hbm",
            "achieved": alloc_bytes / (ev1 / steps) / 1e9,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": alloc_bytes / (ev1 / steps) / 1e9 / HBM_PEAK_GBS,
            "traffic": TRAFFIC_ALLOCATE_BYTES,
            "bytes_per_launch": alloc_bytes,
            "call_ms_mean": alloc_mean * 1e3,
            "call_ms_min": alloc_min * 1e3,
            "achievable": alloc_bytes / plain_mean / 1e9,
            "achievable_kind": "plain stream of the same shape in the same run: one kernel, 4 B read and 16 B "
                               "written per prompt (torch int32 -> complex128 copy)",
            "achievable_ms": plain_mean * 1e3,
            "frac_of_achievable": plain_mean / alloc_mean,
            "sweep": sweep,
        },
    }
    result["other_paths"] = extras
    if not args.no_cpu_baseline:
        from oracle import hora_oracle
        hora_oracle.build()
        result["cpu_baseline"] = cpu_baseline(wl, hora_oracle, w1, a1, (w2, a2))
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
