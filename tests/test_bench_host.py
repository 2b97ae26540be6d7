"""Host logic of bench.py (no GPU): the pending-token schedule behind its byte counts against the integer model of the
cache, the algorithmic byte count of a launch against hand-computed cases, and the refusal of more than one GPU."""
import os
import subprocess
import sys

import numpy as np
import pytest

import oracle
from workload import CONFIGS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


@pytest.mark.parametrize("mode,k", [("both", 4), ("hj_only", 4), ("defer", 4), ("defer", 7)])
def test_pending_schedule_matches_the_integer_model(mode, k):
    """bench.pend_after predicts, per round, how many accepted tokens each sequence still has to replay; the kernels'
    byte counts hang on it.  The integer model of the cache (commit rules of Algorithm 2 with lazy folding) is the
    authority: run it over the same acceptance history."""
    rng = np.random.default_rng(5)
    batch, rounds = 7, 40
    accepted = [rng.integers(0, k + 1, size=batch) for _ in range(rounds)]
    sched = bench.pend_after(accepted, [k] * rounds, mode=mode, kmax=k)
    bk = oracle.BookkeepingModel(batch, ring_len=16, conv_width=4, mode=mode, kmax=k)
    for r in range(rounds):
        assert sched[r].tolist() == list(bk.pend), "before round %d" % r
        bk.verify(k)
        bk.commit(accepted[r])


def test_algorithmic_bytes_of_a_launch_by_hand():
    """cfg1 (one sequence, 32 heads x 128 x 64, k = 4, bf16 tensors, fp32 state): S = 1 MiB.  Nothing pending: the state is
    read once and written once; two tokens pending: a second snapshot and their stashed inputs on top."""
    wl = CONFIGS["cfg1"]
    S = 32 * 128 * 64 * 4
    Cx, H, N, k, e = 4096, 32, 64, 4, 2
    tokens_in = k * (Cx + H + 2 * N) * e
    y_out = k * Cx * e
    stash_out = k * (Cx + H + N) * e
    assert bench.verify_bytes(wl, [0], k, fused=False) == 2 * S + tokens_in + y_out + stash_out
    pending_in = 2 * (Cx + H + N) * e
    assert bench.verify_bytes(wl, [2], k, fused=False) == 3 * S + tokens_in + y_out + stash_out + pending_in
    # conv roll fused in: the ring append, three history rows, four taps and the bias per channel come on top
    fused_extra = (k * Cx + 3 * Cx + 5 * Cx) * e
    assert bench.verify_bytes(wl, [2], k, fused=True) == bench.verify_bytes(wl, [2], k, fused=False) + fused_extra
    # the single-snapshot variant never writes h_k
    assert bench.verify_bytes(wl.scaled(snapshot_mode="hj_only"), [2], k, fused=False) == bench.verify_bytes(wl, [2], k, fused=False) - S
    # deferred advance: no h_k either, and h_j only beyond 16 - 2*4 = 8 pending tokens
    wd = wl.scaled(snapshot_mode="defer")
    assert bench.verify_bytes(wd, [8], k, fused=False) == S + tokens_in + y_out + stash_out + 4 * pending_in
    assert bench.verify_bytes(wd, [9], k, fused=False) == 2 * S + tokens_in + y_out + stash_out + 9 * pending_in // 2
    # a whole split round = the verify launch plus the conv launch (raw in, ring append, xc out, history, weights)
    conv_launch = (k * Cx * 3 + 3 * Cx + 5 * Cx) * e
    assert bench.round_bytes(wl, [0], k, fused=False) == bench.verify_bytes(wl, [0], k, fused=False) + conv_launch


@pytest.mark.parametrize("steps,warmup", [(20, 5), (21 * 64, 21), (1, 0), (100, 3)])
def test_timed_steps_carry_the_workloads_launch_mix(steps, warmup):
    """Whatever the step counts (the first pair is what the harness passes), the timed steps come after three
    priming rounds through every cache and move the workload's steady-state bytes: 94-95 MB per step on cfg3, not the
    73.5 MB of a round on fresh caches."""
    from workload import generate
    wl = CONFIGS["cfg3"]
    acc = [r.accepted for r in generate(wl).rounds]
    plan = bench.step_plan(wl, acc, wl.k, 21, warmup, steps, fused=True)
    assert plan["prime"] == 63 and plan["first_timed"] == 63 + warmup
    assert 92e6 < plan["workload_bytes"] < 96e6
    assert abs(plan["timed_bytes"] / plan["workload_bytes"] - 1.0) <= plan["slack"]
    fresh = bench.round_bytes(wl, np.zeros(wl.batch, dtype=np.int64), wl.k, True)
    assert fresh < 0.8 * plan["workload_bytes"]


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and "--gpus 1" in r.stderr
    assert r.stdout.strip() == ""
