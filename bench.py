#!/usr/bin/env python3
"""Benchmark of the multi-step SSM verification path on one MI355X.

A step is one verify round of one layer over one batch: conv1d_state_update ->
ssm_verify_multistep -> ssm_commit_rollback, inputs already resident in HBM.  Steps rotate
round-robin over enough independent caches that a cache's state has left the last-level cache
before it is touched again (the "cold" protocol: a real decoder streams the model's weights
between two visits to a layer's state).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3] ...
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0          # MI355X published HBM3E bandwidth


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (0: one pass over all caches and rounds)")
    ap.add_argument("--warmup", type=int, default=-1, help="untimed steps (-1: one per cache, at least 3)")
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--footprint-gib", type=float, default=2.0, help="total size of the rotating caches (cold protocol)")
    ap.add_argument("--instances", type=int, default=0, help="number of rotating caches (0: from --footprint-gib)")
    ap.add_argument("--no-graph", action="store_true", help="launch every step from Python instead of one HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-variants", action="store_true",
                    help="the default run also measures the two variants that store fewer snapshots (--single-snapshot, "
                         "--deferred-advance), each in a child process, and reports them beside the headline; this skips them")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle baseline")
    ap.add_argument("--rows", type=int, default=0, help="verify kernel: state rows per lane (0 = auto)")
    ap.add_argument("--waves", type=int, default=0, help="verify kernel: waves per workgroup (0 = auto)")
    ap.add_argument("--kernel-only", action="store_true", help="only the verify-kernel loop (for rocprofv3 runs)")
    ap.add_argument("--engine", choices=["auto", "vector"], default="auto",
                    help="auto: the library picks (the matrix-core kernel on a tiled state where it applies); "
                         "vector: the vector-ALU kernel on a row-major state")
    ap.add_argument("--single-snapshot", action="store_true",
                    help="the single-snapshot variant: h_k is never stored, every accepted token is replayed next round")
    ap.add_argument("--deferred-advance", action="store_true",
                    help="the deferred-advance variant: h_k is never stored and h_j only when the 16-token window is about to "
                         "fill up; most rounds only read the state")
    ap.add_argument("--naive", action="store_true",
                    help="the unfused baseline the paper starts from: one state snapshot copy, then k single-token rounds "
                         "(conv, verify with k=1, commit of 1) per layer-round; rollback work is not even included")
    ap.add_argument("--split", action="store_true",
                    help="three launches per step (conv1d_state_update, ssm_verify_multistep, ssm_commit_rollback) instead of "
                         "the fused conv+verify launch and one commit launch per round over all caches")
    ap.add_argument("--block", action="store_true",
                    help="the launch as a whole Mamba block's recurrence: dt = softplus(raw + bias) ahead of it, SiLU gate behind it")
    ap.add_argument("--draft", action="store_true",
                    help="the draft side: a round is fed by k single-token calls, one commit per round (implies the general "
                         "entry point).  On the matrix-core engine every call recomputes from the live slot and only the "
                         "last one stores the snapshots (replay_round); else, or with --draft-carry, the calls carry the "
                         "state through the h_k slot")
    ap.add_argument("--draft-carry", action="store_true", help="with --draft: carry the state through the h_k slot on every call")
    ap.add_argument("--ceiling", action="store_true",
                    help="measure what the memory system gives plain streams (read, write, copy; three footprints, three piece "
                         "sizes, persistent grids) and the floor of a launch, and print the table as JSON")
    ap.add_argument("--prefill", type=int, default=0, metavar="L",
                    help="measure the chunked prefill instead: a step = one call over L prompt tokens of every sequence")
    ap.add_argument("--prefill-io", choices=["f32", "bf16"], default=None,
                    help="with --prefill: storage type of the tensors (default: the workload's); f32 runs the fp32-MFMA kernel")
    return ap.parse_args()


WINDOW = 16     # tokens a verify launch can take (deferred advance)


def pend_hi_of(wl):
    """A verify stores h_j iff it meets more pending tokens than this."""
    return WINDOW - 2 * wl.kmax_eff if wl.snapshot_mode == "defer" else 0


def pend_after(accepted_rounds, k_rounds, hj_only=False, mode=None, kmax=0):
    """Host-side accounting of the pending-token count per sequence before each round (for byte counts only)."""
    import numpy as np
    mode = mode or ("hj_only" if hj_only else "both")
    pend = np.zeros_like(accepted_rounds[0])
    out = []
    for acc, k in zip(accepted_rounds, k_rounds):
        out.append(pend.copy())
        if mode == "defer":
            pend = np.where(pend > WINDOW - 2 * kmax, acc, pend + acc)
        else:
            pend = acc.copy() if mode == "hj_only" else np.where(acc == k, 0, acc)
    return out


def verify_bytes(wl, pend, k, fused, gate=False, calls=1, replay=False):
    """Algorithmic HBM bytes of one verify launch: state read once, h_k written, h_j written where
    tokens were pending, token inputs read, y and the stash written, pending tokens re-read; with the
    conv roll fused in: the raw inputs instead of xc, the ring append, 3 history rows, weights and bias."""
    e = 2 if wl.io == "bf16" else 4
    S = wl.state_elems * 4
    Cx, H, GN = wl.conv_channels, wl.nheads, wl.ngroups * wl.dstate
    total = 0
    hi = pend_hi_of(wl)
    for pd in pend:
        total += S * ((2 if wl.snapshot_mode == "both" else 1) + (1 if pd > hi else 0))
        total += k * (Cx + H + 2 * GN) * e          # xc (or x_raw), dt, B, C in
        total += k * Cx * e                         # y out
        total += k * (Cx + H + GN) * e              # stash out
        total += int(pd) * (Cx + H + GN) * e        # pending tokens in
        if fused:
            total += (k * Cx + calls * (3 * Cx + 5 * Cx)) * e   # ring append; per call: ring history, conv weights + bias
        if gate:
            total += k * Cx * e                     # z in
        if replay:                                  # every later call: state in; the pending and the round's earlier tokens again
            total += (calls - 1) * S + ((calls - 1) * int(pd) + (calls - 1) * calls // 2) * (Cx + H + GN) * e
        else:
            total += (calls - 1) * 2 * S            # every later call of a round: state in, state out
    return int(total)


def round_bytes(wl, pend, k, fused, gate=False, calls=1, replay=False):
    """Whole round.  Split path: the verify launch plus the conv launch (x_raw in, ring append, xc out, 3
    history rows and weights in).  Fused path: the one launch."""
    e = 2 if wl.io == "bf16" else 4
    if fused:
        return verify_bytes(wl, pend, k, True, gate, calls, replay)
    conv = len(pend) * (k * wl.conv_channels * 3 + 3 * wl.conv_channels + 5 * wl.conv_channels) * e
    return verify_bytes(wl, pend, k, False) + conv


def step_plan(wl, accepted_rounds, k, n_inst, warmup, steps, fused, gate=False, calls=1, replay=False):
    """Which steps are primed, warmed up and timed, and what they move.  Step s works on cache s % n_inst in round
    s // n_inst (the workload's rounds, cyclically).  Whatever `warmup` is, three untimed rounds through every cache come
    first, so that the pending counts - and with them the replay work and the h_j stores - have the workload's mix when
    the timed region starts: round 0 on fresh caches has nothing pending and is 22 % lighter than a steady-state round.
    Returns the step ranges, the mean algorithmic bytes of a timed step, and the workload's own mean over its rounds in
    the steady state (every round but the first)."""
    n_rounds = len(accepted_rounds)
    prime = 3 * n_inst
    first_timed = prime + warmup
    rounds_run = max((first_timed + steps + n_inst - 1) // n_inst + 1, n_rounds)
    sched = pend_after([accepted_rounds[i % n_rounds] for i in range(rounds_run)], [k] * rounds_run, mode=wl.snapshot_mode, kmax=wl.kmax_eff)
    step_bytes = lambda s: round_bytes(wl, sched[s // n_inst], k, fused, gate=gate, calls=calls, replay=replay)
    workload = sum(step_bytes(r * n_inst) for r in range(1, max(2, n_rounds))) / max(1, n_rounds - 1)
    timed = sum(step_bytes(s) for s in range(first_timed, first_timed + steps)) / steps
    return {"prime": prime, "first_timed": first_timed, "timed_bytes": timed, "workload_bytes": workload,
            # the timed steps see the realised pending counts of batch x (rounds they cover) sequence-rounds, not the mean
            # over the workload: 2 % for a long run, 8 % for cfg3's 32 sequences over one round, more for a single sequence
            "slack": min(0.5, max(0.02, 0.45 / math.sqrt(max(1.0, len(accepted_rounds[0]) * steps / n_inst))))}


PEAK_MFMA_F32_TFLOPS = 157.3     # MI355X published dense fp32 matrix rate
PEAK_MFMA_BF16_TFLOPS = 2500.0   # and the dense bf16 matrix rate
PEAK_HBM_GBPS = 8000.0


def bench_prefill(args):
    """Chunked prefill (ssm_prefill_chunked) of one layer: batch sequences of L prompt tokens per step.  Inputs are
    drawn on the device (seeded): x ~ N(0,1), B, C ~ N(0,1)/sqrt(N), dt = softplus(N(0,1) - 4); parameters are the
    workload's.  Roofline: with fp32 tensors the launch is a chain of dense contractions on the fp32 matrix cores and is
    priced against their peak; with bf16 tensors the contractions run on the bf16 matrix cores (16 times that rate), where
    the launch's matrix work (0.08 ms at peak for cfg3, 2048 tokens) is below its HBM traffic (0.15 ms at peak), so HBM is
    the bound it is priced against; the executed matrix rate is reported beside it."""
    import numpy as np
    import torch

    import paper_2408_15237_amd as ssmv
    from workload import CONFIGS, generate

    torch.cuda.set_device(0)
    ssmv.load_library()
    wl = CONFIGS[args.workload].scaled(layers=1, rounds=1)
    if args.prefill_io:
        wl = wl.scaled(io=args.prefill_io)
    L = args.prefill
    lp = generate(wl).layers[0]
    io_t = torch.bfloat16 if wl.io == "bf16" else torch.float32
    dev = "cuda"
    dims = ssmv.make_dims(wl.batch, wl.nheads, wl.headdim, wl.dstate, ngroups=wl.ngroups, kmax=wl.kmax_eff, ring_len=wl.ring_len,
                          io=wl.io, a_mode=wl.a_mode, conv_act=wl.conv_act, engine=args.engine)
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev).to(io_t).contiguous()
    A, D = torch.from_numpy(lp.A).to(dev), torch.from_numpy(lp.D).to(dev)
    conv_w, conv_b = up(lp.conv_w), (None if lp.conv_b is None else up(lp.conv_b))
    h0 = torch.from_numpy(lp.h0).to(dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(wl.seed)
    B_, H, P, N, G, Cx = wl.batch, wl.nheads, wl.headdim, wl.dstate, wl.ngroups, wl.conv_channels
    x = torch.randn((B_, L, Cx), generator=gen, device=dev).to(io_t)
    dt = torch.nn.functional.softplus(torch.randn((B_, L, H), generator=gen, device=dev) - 4.0).to(io_t)
    Bm = (torch.randn((B_, L, G, N), generator=gen, device=dev) / N ** 0.5).to(io_t)
    Cm = (torch.randn((B_, L, G, N), generator=gen, device=dev) / N ** 0.5).to(io_t)
    y = torch.empty_like(x)
    caches = [ssmv.LayerCache.allocate(dims) for _ in range(2)]
    for c in caches:
        ssmv.ssmv_cache_reset(dims, c.c, h0, None)

    def step(i):
        ssmv.ssm_prefill_chunked(dims, caches[i % 2].c, x, conv_w, conv_b, dt, Bm, Cm, A, D, L, y)

    # The clocks take some fifty launches to settle under this kernel's load (430 -> 530 -> 410 us per launch): the
    # defaults warm up past that and time the steady state.
    K = args.steps if args.steps > 0 else 200
    Wm = args.warmup if args.warmup >= 0 else 50
    for i in range(Wm):
        step(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for i in range(K):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / K
    for c in caches:
        ssmv.ssmv_check(c.c)
    Q = 32
    flops = 2.0 * (Q * N + Q * P + 2 * N * P) * B_ * L * H            # the four contractions of a chunk, per token and head
    e = 2 if wl.io == "bf16" else 4
    nbytes = B_ * L * (2 * Cx + H + 2 * G * N) * e + 2 * wl.state_elems * 4 * B_
    tflops = flops / (ms * 1e-3) / 1e12
    gbps = nbytes / (ms * 1e-3) / 1e9
    if wl.io == "bf16":
        # executed matrix work per chunk and wave, in products of 32x32x16: N/16 (G^T, every wave its own) + N/16 (h C^T, head
        # only) + 2 (M X, head only) + 2 N/16 (update, head and tail)
        mfma_flops = (2 + 4 * (N // 16)) * 32768.0 * (P // 32) * math.ceil(L / Q) * B_ * H
        traffic = None                                  # the counters were read on this shape only
        tpath = os.path.join(ROOT, "profiles", "prefill_bf16_kernel_%s_L%d_pmc.txt" % (wl.name, L))
        if not args.prefill_io and os.path.exists(tpath):
            for line in open(tpath):
                if line.startswith("traffic_bytes_per_launch:"):
                    traffic = float(line.split(":")[1])
        roof = {"bound": "hbm", "achieved": round(gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": round(gbps / PEAK_HBM_GBPS, 4),
                "traffic": traffic, "kernel": "prefill_bf16_kernel (bf16 MFMA, split operand in the state update)", "avg_launch_us": round(ms * 1e3, 1),
                "algorithmic_bytes_per_launch": int(nbytes), "algorithmic_flops_per_launch": int(flops),
                "mfma_executed_tflops": round(mfma_flops / (ms * 1e-3) / 1e12, 1),
                "mfma_frac_of_bf16_peak": round(mfma_flops / (ms * 1e-3) / 1e12 / PEAK_MFMA_BF16_TFLOPS, 4)}
        dtype = "bf16 products (fp32 operand of the state update split into head and tail), f32 accumulation"
    else:
        roof = {"bound": "mfma", "achieved": round(tflops, 2), "peak": PEAK_MFMA_F32_TFLOPS, "unit": "TFLOP/s",
                "frac": round(tflops / PEAK_MFMA_F32_TFLOPS, 4), "traffic": None, "kernel": "prefill_kernel (fp32 MFMA)",
                "avg_launch_us": round(ms * 1e3, 1), "algorithmic_flops_per_launch": int(flops), "algorithmic_bytes_per_launch": int(nbytes)}
        dtype = "f32"
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        nb, Lc = min(B_, 2), min(L, 256)
        ora = oracle.EagerOracle(wl.a_mode, lp.A, lp.D, lp.conv_w, lp.conv_b, lp.h0[:nb], wl.io, wl.conv_act, wl.ngroups)
        f = lambda t: t[:nb, :Lc].float().cpu().numpy()
        t0 = time.perf_counter()
        ora.verify(f(x), f(dt), f(Bm), f(Cm))
        el = time.perf_counter() - t0
        cpu = {"value": round(nb * Lc / el, 1), "unit": "tokens/s", "cores": oracle.oracle_threads(), "kind": "oracle",
               "sample": "%d sequences x %d prompt tokens of the same layer (fp64, token by token, %.1f s)" % (nb, Lc, el)}
    print(json.dumps({
        "metric": "prompt tokens/sec per SSM layer (chunked prefill)", "value": round(B_ * L / (ms * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(ms, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": "%s layer shape (batch %d, %d heads x headdim %d x d_state %d, %s I/O), prompt of %d tokens per sequence"
                               % (wl.name, B_, H, P, N, wl.io, L), "batch": B_, "prompt_len": L},
        "hbm_gbps_whole_step": round(gbps, 1), "algorithmic_tflops": round(tflops, 2),
        "roofline": roof,
        "cpu_baseline": cpu}))


def bench_ceiling():
    """The ceilings the roofline figures are read against: ssmv_stream_probe in every direction, launches back to back in a
    HIP graph (as the verify launches are timed), rotating over enough buffers that every launch finds its data in HBM."""
    import torch

    import paper_2408_15237_amd as ssmv
    torch.cuda.set_device(0)
    ssmv.load_library()
    rows = []
    for mib in (32, 96, 1024):
        S = mib << 20
        n_buf = max(2, (3 << 30) // (3 * S))
        bufs = [torch.zeros(3 * S // 4, dtype=torch.float32, device="cuda") for _ in range(n_buf)]
        for mode, traffic in (("read", 1), ("write", 1), ("r1w1", 2), ("r1w2", 3), ("empty", 0)):
            for piece, grid in ((4, 0), (8, 0), (32, 0), (32, 1024), (32, 2048)):
                if mode == "empty" and (piece != 32 or grid == 2048):
                    continue
                n = max(8, min(256, (64 << 30) // (S * max(1, traffic))))

                def launch(i):
                    p0 = bufs[i % n_buf].data_ptr()
                    ssmv.ssmv_stream_probe(mode, p0, p0 + S, p0 + 2 * S, S, piece, grid)
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                g = torch.cuda.CUDAGraph()
                with torch.cuda.stream(side):
                    g.capture_begin()
                    for i in range(n):
                        launch(i)
                    g.capture_end()
                torch.cuda.current_stream().wait_stream(side)
                g.replay()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(); g.replay(); e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / n
                rows.append({"mode": mode, "source_mib": mib, "piece_kib": piece, "grid": grid or "one workgroup per piece",
                             "us_per_launch": round(us, 2), "gbps": round(traffic * S / us / 1e3, 1)})
        del bufs
    print(json.dumps({"ceiling": rows, "peak_gbps": PEAK_HBM_GBPS}))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU (the path shards over sequences/heads with no exchange step); "
              "--gpus %d is not supported, run with --gpus 1" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2408_15237_amd as ssmv
    from workload import CONFIGS, block_extras, generate

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    if args.ceiling:
        bench_ceiling()
        return
    if args.prefill > 0:
        bench_prefill(args)
        return
    torch.cuda.set_device(0)
    ssmv.load_library()
    ssmv.ssmv_set_tuning(args.rows, args.waves)

    wl = CONFIGS[args.workload]
    if wl.layers != 1:
        wl = wl.scaled(layers=1)           # the metric is per SSM layer; the stack is covered by the parity tests
    if args.single_snapshot:
        wl = wl.scaled(snapshot_mode="hj_only")
    if args.deferred_advance:
        if args.single_snapshot or 2 * wl.kmax_eff > WINDOW:
            print("bench.py: --deferred-advance needs 2*kmax <= %d and excludes --single-snapshot" % WINDOW, file=sys.stderr)
            sys.exit(2)
        wl = wl.scaled(snapshot_mode="defer")
    data = generate(wl)
    lp = data.layers[0]
    io_t = torch.bfloat16 if wl.io == "bf16" else torch.float32
    dev = "cuda"

    def up(a):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev).to(io_t).contiguous()

    dims = ssmv.make_dims(wl.batch, wl.nheads, wl.headdim, wl.dstate, ngroups=wl.ngroups, kmax=wl.kmax_eff,
                          ring_len=wl.ring_len, io=wl.io, a_mode=wl.a_mode, conv_act=wl.conv_act,
                          snapshot_mode=wl.snapshot_mode, engine=args.engine)
    sizes = ssmv.ssmv_cache_sizes(dims)
    matrix_engine = ssmv.ssmv_engine_of(dims) == 1
    cache_bytes = sum(sizes)
    # (at most 1024 caches: a tiny workload such as cfg0 would otherwise ask for 10^5 of them and a graph of 10^6 launches,
    # which the runtime does not survive; its footprint is then below --footprint-gib and `config.instances` says so)
    n_inst = args.instances or min(1024, max(1, math.ceil(args.footprint_gib * 2 ** 30 / cache_bytes)))
    caches = [ssmv.LayerCache.allocate(dims) for _ in range(n_inst)]
    A = torch.from_numpy(lp.A).to(dev)
    D = torch.from_numpy(lp.D).to(dev)
    conv_w, conv_b = up(lp.conv_w), (None if lp.conv_b is None else up(lp.conv_b))
    h0 = torch.from_numpy(lp.h0).to(dev)
    rounds = [dict(x=up(r.x_raw), dt=up(r.dt[0]), B=up(r.B[0]), C=up(r.C[0]),
                   acc=torch.from_numpy(r.accepted).to(dev)) for r in data.rounds]
    n_rounds = len(rounds)
    k = wl.k
    xc_buf = torch.empty_like(rounds[0]["x"])
    y_buf = torch.empty_like(rounds[0]["x"])
    for c in caches:
        ssmv.ssmv_cache_reset(dims, c.c, h0, None)
    torch.cuda.synchronize()

    fused = not (args.split or args.naive)
    general = args.block or args.draft
    if general and not fused:
        print("bench.py: --block/--draft use the fused launch; not with --split/--naive", file=sys.stderr)
        sys.exit(2)
    replay = args.draft and matrix_engine and not args.draft_carry and args.rows == 0 and args.waves == 0
    if args.draft and wl.snapshot_mode != "both" and not replay:
        print("bench.py: a round whose calls carry the state needs the h_k slot; not with --single-snapshot or --deferred-advance", file=sys.stderr)
        sys.exit(2)
    blk = {}
    if args.block:
        ex = block_extras(data)
        blk = dict(dt_bias=torch.from_numpy(ex.dt_bias[0]).to(dev), dt_softplus=True)
        for r, raw, zz in zip(rounds, ex.dt_raw, ex.z):
            r["dt"], r["z"] = up(raw[0]), up(zz)
    if args.draft:
        for r in rounds:
            for name in ("x", "dt", "B", "C") + (("z",) if args.block else ()):
                r[name + "1"] = [r[name][:, t:t + 1].contiguous() for t in range(k)]
        y1_buf = torch.empty_like(rounds[0]["x1"][0])
    if args.naive:
        ones = torch.ones(wl.batch, dtype=torch.int32, device=dev)
        for r in rounds:
            for name in ("x", "dt", "B", "C"):
                r[name + "1"] = [r[name][:, t:t + 1].contiguous() for t in range(k)]
        x1_buf, y1_buf = torch.empty_like(rounds[0]["x1"][0]), torch.empty_like(rounds[0]["x1"][0])
        slot_bytes = (sizes[0] // 3) // 16 * 16
    all_caches = (ssmv.ssmv_cache * n_inst)(*[c.c for c in caches])

    # The rotating caches play the SSM layers of one model: a round verifies layer after layer, then the
    # accepted lengths are known and every layer commits.  Step s = (layer s % n_inst, round s // n_inst).
    def step(s):
        i = s % n_inst
        c = caches[i].c
        r = rounds[(s // n_inst) % n_rounds]
        if args.naive:
            base = caches[i].buffers["state"].data_ptr()
            ssmv.ssmv_copy_probe(base, base + slot_bytes, None, slot_bytes)          # snapshot of the state before the drafts
            for t in range(k):
                ssmv.conv1d_state_update(dims, c, r["x1"][t], conv_w, conv_b, 1, x1_buf)
                ssmv.ssm_verify_multistep(dims, c, x1_buf, r["dt1"][t], r["B1"][t], r["C1"][t], A, D, 1, y1_buf)
                ssmv.ssm_commit_rollback(dims, c, ones)
        elif args.draft:
            for t in range(k):
                ssmv.ssm_block_multistep(dims, c, x_raw=r["x1"][t], conv_wgt=conv_w, conv_bias=conv_b, dt=r["dt1"][t], Bm=r["B1"][t],
                                         Cm=r["C1"][t], A=A, D=D, k=1, tok0=t, y_out=y1_buf, replay_round=replay, last_call=replay and t == k - 1,
                                         z=r["z1"][t] if args.block else None, **blk)
            if i == n_inst - 1:
                ssmv.ssm_commit_rollback_multi(dims, all_caches, r["acc"])
        elif general:
            ssmv.ssm_block_multistep(dims, c, x_raw=r["x"], conv_wgt=conv_w, conv_bias=conv_b, dt=r["dt"], Bm=r["B"], Cm=r["C"],
                                     A=A, D=D, k=k, y_out=y_buf, z=r["z"], **blk)
            if i == n_inst - 1:
                ssmv.ssm_commit_rollback_multi(dims, all_caches, r["acc"])
        elif fused:
            ssmv.ssm_conv_verify_multistep(dims, c, r["x"], conv_w, conv_b, r["dt"], r["B"], r["C"], A, D, k, y_buf)
            if i == n_inst - 1:
                ssmv.ssm_commit_rollback_multi(dims, all_caches, r["acc"])
        else:
            ssmv.conv1d_state_update(dims, c, r["x"], conv_w, conv_b, k, xc_buf)
            ssmv.ssm_verify_multistep(dims, c, xc_buf, r["dt"], r["B"], r["C"], A, D, k, y_buf)
            ssmv.ssm_commit_rollback(dims, c, r["acc"])

    def finish(s_end):
        """Commit the layers of a round that the timed region cut short (fused path only; after the timed region)."""
        done = s_end % n_inst
        if fused and done:
            part = (ssmv.ssmv_cache * done)(*[c.c for c in caches[:done]])
            ssmv.ssm_commit_rollback_multi(dims, part, rounds[(s_end // n_inst) % n_rounds]["acc"])

    K = args.steps if args.steps > 0 else n_inst * n_rounds
    if K > 65536:
        print("bench.py: %d timed steps would be one graph of that many launches; at most 65536" % K, file=sys.stderr)
        sys.exit(2)
    W = args.warmup if args.warmup >= 0 else max(3, n_inst)
    plan = step_plan(wl, [r.accepted for r in data.rounds], k, n_inst, W, K, fused, gate=args.block, calls=k if args.draft else 1, replay=replay)
    PRIME, workload_bytes = plan["prime"], plan["workload_bytes"]

    # A launch that keeps the GPU busy for ~0.1 ms (a plain 256 MiB copy, which also sweeps the caches): queued ahead of the
    # first event of a timed graph, so that the event and the whole graph are already in the queue when the GPU reaches them
    # and the timed region holds the K steps back to back, not the host's one-off latency of submitting the graph (some
    # 20 us, which K = 20 steps of 17 us would otherwise carry as 6 %).
    filler_buf = torch.empty(2 * 256 * 2 ** 20, dtype=torch.uint8, device=dev)

    def filler(n=1):                                  # (the stream probe, not the copy probe: that one calibrates the byte counters)
        for _ in range(n):
            ssmv.ssmv_stream_probe("r1w1", filler_buf.data_ptr(), filler_buf.data_ptr() + 256 * 2 ** 20, None, 256 * 2 ** 20)

    result = {}
    for s in range(PRIME):
        step(s)
    torch.cuda.synchronize()
    if not args.kernel_only:
        W0, W = PRIME, PRIME + W                       # first warm-up step, first timed step
        for s in range(W0, W):
            step(s)
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if args.no_graph:
            torch.cuda.synchronize()
            ev0.record()
            for s in range(W, W + K):
                step(s)
            ev1.record()
            torch.cuda.synchronize()
        elif K <= 128:
            # A handful of steps: a graph's own start and end (some 20 us per replay, measured: K = 20 reads 1 us per step
            # more than K = 1344) would be a visible share of the timed region.  The steps are launched one by one instead,
            # INTO A BUSY QUEUE: enough filler launches go first that the host has submitted every step before the GPU
            # reaches the first event, so the GPU runs the K steps back to back, as it runs them inside a long graph.
            launches = K * ((k if (args.draft or args.naive) else 1) * (3 if args.naive else 1) + (0 if fused else 2)) + K // n_inst + 2
            torch.cuda.synchronize()
            filler(3 + launches * 25 // 90)             # 25 us of host time per launch against 90 us per filler launch
            ev0.record()
            for s in range(W, W + K):
                step(s)
            ev1.record()
            torch.cuda.synchronize()
        else:
            # the K timed steps as one HIP graph (kernel nodes only): no launch gaps from Python
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                graph.capture_begin()
                for s in range(W, W + K):
                    step(s)
                graph.capture_end()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            filler()
            ev0.record()
            graph.replay()
            ev1.record()
            torch.cuda.synchronize()
        total_ms = ev0.elapsed_time(ev1)
        finish(W + K)                                    # tidy up: the timed steps hold their share of commits, one per n_inst steps
        for c in caches:
            ssmv.ssmv_check(c.c)
        # algorithmic bytes of exactly the timed steps; they must be the workload's mix
        timed_bytes = plan["timed_bytes"]
        tot_bytes = timed_bytes * K
        if abs(timed_bytes / workload_bytes - 1.0) > plan["slack"]:
            print("bench.py: the timed steps move %.1f MB each, the workload %.1f MB: not the workload's launch mix"
                  % (timed_bytes / 1e6, workload_bytes / 1e6), file=sys.stderr)
            sys.exit(3)
        W -= PRIME                                       # reported as given
        tokens = wl.batch * k * K
        result.update(
            value=tokens / (total_ms * 1e-3),
            ms_per_step=total_ms / K,
            step_hbm_gbps=tot_bytes / (total_ms * 1e-3) / 1e9,
            timed_bytes=timed_bytes,
        )

    # ---- the dominant kernel alone: n_meas back-to-back launches (one HIP graph, kernel nodes only) rotating
    # over the caches, bracketed by HIP events on the launch stream.  The average therefore includes the gap
    # between two kernels of one stream; rocprofv3's per-dispatch duration excludes it and reads lower.
    torch.cuda.synchronize()
    n_meas = max(64, min(512, 4 * n_inst))
    pend_now = [c.ints()["pend"] for c in caches]
    r0 = rounds[0]

    def dominant(c):
        if args.draft:      # a later call of a round: one token; state read and written in place, or (replayed round) read only
            ssmv.ssm_block_multistep(dims, c, x_raw=r0["x1"][1], conv_wgt=conv_w, conv_bias=conv_b, dt=r0["dt1"][1], Bm=r0["B1"][1],
                                     Cm=r0["C1"][1], A=A, D=D, k=1, tok0=1, y_out=y1_buf, z=r0["z1"][1] if args.block else None,
                                     replay_round=replay, **blk)
        elif general:
            ssmv.ssm_block_multistep(dims, c, x_raw=r0["x"], conv_wgt=conv_w, conv_bias=conv_b, dt=r0["dt"], Bm=r0["B"], Cm=r0["C"],
                                     A=A, D=D, k=k, y_out=y_buf, z=r0["z"], **blk)
        elif fused:
            ssmv.ssm_conv_verify_multistep(dims, c, r0["x"], conv_w, conv_b, r0["dt"], r0["B"], r0["C"], A, D, k, y_buf)
        else:
            ssmv.ssm_verify_multistep(dims, c, r0["x"], r0["dt"], r0["B"], r0["C"], A, D, k, y_buf)

    for i in range(n_inst):
        dominant(caches[i].c)
    torch.cuda.synchronize()
    if args.draft:
        e_io = 2 if wl.io == "bf16" else 4
        Cx_, H_, GN_ = wl.conv_channels, wl.nheads, wl.ngroups * wl.dstate
        per_seq = ((Cx_ + H_ + 2 * GN_) + Cx_ + (Cx_ + H_ + GN_) + Cx_ + 8 * Cx_ + (Cx_ if args.block else 0)) * e_io
        if replay:
            kbytes = sum(int(np.sum(wl.state_elems * 4 + per_seq + (pend_now[i % n_inst] + 1) * (Cx_ + H_ + GN_) * e_io)) for i in range(n_meas))
        else:
            kbytes = (2 * wl.state_elems * 4 + per_seq) * wl.batch * n_meas
    else:
        kbytes = sum(verify_bytes(wl, pend_now[i % n_inst], k, fused, gate=args.block) for i in range(n_meas))
    side2 = torch.cuda.Stream()
    side2.wait_stream(torch.cuda.current_stream())
    kgraph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side2):
        kgraph.capture_begin()
        for i in range(n_meas):
            dominant(caches[i % n_inst].c)
        kgraph.capture_end()
    torch.cuda.current_stream().wait_stream(side2)
    torch.cuda.synchronize()
    durs = []
    for rep in range(5):
        ka, kb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        filler()
        ka.record()
        kgraph.replay()
        kb.record()
        torch.cuda.synchronize()
        durs.append(ka.elapsed_time(kb) / n_meas)
    durs.sort()
    avg_ms = sum(durs) / len(durs)
    achieved = (kbytes / n_meas) / (avg_ms * 1e-3) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "%s_%s_pmc.txt" % ("verify_mfma_kernel" if matrix_engine else "verify_kernel", wl.name))
    default_path = fused and not general and wl.snapshot_mode == "both" and args.rows == 0 and args.waves == 0
    if default_path and os.path.exists(tpath):     # the counters were read on the default launch only
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":")[1])
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                "frac": round(achieved / PEAK_HBM_GBPS, 4), "traffic": traffic,
                "kernel": ("verify_mfma_kernel" if matrix_engine and args.rows == 0 and args.waves == 0 else "verify_kernel") +
                          (" (conv roll fused, one token appended to the round)" if args.draft else " (conv roll fused)" if fused else ""),
                "avg_launch_us": round(avg_ms * 1e3, 3),
                "median_launch_us": round(durs[len(durs) // 2] * 1e3, 3),
                "algorithmic_bytes_per_launch": kbytes // n_meas, "launches_timed": n_meas * len(durs)}

    # ---- achievable ceiling: plain copy, read S / write 2S, same footprint --------------------------
    nbytes = (sizes[0] // 3) // 16 * 16
    ce0, ce1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = max(2 * n_inst, 16)
    for i in range(min(4, n_inst)):
        st = caches[i % n_inst].buffers["state"]
        base = st.data_ptr()
        ssmv.ssmv_copy_probe(base, base + nbytes, base + 2 * nbytes, nbytes)
    torch.cuda.synchronize()
    ce0.record()
    for i in range(reps):
        base = caches[i % n_inst].buffers["state"].data_ptr()
        ssmv.ssmv_copy_probe(base, base + nbytes, base + 2 * nbytes, nbytes)
    ce1.record()
    torch.cuda.synchronize()
    copy_gbps = 3 * nbytes * reps / (ce0.elapsed_time(ce1) * 1e-3) / 1e9

    if args.kernel_only:
        print(json.dumps({"kernel_only": True, "roofline": roofline, "copy_r1w2_gbps": round(copy_gbps, 1)}))
        return

    # ---- the oracle on the host cores, bounded sample ------------------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle                      # cpu_baseline leg only
        ora = oracle.EagerOracle(wl.a_mode, lp.A, lp.D, lp.conv_w, lp.conv_b, lp.h0, wl.io, wl.conv_act, wl.ngroups)
        t0 = time.perf_counter()
        done = 0
        while True:                         # the workload's rounds, again from the first when they run out
            r = data.rounds[done % n_rounds]
            ora.verify(r.x_raw, r.dt[0], r.B[0], r.C[0])
            ora.commit(r.accepted)
            done += 1
            el = time.perf_counter() - t0
            if el >= args.cpu_seconds or (done >= 2 and el / done * (done + 1) > 2.5 * args.cpu_seconds):
                break
        el = time.perf_counter() - t0
        cpu = {"value": round(wl.batch * k * done / el, 1), "unit": "tokens/s", "cores": oracle.oracle_threads(),
               "kind": "oracle", "sample": "%d rounds of %s (its %d rounds, cyclically), all %d sequences (fp64, eager, %.1f s)"
               % (done, wl.name, n_rounds, wl.batch, el)}

    out = {
        "metric": "verified draft tokens/sec per SSM layer",
        "value": round(result["value"], 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(result["ms_per_step"], 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": ("f32 state and accumulation; bf16 matrix products of head+tail split f32 operands" if matrix_engine else "f32"),
        "data": "synthetic",
        "config": {"workload": "%s: %s-A layer, batch %d, %d heads x headdim %d x d_state %d, k=%d, %s I/O + fp32 state, "
                               "%s acceptance, %d rounds, cold protocol over %d rotating caches (%.2f GiB)"
                               % (wl.name, wl.a_mode, wl.batch, wl.nheads, wl.headdim, wl.dstate, k, wl.io, wl.accept,
                                  n_rounds, n_inst, n_inst * cache_bytes / 2 ** 30),
                   "batch": wl.batch, "k": k, "rounds": n_rounds, "instances": n_inst,
                   "launch": "eager" if args.no_graph else ("hip-graph" if K > 128 else "single launches into a busy queue"),
                   "snapshots": {"both": "h_j and h_k (Algorithm 2)", "hj_only": "h_j only (single-snapshot variant)",
                                 "defer": "h_j only, and only when the 16-token window fills up (deferred advance)"}[wl.snapshot_mode],
                   "path": ("draft side: k single-token calls per layer-round, every call recomputing from the live slot, snapshots stored by the last; one commit launch per round" if replay else
                            "draft side: k single-token calls per layer-round carrying the state through the h_k slot (first one replays), one commit launch per round" if args.draft else
                            "fused conv+verify launch per layer, one commit launch per round over all caches") +
                           (", softplus(dt+bias) and SiLU gate fused" if args.block else "") if fused
                           else ("naive: snapshot copy + k single-token (conv, verify, commit) rounds per layer" if args.naive
                                 else "conv, verify and commit launches per layer")},
        "hbm_gbps_whole_step": round(result["step_hbm_gbps"], 1),
        "algorithmic_bytes_per_step_timed": int(result["timed_bytes"]),
        "algorithmic_bytes_per_step_workload": int(workload_bytes),
        "engine": "matrix cores, tiled state" if matrix_engine else "vector ALUs, row-major state",
        "copy_r1w2_gbps": round(copy_gbps, 1),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    # ---- the variants that store fewer snapshots, beside the headline (same workload, protocol and step counts) ----
    plain = not (args.single_snapshot or args.deferred_advance or args.naive or args.split or args.block or args.draft or
                 args.no_graph or args.rows or args.waves)
    if plain and not args.no_variants:
        import subprocess
        variants = {}
        flags = ["--single-snapshot"] + (["--deferred-advance"] if 2 * wl.kmax_eff <= WINDOW else [])
        for flag in flags:
            cmd = [sys.executable, os.path.abspath(__file__), flag, "--no-variants", "--no-cpu-baseline", "--workload", args.workload,
                   "--steps", str(args.steps), "--warmup", str(args.warmup), "--engine", args.engine,
                   "--footprint-gib", str(args.footprint_gib), "--instances", str(args.instances)]
            try:
                r = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
                line = [l for l in r.stdout.splitlines() if l.startswith("{")][-1]
                v = json.loads(line)
                variants[flag.lstrip("-").replace("-", "_")] = {
                    "value": v["value"], "unit": v["unit"], "ms_per_step": v["ms_per_step"], "snapshots": v["config"]["snapshots"],
                    "algorithmic_bytes_per_step_timed": v["algorithmic_bytes_per_step_timed"],
                    "roofline": {kk: v["roofline"][kk] for kk in ("achieved", "frac", "avg_launch_us", "algorithmic_bytes_per_launch")}}
            except Exception as exc:             # a variant that did not run is reported as such, the headline stands
                variants[flag.lstrip("-").replace("-", "_")] = {"error": "%s: %s" % (type(exc).__name__, exc)}
        out["variants"] = variants
        if args.workload == "cfg3":                  # the other 8B-shaped configuration (24-layer stack, k = 8): its layer shape, same protocol
            cmd = [sys.executable, os.path.abspath(__file__), "--workload", "cfg4", "--no-variants", "--no-cpu-baseline",
                   "--steps", str(args.steps), "--warmup", str(args.warmup), "--engine", args.engine,
                   "--footprint-gib", str(args.footprint_gib)]
            try:
                r = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
                v = json.loads([l for l in r.stdout.splitlines() if l.startswith("{")][-1])
                out["other_workloads"] = {"cfg4": {"value": v["value"], "unit": v["unit"], "ms_per_step": v["ms_per_step"],
                                                   "workload": v["config"]["workload"], "roofline": v["roofline"]}}
            except Exception as exc:
                out["other_workloads"] = {"cfg4": {"error": "%s: %s" % (type(exc).__name__, exc)}}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
