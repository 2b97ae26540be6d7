"""Timeline of the matrix-core verify kernel from inside: builds the library with -DSSMV_TRACE (libssmv_trace.so), runs a
workload's fused conv+verify launches back to back (one HIP graph, rotating caches, pending counts as the workload leaves
them) and prints, for the LAST launch of the graph, the distribution over its workgroups of eight wall-clock stamps
(microseconds since the launch's first workgroup started).  A profiling aid: the stamps and one extra wait change the
kernel slightly, so its timings are not the library's.

  python -m paper_2408_15237_amd.trace_stamps [--workload cfg3] [--launches 64] [--snapshot-mode both|hj_only|defer] [--prime 3]
"""
from __future__ import annotations

import argparse
import ctypes
import math
import os
import sys

STAMPS = ["start", "token loads issued", "state loads issued", "tokens arrived", "staged, barrier passed",
          "state arrived", "products done, stores issued", "stores acknowledged"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--launches", type=int, default=64)
    ap.add_argument("--footprint-gib", type=float, default=2.0)
    ap.add_argument("--snapshot-mode", default="both", choices=["both", "hj_only", "defer"])
    ap.add_argument("--prime", type=int, default=3, help="committed rounds ahead of the traced one (they set the pending counts)")
    args = ap.parse_args()
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    import numpy as np
    import torch

    from . import binding
    from .build import build
    binding.LIB_PATH = build(trace=True)
    import paper_2408_15237_amd as ssmv
    from workload import CONFIGS, generate

    lib = ssmv.load_library()
    wl = CONFIGS[args.workload].scaled(layers=1)
    data = generate(wl)
    lp = data.layers[0]
    dev, io_t = "cuda", torch.bfloat16 if wl.io == "bf16" else torch.float32
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev).to(io_t).contiguous()
    dims = ssmv.make_dims(wl.batch, wl.nheads, wl.headdim, wl.dstate, ngroups=wl.ngroups, kmax=wl.kmax_eff, ring_len=wl.ring_len,
                          io=wl.io, a_mode=wl.a_mode, conv_act=wl.conv_act, snapshot_mode=args.snapshot_mode)
    n_inst = max(1, math.ceil(args.footprint_gib * 2 ** 30 / sum(ssmv.ssmv_cache_sizes(dims))))
    caches = [ssmv.LayerCache.allocate(dims) for _ in range(n_inst)]
    A, D = torch.from_numpy(lp.A).to(dev), torch.from_numpy(lp.D).to(dev)
    cw, cb, h0 = up(lp.conv_w), up(lp.conv_b), torch.from_numpy(lp.h0).to(dev)
    rounds = [dict(x=up(r.x_raw), dt=up(r.dt[0]), B=up(r.B[0]), C=up(r.C[0]), acc=torch.from_numpy(r.accepted).to(dev)) for r in data.rounds[:args.prime + 1]]
    y = torch.empty_like(rounds[0]["x"])
    allc = (ssmv.ssmv_cache * n_inst)(*[c.c for c in caches])
    for c in caches:
        ssmv.ssmv_cache_reset(dims, c.c, h0, None)
    verify = lambda c, r: ssmv.ssm_conv_verify_multistep(dims, c.c, r["x"], cw, cb, r["dt"], r["B"], r["C"], A, D, wl.k, y)
    for r in rounds[:args.prime]:                            # so that the pending counts have their mix
        for c in caches:
            verify(c, r)
        ssmv.ssm_commit_rollback_multi(dims, allc, r["acc"])
    n_wg = wl.batch * wl.nheads * (wl.headdim // 64)         # an upper bound on the workgroups of a launch
    stamps = torch.zeros(n_wg * 8, dtype=torch.int64, device=dev)
    lib.ssmv_debug_set_trace.argtypes = [ctypes.c_void_p]
    assert lib.ssmv_debug_set_trace(stamps.data_ptr()) == 0
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        g.capture_begin()
        for i in range(args.launches):
            verify(caches[i % n_inst], rounds[args.prime])
        g.capture_end()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(); g.replay(); e1.record()
    torch.cuda.synchronize()
    st = stamps.cpu().numpy().reshape(-1, 8)
    st = st[st[:, 0] > 0]
    t0 = st[:, 0].min()
    pend = caches[0].ints()["pend"]
    print("snapshot mode %s, pending tokens per sequence %s" % (args.snapshot_mode, pend.tolist()))
    print("workload %s, %d workgroups in the last of %d back-to-back launches; %.2f us per launch" %
          (wl.name, len(st), args.launches, e0.elapsed_time(e1) * 1e3 / args.launches))
    print("%-32s %8s %8s %8s %8s %8s" % ("stamp (us since first start)", "min", "p10", "median", "p90", "max"))
    for i, name in enumerate(STAMPS):
        v = np.sort((st[:, i] - t0) / 100.0)
        print("%-32s %8.2f %8.2f %8.2f %8.2f %8.2f" % (name, v[0], v[len(v) // 10], v[len(v) // 2], v[len(v) * 9 // 10], v[-1]))


if __name__ == "__main__":
    main()
