"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times (automatic
launch shape, conv roll fused into the verify launch, one commit launch over the caches).

The fp64 oracle (OpenMP over sequence x head) does a cfg3 round in some tens of milliseconds, so every
element of every round is compared at every size; the integer bookkeeping is compared for every sequence.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2408_15237_amd as ssmv
from workload import CONFIGS, generate, round_to_io

from _harness import HipLayer, TOL, check_close, eager_oracle, rel_err, run_parity, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _auto_tuning():
    ssmv.ssmv_set_tuning(0, 0)
    yield
    ssmv.ssmv_set_tuning(0, 0)


@pytest.mark.parametrize("engine", ["auto", "vector"])
def test_cfg3_full_size_every_element(engine):
    """All 32 sequences x 32 heads x 64 rounds, every y and conv output, the state every 8 rounds: on the kernel the
    library picks (matrix cores, tiled state) and on the vector kernel (row-major state)."""
    wl = CONFIGS["cfg3"].scaled(engine=engine)
    assert ssmv.ssmv_engine_of(ssmv.make_dims(wl.batch, wl.nheads, wl.headdim, wl.dstate, kmax=wl.k, io=wl.io, engine=engine)) == (engine == "auto")
    worst = run_parity(wl, generate(wl), check_state_every=8, fused=True)
    print("cfg3 full size, engine %s: worst errors %s" % (engine, {k: "%.3g" % v for k, v in worst.items()}))


def test_cfg3_full_size_deferred_advance_every_element():
    """The same with SSMV_SNAP_DEFER, the configuration `bench.py --deferred-advance` times: all 64 rounds, every y and
    conv output, the logical state every 8 rounds, the integers of all 32 sequences every round."""
    wl = CONFIGS["cfg3"].scaled(snapshot_mode="defer")
    worst = run_parity(wl, generate(wl), check_state_every=8, fused=True)
    print("cfg3 full size, deferred advance: worst errors %s" % {k: "%.3g" % v for k, v in worst.items()})


def test_cfg1_full_size_every_element():
    wl = CONFIGS["cfg1"]
    for fused in (False, True):
        run_parity(wl, generate(wl), check_state_every=8, fused=fused)


def test_cfg2_full_size_every_element():
    wl = CONFIGS["cfg2"]
    for fused in (False, True):
        run_parity(wl, generate(wl), check_state_every=8, fused=fused)


def test_cfg4_stack_every_layer_every_sequence():
    """24 layers in sequence, all 16 sequences, all 32 rounds.  The oracle runs its own chain (layer output -> rounded to
    bf16 -> fixed projection in fp64 -> rounded to bf16 -> next layer's raw input).  Two GPU stacks run beside it:
    * teacher-forced: every layer is fed the ORACLE chain's input, so every layer of every round is compared at
      single-layer tolerance and nothing the GPU computed ever enters the oracle;
    * free-running: every layer is fed the previous GPU layer's own output through the projection (torch.matmul: glue,
      not part of the library).  A bf16 output that lands on the other side of a rounding boundary moves the next
      layer's input by one bf16 step, so the chains drift apart by rounding noise; the last layer's output is held to
      FREE_TOL on max|g - r| / max|r|, a bound set from the measured drift (printed) with a margin."""
    FREE_TOL = 0.06
    wl = CONFIGS["cfg4"]
    data = generate(wl)
    tol = TOL[wl.io]
    Wp64 = data.Wp.astype(np.float64)
    Wp_dev = to_dev(data.Wp, wl.io)
    forced = [HipLayer(wl, lp) for lp in data.layers]
    free = [HipLayer(wl, lp) for lp in data.layers]
    oras = [eager_oracle(wl, lp) for lp in data.layers]
    bk = oracle.BookkeepingModel(wl.batch, wl.ring_len, wl.conv_width, mode=wl.snapshot_mode, kmax=wl.kmax_eff)
    worst, worst_free = 0.0, 0.0
    for i, rd in enumerate(data.rounds):
        x_ora = rd.x_raw.astype(np.float64)                   # the oracle chain's input to layer 0
        x_free = to_dev(rd.x_raw, wl.io)
        for li in range(wl.layers):
            dt, Bm, Cm = (to_dev(v[li], wl.io) for v in (rd.dt, rd.B, rd.C))
            y_ref, _, _ = oras[li].verify(x_ora, rd.dt[li], rd.B[li], rd.C[li])
            y, _ = forced[li].conv_verify(to_dev(x_ora, wl.io), dt, Bm, Cm)           # CPU values into the GPU, never back
            e_y, _ = check_close(to_host(y), y_ref, tol, "round %d layer %d: y" % (i, li))
            worst = max(worst, e_y)
            y_f, _ = free[li].conv_verify(x_free, dt, Bm, Cm)
            if li == wl.layers - 1:
                m = float(np.max(np.abs(to_host(y_f) - y_ref)) / np.max(np.abs(y_ref)))
                worst_free = max(worst_free, m)
                assert m <= FREE_TOL, "round %d: free-running chain, last layer: %.3g" % (i, m)
            # hand-off to the next layer
            x_free = torch.matmul(y_f, Wp_dev.t()).contiguous()
            x_ora = oracle.round_io(oracle.round_io(y_ref, wl.io) @ Wp64.T, wl.io)
        acc = torch.from_numpy(rd.accepted).to("cuda")
        for stack in (forced, free):
            ssmv.ssm_commit_rollback_multi(stack[0].dims, [l.cache.c for l in stack], acc)
        bk.verify(wl.k)
        bk.commit(rd.accepted)
        for li in range(wl.layers):
            oras[li].commit(rd.accepted)
            for stack in (forced, free):
                ints = stack[li].cache.ints()
                assert ints["cur_slot"].tolist() == bk.cur and ints["pend"].tolist() == bk.pend and ints["pos"].tolist() == bk.pos
                assert ints["conv_head"].tolist() == bk.conv_head and ints["err_flag"] == 0
        if i % 8 == 7 or i == len(data.rounds) - 1:
            for li in (0, 11, 23):
                check_close(to_host(forced[li].materialize()), oras[li].h, tol, "round %d layer %d: state" % (i, li))
    print("cfg4 stack: worst y error, teacher-forced %.3g; free-running last layer max|g-r|/max|r| %.3g" % (worst, worst_free))


@pytest.mark.parametrize("snap", ["both", "defer"])
def test_one_round_as_a_hip_graph_replayed_with_eager_work_in_between(snap):
    """A verify round captured once (kernel nodes only) and replayed for several rounds, with eager work and
    synchronisation between the replays; every replay must equal the eager path bit for bit.  With the deferred advance
    the window entries a replay reads and writes follow from pos and pend on the device, round after round."""
    wl = CONFIGS["cfg1"].scaled(nheads=4, batch=3, rounds=8 if snap == "both" else 20, snapshot_mode=snap)
    data = generate(wl)
    lp = data.layers[0]
    eager, graphed = HipLayer(wl, lp), HipLayer(wl, lp)
    sx = torch.empty((wl.batch, wl.k, wl.conv_channels), dtype=torch.bfloat16, device="cuda")
    sdt = torch.empty((wl.batch, wl.k, wl.nheads), dtype=torch.bfloat16, device="cuda")
    sB = torch.empty((wl.batch, wl.k, wl.ngroups, wl.dstate), dtype=torch.bfloat16, device="cuda")
    sC = torch.empty_like(sB)
    sacc = torch.empty(wl.batch, dtype=torch.int32, device="cuda")
    sy = torch.empty_like(sx)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        g.capture_begin()
        ssmv.ssm_conv_verify_multistep(graphed.dims, graphed.cache.c, sx, graphed.conv_w, graphed.conv_b, sdt, sB, sC,
                                       graphed.A, graphed.D, wl.k, sy)
        ssmv.ssm_commit_rollback(graphed.dims, graphed.cache.c, sacc)
        g.capture_end()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for rd in data.rounds:
        dx, ddt, dB, dC = (to_dev(v, wl.io) for v in (rd.x_raw, rd.dt[0], rd.B[0], rd.C[0]))
        acc = torch.from_numpy(rd.accepted).to("cuda")
        y_e, _ = eager.conv_verify(dx, ddt, dB, dC)
        eager.commit(acc)
        sx.copy_(dx); sdt.copy_(ddt); sB.copy_(dB); sC.copy_(dC); sacc.copy_(acc)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(sy, y_e)
        assert torch.equal(graphed.materialize(), eager.materialize())       # eager work between the replays
        a, b = graphed.cache.ints(), eager.cache.ints()
        for name in ("cur_slot", "pend", "pos", "conv_head", "last_k"):
            assert np.array_equal(a[name], b[name])
        assert a["win_par"] == b["win_par"]
