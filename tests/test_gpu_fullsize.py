"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times (automatic
launch shape, conv roll fused into the verify launch, one commit launch over the caches).

The oracle is too slow for every element at these sizes, so it computes sampled (sequence, head)
recurrences one by one -- they are independent, so the sample is exact, not approximate -- while the
integer bookkeeping is still compared for every sequence.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2408_15237_amd as ssmv
from workload import CONFIGS, generate, round_to_io

from _harness import HipLayer, TOL, eager_oracle, rel_err, run_parity, slice_workload, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _auto_tuning():
    ssmv.ssmv_set_tuning(0, 0)
    yield
    ssmv.ssmv_set_tuning(0, 0)


def _sampled_parity(wl, data, seqs, heads, state_every=8, layer=0):
    """Full-size GPU run; oracle on the (seqs x heads) sub-problem."""
    tol = TOL[wl.io]
    P, N = wl.headdim, wl.dstate
    sub_wl, sub, ch = slice_workload(wl, data, seqs, heads, layer)
    ora = eager_oracle(sub_wl, sub.layers[0])
    hip = HipLayer(wl, data.layers[layer])
    bk = oracle.BookkeepingModel(wl.batch, wl.ring_len, wl.conv_width)
    caches = [hip.cache.c]
    worst = 0.0
    for i, rd in enumerate(data.rounds):
        k = rd.x_raw.shape[1]
        srd = sub.rounds[i]
        y_ref, xc_ref, _ = ora.verify(srd.x_raw, srd.dt[0], srd.B[0], srd.C[0])
        y, xc = hip.conv_verify(to_dev(rd.x_raw, wl.io), to_dev(rd.dt[layer], wl.io), to_dev(rd.B[layer], wl.io),
                                to_dev(rd.C[layer], wl.io))
        y_s = to_host(y)[seqs][:, :, ch]
        xc_s = to_host(xc)[seqs][:, :, ch]
        e_y, e_xc = rel_err(y_s, y_ref), rel_err(xc_s, xc_ref)
        assert e_y <= tol and e_xc <= tol, "round %d: y %.3g xc %.3g (bound %.3g)" % (i, e_y, e_xc, tol)
        worst = max(worst, e_y)
        ssmv.ssm_commit_rollback_multi(hip.dims, caches, torch.from_numpy(rd.accepted).to("cuda"))
        ora.commit(srd.accepted)
        bk.verify(k)
        bk.commit(rd.accepted)
        ints = hip.cache.ints()
        assert ints["cur_slot"].tolist() == bk.cur and ints["pend"].tolist() == bk.pend
        assert ints["pos"].tolist() == bk.pos and ints["conv_head"].tolist() == bk.conv_head
        assert ints["win_par"] == bk.win_par and ints["err_flag"] == 0
        if i % state_every == 0 or i == len(data.rounds) - 1:
            h = to_host(hip.materialize())[seqs][:, heads]
            e_h = rel_err(h, ora.h)
            assert e_h <= tol, "round %d: state %.3g" % (i, e_h)
    ssmv.ssmv_check(hip.cache.c)
    return worst


def test_cfg3_full_size_sampled():
    wl = CONFIGS["cfg3"]
    worst = _sampled_parity(wl, generate(wl), seqs=[0, 13, 31], heads=[0, 17, 31])
    print("cfg3 full size: worst y error on the sample %.3g" % worst)


def test_cfg1_full_size_every_element():
    wl = CONFIGS["cfg1"]
    for fused in (False, True):
        run_parity(wl, generate(wl), check_state_every=8, fused=fused)


def test_cfg2_full_size_every_element():
    wl = CONFIGS["cfg2"]
    for fused in (False, True):
        run_parity(wl, generate(wl), check_state_every=8, fused=fused)


def test_cfg4_stack_teacher_forced_from_the_oracle_chain():
    """24 layers in sequence.  The oracle runs its own chain on two sampled sequences (layer output ->
    rounded to bf16 -> fixed projection in fp64 -> rounded to bf16 -> next layer's raw input); each GPU layer is
    fed the ORACLE chain's input for those sequences, so every layer is compared at single-layer tolerance and
    nothing the GPU computed ever enters the oracle.  The other sequences follow the GPU's own chain (projection
    glue by torch.matmul, not part of the library), which keeps every launch at its full size."""
    wl = CONFIGS["cfg4"].scaled(rounds=6)
    data = generate(wl)
    tol = TOL[wl.io]
    seqs = [3, 12]
    heads = list(range(wl.nheads))
    Wp64 = data.Wp.astype(np.float64)
    Wp_dev = to_dev(data.Wp, wl.io)
    layers = [HipLayer(wl, lp) for lp in data.layers]
    oras, subs = [], []
    for li in range(wl.layers):
        sub_wl, sub, _ = slice_workload(wl, data, seqs, heads, li)
        oras.append(eager_oracle(sub_wl, sub.layers[0]))
        subs.append(sub)
    bk = oracle.BookkeepingModel(wl.batch, wl.ring_len, wl.conv_width)
    all_caches = [l.cache.c for l in layers]
    worst = 0.0
    for i, rd in enumerate(data.rounds):
        x_gpu = to_dev(rd.x_raw, wl.io)                       # layer 0 input, all sequences
        x_ora = rd.x_raw[seqs].astype(np.float64)             # oracle chain input, sampled sequences
        for li, layer in enumerate(layers):
            x_gpu[seqs] = to_dev(x_ora, wl.io)                # teacher forcing: CPU values into the GPU, never back
            srd = subs[li].rounds[i]
            y_ref, _, _ = oras[li].verify(x_ora, srd.dt[0], srd.B[0], srd.C[0])
            y, _ = layer.conv_verify(x_gpu, to_dev(rd.dt[li], wl.io), to_dev(rd.B[li], wl.io), to_dev(rd.C[li], wl.io))
            e_y = rel_err(to_host(y)[seqs], y_ref)
            assert e_y <= tol, "round %d layer %d: y error %.3g > %.3g" % (i, li, e_y, tol)
            worst = max(worst, e_y)
            # hand-off to the next layer
            x_gpu = torch.matmul(y, Wp_dev.t()).contiguous()
            x_ora = oracle.round_io(oracle.round_io(y_ref, wl.io) @ Wp64.T, wl.io)
        acc = torch.from_numpy(rd.accepted).to("cuda")
        ssmv.ssm_commit_rollback_multi(layers[0].dims, all_caches, acc)
        bk.verify(wl.k)
        bk.commit(rd.accepted)
        for li, layer in enumerate(layers):
            oras[li].commit(rd.accepted[seqs])
            ints = layer.cache.ints()
            assert ints["cur_slot"].tolist() == bk.cur and ints["pend"].tolist() == bk.pend and ints["pos"].tolist() == bk.pos
        if i == len(data.rounds) - 1:
            for li in (0, 11, 23):
                e_h = rel_err(to_host(layers[li].materialize())[seqs], oras[li].h)
                assert e_h <= tol, "layer %d final state error %.3g" % (li, e_h)
    print("cfg4 stack: worst y error %.3g" % worst)


def test_one_round_as_a_hip_graph_replayed_with_eager_work_in_between():
    """A verify round captured once (kernel nodes only) and replayed for several rounds, with eager work and
    synchronisation between the replays; every replay must equal the eager path bit for bit."""
    wl = CONFIGS["cfg1"].scaled(nheads=4, batch=3, rounds=8)
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
