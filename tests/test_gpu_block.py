"""GPU parity of the optional pieces around the recurrence (ssm_block_multistep): the step-size transform
softplus(dt + dt_bias), the SiLU output gate, and rounds that several calls feed (the draft side)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2408_15237_amd as ssmv
from workload import CONFIGS, block_extras, generate

from _harness import HipLayer, TOL, dims_of, rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _auto_tuning():
    ssmv.ssmv_set_tuning(0, 0)
    yield
    ssmv.ssmv_set_tuning(0, 0)


def _block_oracle(wl, lp, bias, softplus):
    return oracle.EagerOracle(wl.a_mode, lp.A, lp.D, lp.conv_w, lp.conv_b, lp.h0, wl.io, wl.conv_act, wl.ngroups,
                              dt_bias=bias, dt_softplus=softplus)


def _check_ints(hip, bk, where):
    ints = hip.cache.ints()
    assert ints["cur_slot"].tolist() == bk.cur, where
    assert ints["pend"].tolist() == bk.pend, where
    assert ints["pos"].tolist() == bk.pos, where
    assert ints["conv_head"].tolist() == bk.conv_head, where
    assert ints["last_k"].tolist() == bk.last_k, where
    assert ints["win_par"] == bk.win_par and ints["err_flag"] == bk.err == 0, where


CASES = {
    "cfg0": CONFIGS["cfg0"],
    "cfg1_small": CONFIGS["cfg1"].scaled(nheads=4, batch=3, rounds=10),
    "cfg2_small": CONFIGS["cfg2"].scaled(nheads=192, rounds=10),
    "f32_groups": CONFIGS["cfg0"].scaled(io="f32", ngroups=2, nheads=4, batch=5, k=3, kmax=5, rounds=10),
    "ragged_rows": CONFIGS["cfg0"].scaled(headdim=24, dstate=32, batch=3, rounds=8),
    "cfg1_full": CONFIGS["cfg1"].scaled(rounds=8),              # the 8B-shaped layer at its full size, every element
    # the deferred advance: window ring, states stored only when it fills up (matrix-core engine; vector engine, fp32)
    "cfg1_small_defer": CONFIGS["cfg1"].scaled(nheads=4, batch=3, rounds=24, snapshot_mode="defer"),
    "f32_groups_defer": CONFIGS["cfg0"].scaled(io="f32", ngroups=2, nheads=4, batch=5, k=3, kmax=5, rounds=20, snapshot_mode="defer"),
}


@pytest.mark.parametrize("fused", [False, True], ids=["split", "fused"])
@pytest.mark.parametrize("gate", [False, True], ids=["nogate", "gate"])
@pytest.mark.parametrize("name", sorted(CASES))
def test_step_size_transform_and_gate(name, gate, fused):
    wl = CASES[name]
    data = generate(wl)
    ex = block_extras(data)
    lp, bias = data.layers[0], ex.dt_bias[0]
    tol = TOL[wl.io]
    hip = HipLayer(wl, lp)
    ora = _block_oracle(wl, lp, bias, True)
    bk = oracle.BookkeepingModel(wl.batch, wl.ring_len, wl.conv_width, mode=wl.snapshot_mode, kmax=wl.kmax_eff)
    d_bias = torch.from_numpy(bias).to("cuda")
    for i, rd in enumerate(data.rounds):
        k = rd.x_raw.shape[1]
        z = ex.z[i] if gate else None
        y_ref, xc_ref, _ = ora.verify(rd.x_raw, ex.dt_raw[i][0], rd.B[0], rd.C[0], z=z)
        d_x = to_dev(rd.x_raw, wl.io)
        y = torch.empty_like(d_x)
        kw = dict(dt=to_dev(ex.dt_raw[i][0], wl.io), Bm=to_dev(rd.B[0], wl.io), Cm=to_dev(rd.C[0], wl.io), A=hip.A, D=hip.D,
                  k=k, y_out=y, dt_bias=d_bias, dt_softplus=True, z=None if z is None else to_dev(z, wl.io))
        if fused:
            ssmv.ssm_block_multistep(hip.dims, hip.cache.c, x_raw=d_x, conv_wgt=hip.conv_w, conv_bias=hip.conv_b, **kw)
        else:
            ssmv.ssm_block_multistep(hip.dims, hip.cache.c, xc=hip.conv(d_x), **kw)
        bk.verify(k)
        e_y = rel_err(to_host(y), y_ref)
        assert e_y <= tol, "round %d: y error %.3g > %.3g" % (i, e_y, tol)
        hip.commit(torch.from_numpy(rd.accepted.astype(np.int32)).to("cuda"))
        ora.commit(rd.accepted)
        bk.commit(rd.accepted)
        _check_ints(hip, bk, "round %d" % i)
        h = torch.empty((wl.batch, wl.nheads, wl.headdim, wl.dstate), dtype=torch.float32, device="cuda")
        ssmv.ssmv_materialize_block(hip.dims, hip.cache.c, hip.A, d_bias, True, h)
        e_h = rel_err(to_host(h), ora.h)
        assert e_h <= tol, "round %d: state error %.3g > %.3g" % (i, e_h, tol)
    ssmv.ssmv_check(hip.cache.c)


def test_transform_off_and_no_gate_is_the_plain_call_bit_for_bit():
    wl = CASES["cfg1_small"]
    data = generate(wl)
    a, b = HipLayer(wl, data.layers[0]), HipLayer(wl, data.layers[0])
    for rd in data.rounds:
        d_x, d_dt, d_B, d_C = (to_dev(v, wl.io) for v in (rd.x_raw, rd.dt[0], rd.B[0], rd.C[0]))
        y_a, _ = a.conv_verify(d_x, d_dt, d_B, d_C)
        y_b = torch.empty_like(d_x)
        ssmv.ssm_block_multistep(b.dims, b.cache.c, x_raw=d_x, conv_wgt=b.conv_w, conv_bias=b.conv_b, dt=d_dt, Bm=d_B, Cm=d_C,
                                 A=b.A, D=b.D, k=rd.x_raw.shape[1], y_out=y_b)
        assert torch.equal(y_a, y_b)
        acc = torch.from_numpy(rd.accepted.astype(np.int32)).to("cuda")
        a.commit(acc); b.commit(acc)
    assert torch.equal(a.cache.state_view(), b.cache.state_view())


SPLITS = {"ones": None, "2+2": [2, 2], "1+3": [1, 3], "3+1": [3, 1]}


@pytest.mark.parametrize("split", sorted(SPLITS))
@pytest.mark.parametrize("name", ["cfg0", "cfg1_small", "cfg2_small", "f32_groups"])
def test_round_fed_by_several_calls_equals_one_call(name, split):
    """Draft side: the calls of one round (first with tok0 = 0, later ones continuing in the h_k slot) leave the
    window, the ring and - after the same commit - the integers exactly as ONE call with all the tokens does,
    and the outputs and the three slots equal up to fp32 rounding (the kernel rescales the state by the decay
    accumulated over the tokens of a launch, so the split changes the rounding); both match the oracle."""
    wl = CASES[name]
    data = generate(wl)
    lp = data.layers[0]
    tol = TOL[wl.io]
    one, many = HipLayer(wl, lp), HipLayer(wl, lp)
    ora = oracle.EagerOracle(wl.a_mode, lp.A, lp.D, lp.conv_w, lp.conv_b, lp.h0, wl.io, wl.conv_act, wl.ngroups)
    bk = oracle.BookkeepingModel(wl.batch, wl.ring_len, wl.conv_width, mode=wl.snapshot_mode, kmax=wl.kmax_eff)
    for i, rd in enumerate(data.rounds):
        k = rd.x_raw.shape[1]
        parts = SPLITS[split] if SPLITS[split] is not None and sum(SPLITS[split]) == k else [1] * k
        d_x, d_dt, d_B, d_C = (to_dev(v, wl.io) for v in (rd.x_raw, rd.dt[0], rd.B[0], rd.C[0]))
        y_one, _ = one.conv_verify(d_x, d_dt, d_B, d_C)
        y_ref, _, _ = ora.verify(rd.x_raw, rd.dt[0], rd.B[0], rd.C[0])
        t0, ys = 0, []
        for n in parts:
            sl = slice(t0, t0 + n)
            y = torch.empty_like(d_x[:, sl])
            ssmv.ssm_block_multistep(many.dims, many.cache.c, x_raw=d_x[:, sl].contiguous(), conv_wgt=many.conv_w,
                                     conv_bias=many.conv_b, dt=d_dt[:, sl].contiguous(), Bm=d_B[:, sl].contiguous(),
                                     Cm=d_C[:, sl].contiguous(), A=many.A, D=many.D, k=n, tok0=t0, y_out=y)
            bk.verify(n, tok0=t0)
            ys.append(y)
            t0 += n
        y_many = torch.cat(ys, dim=1)
        assert rel_err(to_host(y_many), to_host(y_one)) <= tol, "round %d: outputs differ from the single call" % i
        assert rel_err(to_host(y_many), y_ref) <= tol
        assert many.cache.ints()["last_k"].tolist() == [k] * wl.batch
        acc = torch.from_numpy(rd.accepted.astype(np.int32)).to("cuda")
        one.commit(acc); many.commit(acc)
        ora.commit(rd.accepted)
        bk.commit(rd.accepted)
        _check_ints(many, bk, "round %d" % i)
        idx = torch.from_numpy(many.cache.ints()["cur_slot"]).long()
        live_many, live_one = (v.cache.state_view()[idx, torch.arange(wl.batch)] for v in (many, one))
        # fp32 rounding on the vector path; on the matrix-core path (bf16 tokens) every fp32 operand of a product enters
        # as a bf16 head plus tail, 2^-17 relative per product, and the split decides which products are formed
        h_same = 1e-5 if wl.io == "f32" else 1e-4
        assert rel_err(to_host(live_many), to_host(live_one)) <= h_same, "round %d: live slots differ" % i
        assert rel_err(to_host(many.materialize()), to_host(one.materialize())) <= h_same, "round %d: states differ" % i
        for nm in ("conv_ring", "win_xc0", "win_xc1", "win_dt0", "win_dt1", "win_B0", "win_B1"):
            assert torch.equal(many.cache.buffers[nm], one.cache.buffers[nm]), nm
        assert rel_err(to_host(many.materialize()), ora.h) <= tol
    ssmv.ssmv_check(many.cache.c)


REPLAY_CASES = {
    "cfg1_small": CONFIGS["cfg1"].scaled(nheads=4, batch=3, rounds=10),
    "k8_narrow_heads": CONFIGS["cfg1"].scaled(nheads=3, headdim=64, dstate=128, batch=2, k=8, rounds=10, ngroups=1),
    "cfg1_small_hj": CONFIGS["cfg1"].scaled(nheads=4, batch=3, rounds=10, snapshot_mode="hj_only"),
    "cfg1_small_defer": CONFIGS["cfg1"].scaled(nheads=4, batch=3, rounds=14, snapshot_mode="defer"),
    "groups_silu": CONFIGS["cfg1"].scaled(nheads=4, headdim=64, dstate=32, ngroups=2, batch=5, rounds=8, conv_act="silu"),
}
REPLAY_SPLITS = {"ones": None, "2+2": [2, 2], "1+3": [1, 3], "3+1": [3, 1], "1+5+2": [1, 5, 2]}


@pytest.mark.parametrize("split", sorted(REPLAY_SPLITS))
@pytest.mark.parametrize("name", sorted(REPLAY_CASES))
def test_replayed_round_equals_one_call(name, split):
    """replay_round: every call of a round recomputes from the live slot (pending tokens, then the round's earlier
    tokens out of the round's stash), only the last one stores h_j and h_k.  Outputs, window, ring, integers and - after
    the last call - the slots must be what ONE call with all the tokens leaves; no slot changes before the last call;
    a call repeated gives the same outputs."""
    wl = REPLAY_CASES[name]
    parts0 = REPLAY_SPLITS[split]
    if parts0 is not None and sum(parts0) != wl.k:
        pytest.skip("split does not add up to this case's k")
    data = generate(wl)
    lp = data.layers[0]
    tol = TOL[wl.io]
    one, many = HipLayer(wl, lp), HipLayer(wl, lp)
    assert ssmv.ssmv_engine_of(many.dims) == 1
    ora = oracle.EagerOracle(wl.a_mode, lp.A, lp.D, lp.conv_w, lp.conv_b, lp.h0, wl.io, wl.conv_act, wl.ngroups)
    bk = oracle.BookkeepingModel(wl.batch, wl.ring_len, wl.conv_width, mode=wl.snapshot_mode, kmax=wl.kmax_eff)
    for i, rd in enumerate(data.rounds):
        k = rd.x_raw.shape[1]
        parts = parts0 if parts0 is not None else [1] * k
        d_x, d_dt, d_B, d_C = (to_dev(v, wl.io) for v in (rd.x_raw, rd.dt[0], rd.B[0], rd.C[0]))
        y_one, _ = one.conv_verify(d_x, d_dt, d_B, d_C)
        y_ref, _, _ = ora.verify(rd.x_raw, rd.dt[0], rd.B[0], rd.C[0])
        slots_before = many.cache.state_view().clone()
        t0, ys = 0, []
        for ci, n in enumerate(parts):
            sl = slice(t0, t0 + n)
            last = ci == len(parts) - 1
            outs = []
            for rep in range(2):                           # every call twice: idempotent
                y = torch.empty_like(d_x[:, sl])
                ssmv.ssm_block_multistep(many.dims, many.cache.c, x_raw=d_x[:, sl].contiguous(), conv_wgt=many.conv_w,
                                         conv_bias=many.conv_b, dt=d_dt[:, sl].contiguous(), Bm=d_B[:, sl].contiguous(),
                                         Cm=d_C[:, sl].contiguous(), A=many.A, D=many.D, k=n, tok0=t0, y_out=y,
                                         replay_round=True, last_call=last)
                outs.append(y)
            assert torch.equal(outs[0], outs[1]), "round %d call %d is not idempotent" % (i, ci)
            if not last:
                assert torch.equal(many.cache.state_view(), slots_before), "round %d call %d touched a slot" % (i, ci)
            bk.verify(n, tok0=t0)
            ys.append(outs[0])
            t0 += n
        y_many = torch.cat(ys, dim=1)
        assert rel_err(to_host(y_many), y_ref) <= tol, "round %d" % i
        assert rel_err(to_host(y_many), to_host(y_one)) <= tol
        assert many.cache.ints()["last_k"].tolist() == [k] * wl.batch
        # the slots after the last call against the single call's (2^-17 per product, and the split decides which are formed)
        assert rel_err(to_host(many.cache.state_view()), to_host(one.cache.state_view())) <= 1e-4, "round %d: slots" % i
        acc = torch.from_numpy(rd.accepted.astype(np.int32)).to("cuda")
        one.commit(acc); many.commit(acc)
        ora.commit(rd.accepted)
        bk.commit(rd.accepted)
        _check_ints(many, bk, "round %d" % i)
        for nm in ("conv_ring", "win_xc0", "win_xc1", "win_dt0", "win_dt1", "win_B0", "win_B1"):
            assert torch.equal(many.cache.buffers[nm], one.cache.buffers[nm]), nm
        assert rel_err(to_host(many.materialize()), ora.h) <= tol
    ssmv.ssmv_check(many.cache.c)


def test_draft_model_round_trip_with_rejections():
    """A draft-side round as the paper describes it: k single-token calls (the first recomputes the tokens
    accepted last round), then the verifier's verdict rolls the draft's own cache back."""
    wl = CONFIGS["cfg1"].scaled(nheads=4, batch=4, rounds=12, accept="geometric", accept_p=0.4)
    data = generate(wl)
    ex = block_extras(data)
    lp, bias = data.layers[0], ex.dt_bias[0]
    hip = HipLayer(wl, lp)
    ora = _block_oracle(wl, lp, bias, True)
    d_bias = torch.from_numpy(bias).to("cuda")
    tol = TOL[wl.io]
    for i, rd in enumerate(data.rounds):
        k = rd.x_raw.shape[1]
        y_ref, _, _ = ora.verify(rd.x_raw, ex.dt_raw[i][0], rd.B[0], rd.C[0], z=ex.z[i])
        d_x, d_dt, d_B, d_C, d_z = (to_dev(v, wl.io) for v in (rd.x_raw, ex.dt_raw[i][0], rd.B[0], rd.C[0], ex.z[i]))
        for t in range(k):
            sl = slice(t, t + 1)
            y = torch.empty_like(d_x[:, sl])
            ssmv.ssm_block_multistep(hip.dims, hip.cache.c, x_raw=d_x[:, sl].contiguous(), conv_wgt=hip.conv_w, conv_bias=hip.conv_b,
                                     dt=d_dt[:, sl].contiguous(), dt_bias=d_bias, dt_softplus=True, Bm=d_B[:, sl].contiguous(),
                                     Cm=d_C[:, sl].contiguous(), z=d_z[:, sl].contiguous(), A=hip.A, D=hip.D, k=1, tok0=t, y_out=y)
            e = rel_err(to_host(y), y_ref[:, sl])
            assert e <= tol, "round %d token %d: %.3g" % (i, t, e)
        hip.commit(torch.from_numpy(rd.accepted.astype(np.int32)).to("cuda"))
        ora.commit(rd.accepted)
    h = torch.empty((wl.batch, wl.nheads, wl.headdim, wl.dstate), dtype=torch.float32, device="cuda")
    ssmv.ssmv_materialize_block(hip.dims, hip.cache.c, hip.A, d_bias, True, h)
    assert rel_err(to_host(h), ora.h) <= tol
    ssmv.ssmv_check(hip.cache.c)


@pytest.mark.parametrize("fused", [False, True], ids=["split", "fused"])
@pytest.mark.parametrize("name", ["cfg0", "cfg1_small", "cfg2_small", "f32_groups", "cfg1_small_defer", "f32_groups_defer"])
def test_ragged_draft_counts(name, fused):
    """Per-sequence draft counts k_seq[b] <= k.  The recurrence is causal, so the oracle's outputs and states for
    the first kb tokens of a sequence do not depend on the tokens behind them: the oracle verifies all k tokens
    and commits min(accepted, kb); the GPU must match it on y[b][:kb], write zeros behind, report last_k = kb
    and keep the integer model's bookkeeping (which clamps accepted to last_k)."""
    wl = CASES[name].scaled(batch=max(CASES[name].batch, 4))
    data = generate(wl)
    lp = data.layers[0]
    tol = TOL[wl.io]
    rng = np.random.default_rng(77)
    hip = HipLayer(wl, lp)
    ora = oracle.EagerOracle(wl.a_mode, lp.A, lp.D, lp.conv_w, lp.conv_b, lp.h0, wl.io, wl.conv_act, wl.ngroups)
    bk = oracle.BookkeepingModel(wl.batch, wl.ring_len, wl.conv_width, mode=wl.snapshot_mode, kmax=wl.kmax_eff)
    for i, rd in enumerate(data.rounds):
        k = rd.x_raw.shape[1]
        kseq = rng.integers(1, k + 1, size=wl.batch).astype(np.int32)
        if i == 0:
            kseq[:2] = [k, 1]                                   # the two ends in one launch
        d_x, d_dt, d_B, d_C = (to_dev(v, wl.io) for v in (rd.x_raw, rd.dt[0], rd.B[0], rd.C[0]))
        y = torch.full_like(d_x, 7.0)
        kw = dict(dt=d_dt, Bm=d_B, Cm=d_C, A=hip.A, D=hip.D, k=k, y_out=y, k_seq=torch.from_numpy(kseq).to("cuda"))
        if fused:
            ssmv.ssm_block_multistep(hip.dims, hip.cache.c, x_raw=d_x, conv_wgt=hip.conv_w, conv_bias=hip.conv_b, **kw)
        else:
            ssmv.ssm_block_multistep(hip.dims, hip.cache.c, xc=hip.conv(d_x), **kw)
        y_ref, _, _ = ora.verify(rd.x_raw, rd.dt[0], rd.B[0], rd.C[0])
        y_h = to_host(y)
        for b in range(wl.batch):
            kb = int(kseq[b])
            assert rel_err(y_h[b, :kb], y_ref[b, :kb]) <= tol, "round %d seq %d" % (i, b)
            assert np.all(y_h[b, kb:] == 0.0), "round %d seq %d: tokens not taken must read as zeros" % (i, b)
        assert hip.cache.ints()["last_k"].tolist() == kseq.tolist()
        bk.last_k = kseq.tolist()                               # what verify sets, per sequence
        acc = rd.accepted.astype(np.int32)
        hip.commit(torch.from_numpy(acc).to("cuda"))
        clamped = np.minimum(acc, kseq)
        err_expected = bool(np.any(acc > kseq))
        ora.commit(clamped)
        bk.commit(acc)
        assert bk.err == int(err_expected) or bk.err == 1
        ints = hip.cache.ints()
        assert ints["cur_slot"].tolist() == bk.cur and ints["pend"].tolist() == bk.pend
        assert ints["pos"].tolist() == bk.pos and ints["conv_head"].tolist() == bk.conv_head
        assert ints["win_par"] == bk.win_par and ints["err_flag"] == bk.err
        assert rel_err(to_host(hip.materialize()), ora.h) <= tol, "round %d: state" % i


@pytest.mark.parametrize("io,channels,group,gate", [("bf16", 4096, 4096, True), ("bf16", 4096, 512, False), ("f32", 192, 64, True),
                                                     ("bf16", 8192, 8192, True), ("f32", 96, 4, False), ("bf16", 2304, 768, True)])
def test_gated_rmsnorm(io, channels, group, gate):
    from workload import round_to_io
    rng = np.random.default_rng(91)
    rows = 37
    y = round_to_io(rng.standard_normal((rows, channels)) * 3, io)
    z = round_to_io(rng.standard_normal((rows, channels)), io) if gate else None
    w = rng.standard_normal(channels).astype(np.float32)
    out = torch.empty_like(to_dev(y, io))
    ssmv.ssmv_gated_rmsnorm(to_dev(y, io), None if z is None else to_dev(z, io), torch.from_numpy(w).to("cuda"), rows, channels, group,
                            1e-5, io, out)
    ref = oracle.rmsnorm_gated(y, z, w, group, 1e-5)
    assert rel_err(to_host(out), ref) <= (1e-5 if io == "f32" else TOL[io])
