"""GPU parity: the HIP library (through its C ABI) against the fp64 CPU oracle, element by element.

Sizes are chosen so that the oracle finishes in seconds while the kernels still see several
workgroup tiles and ragged tails; the full benchmark shapes are covered in test_gpu_fullsize.py.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2408_15237_amd as ssmv
from workload import CONFIGS, Workload, generate

from _harness import HipLayer, TOL, dims_of, rel_err, run_parity, to_dev, to_host, untile_state

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _auto_tuning():
    ssmv.ssmv_set_tuning(0, 0)
    yield
    ssmv.ssmv_set_tuning(0, 0)


FUSED = pytest.mark.parametrize("fused", [False, True], ids=["split", "fused"])


@FUSED
def test_cfg0_tiny_fp32(fused):
    wl = CONFIGS["cfg0"]
    worst = run_parity(wl, generate(wl), reverify=True, fused=fused)
    print("cfg0 worst errors", worst)


@FUSED
def test_cfg1_shape_reduced_batch_bf16(fused):
    wl = CONFIGS["cfg1"].scaled(nheads=4, rounds=16)
    run_parity(wl, generate(wl), reverify=True, fused=fused)


@FUSED
def test_cfg1_shape_reduced_fp32(fused):
    wl = CONFIGS["cfg1"].scaled(nheads=3, rounds=16, io="f32", batch=2)
    run_parity(wl, generate(wl), fused=fused)


@FUSED
@pytest.mark.parametrize("rows,waves", [(r, w) for r in (1, 2, 4, 8) for w in (1, 2, 4)])
def test_every_launch_shape_scalar(rows, waves, fused):
    ssmv.ssmv_set_tuning(rows, waves)
    wl = Workload("shape", "scalar", batch=3, nheads=3, headdim=72, dstate=64, k=4, rounds=8, io="f32",
                  accept="uniform", seed=rows * 10 + waves)
    run_parity(wl, generate(wl), fused=fused)


@FUSED
@pytest.mark.parametrize("rows,waves", [(r, w) for r in (1, 2, 4) for w in (1, 2, 4)])
def test_every_launch_shape_diag(rows, waves, fused):
    ssmv.ssmv_set_tuning(rows, waves)
    wl = Workload("shaped", "diag", batch=2, nheads=203, headdim=1, dstate=16, k=5, rounds=8, io="f32",
                  accept="geometric", seed=rows * 10 + waves)
    run_parity(wl, generate(wl), fused=fused)


@FUSED
@pytest.mark.parametrize("N,P,G,io", [(16, 24, 1, "f32"), (32, 20, 2, "bf16"), (64, 40, 2, "f32"),
                                      (128, 12, 1, "f32"), (256, 6, 4, "bf16"), (64, 1, 1, "f32"), (16, 100, 4, "bf16"),
                                      (64, 128, 1, "bf16"), (128, 64, 8, "bf16")])
def test_state_sizes_groups_and_ragged_tiles(N, P, G, io, fused):
    wl = Workload("sz", "scalar", batch=2, nheads=8 if G == 8 else 4, headdim=P, dstate=N, k=3, rounds=10, io=io,
                  accept="uniform", ngroups=G, kmax=5, seed=N + P)
    run_parity(wl, generate(wl), fused=fused)


@FUSED
@pytest.mark.parametrize("N,io", [(16, "bf16"), (32, "f32"), (64, "bf16")])
def test_diag_mode(N, io, fused):
    wl = CONFIGS["cfg2"].scaled(nheads=1000, dstate=N, rounds=12, io=io, batch=2)
    run_parity(wl, generate(wl), reverify=True, fused=fused)


@FUSED
@pytest.mark.parametrize("act,bias", [("silu", True), ("none", False), ("silu", False)])
@pytest.mark.parametrize("P,io", [(36, "bf16"), (64, "bf16"), (64, "f32")])
def test_conv_variants_and_initial_history(act, bias, P, io, fused):
    wl = Workload("conv", "scalar", batch=2, nheads=2, headdim=P, dstate=16, k=4, rounds=8, io=io,
                  accept="uniform", conv_act=act, conv_bias=bias, seed=5)
    data = generate(wl)
    init = np.random.default_rng(1).standard_normal((wl.batch, wl.conv_width - 1, wl.conv_channels)).astype(np.float32)
    from workload import round_to_io
    run_parity(wl, data, conv_init=round_to_io(init, wl.io), fused=fused)


@FUSED
def test_conv_scalar_channel_path(fused):
    # channel count that is no multiple of the 16-byte vector: one channel at a time
    wl = Workload("convs", "scalar", batch=2, nheads=3, headdim=7, dstate=16, k=4, rounds=6, io="bf16",
                  accept="uniform", seed=6)
    run_parity(wl, generate(wl), fused=fused)


@FUSED
def test_varying_k_up_to_the_limit(fused):
    ks = [1, 16, 7, 16, 2, 9, 1, 1, 16, 4]
    wl = Workload("kmax", "scalar", batch=3, nheads=2, headdim=32, dstate=64, k=4, kmax=16, rounds=len(ks), io="f32",
                  accept="uniform", seed=8)
    run_parity(wl, generate(wl, k_schedule=ks), fused=fused)


@FUSED
def test_varying_k_diag(fused):
    ks = [3, 16, 1, 12, 16, 5]
    wl = Workload("kmaxd", "diag", batch=2, nheads=70, headdim=1, dstate=16, k=4, kmax=16, rounds=len(ks), io="bf16",
                  accept="uniform", seed=9)
    run_parity(wl, generate(wl, k_schedule=ks), fused=fused)


@FUSED
def test_large_k_on_the_8b_shape(fused):
    # k = 16 with up to 15 pending tokens: the staging needs more than one pass per thread
    ks = [16, 16, 8, 16, 16, 3]
    wl = CONFIGS["cfg1"].scaled(nheads=2, batch=3, kmax=16, rounds=len(ks), seed=21)
    data = generate(wl, k_schedule=ks)
    data.rounds[0].accepted[:] = [15, 7, 16]
    data.rounds[1].accepted[:] = [15, 15, 2]
    run_parity(wl, data, fused=fused)


@FUSED
@pytest.mark.parametrize("accept", ["all", "none"])
def test_accept_streaks(accept, fused):
    wl = Workload("streak", "scalar", batch=2, nheads=2, headdim=64, dstate=64, k=4, rounds=7, io="bf16",
                  accept=accept, seed=10)
    run_parity(wl, generate(wl), fused=fused)


@FUSED
def test_mixed_pending_counts_in_one_batch(fused):
    wl = Workload("mixed", "scalar", batch=9, nheads=2, headdim=64, dstate=64, k=6, rounds=12, io="f32",
                  accept="uniform", seed=11)
    data = generate(wl)
    # force every pend value 0..k-1 to occur together in one launch
    data.rounds[0].accepted[:] = [0, 1, 2, 3, 4, 5, 6, 3, 0]
    run_parity(wl, data, fused=fused)


@FUSED
@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("dt_scale", [60.0, 400.0, 4000.0])
def test_strong_decay(dt_scale, io, fused):
    """The scalar-mode kernel carries the state divided by the decay accumulated over the tokens of a launch.  With
    dt*|A| of order 1 per token (x60) that scale has to be folded back every few tokens, with dt*|A| of tens (x400)
    every token, and beyond 64*ln2 per token (x4000: the decay underflows to 0) the plain step has to take over;
    k = 8 with up to 7 pending tokens gives launches of 15 tokens."""
    from workload import round_to_io
    wl = Workload("decay", "scalar", batch=3, nheads=4, headdim=32, dstate=64, k=8, rounds=8, io=io,
                  accept="uniform", seed=21)
    data = generate(wl)
    for rd in data.rounds:
        rd.dt[0] = round_to_io(rd.dt[0] * dt_scale, io)
    run_parity(wl, data, fused=fused)


@FUSED
def test_k1_single_step_rounds(fused):
    wl = Workload("k1", "scalar", batch=2, nheads=2, headdim=64, dstate=64, k=1, rounds=10, io="f32",
                  accept="uniform", seed=12)
    run_parity(wl, generate(wl), fused=fused)


@FUSED
@pytest.mark.parametrize("case", ["cfg1", "cfg2", "kmax16", "all", "none", "mixed"])
def test_single_snapshot_variant(case, fused):
    """SSMV_SNAP_HJ_ONLY: h_k is never stored and every accepted token stays pending (up to kmax of them);
    outputs, logical state and the integer model's bookkeeping must still match."""
    if case == "cfg1":
        wl, ks = CONFIGS["cfg1"].scaled(nheads=4, batch=3, rounds=16, snapshot_mode="hj_only"), None
    elif case == "cfg2":
        wl, ks = CONFIGS["cfg2"].scaled(nheads=1000, batch=2, rounds=12, snapshot_mode="hj_only"), None
    elif case == "kmax16":
        ks = [16, 16, 1, 16, 7, 16, 16, 2]
        wl = Workload("hj16", "scalar", batch=3, nheads=2, headdim=64, dstate=64, k=4, kmax=16, rounds=len(ks), io="f32",
                      accept="uniform", seed=31, snapshot_mode="hj_only")
    elif case in ("all", "none"):
        wl, ks = Workload("hjs", "scalar", batch=2, nheads=2, headdim=64, dstate=64, k=4, rounds=7, io="bf16",
                          accept=case, seed=32, snapshot_mode="hj_only"), None
    else:
        wl, ks = Workload("hjm", "scalar", batch=9, nheads=2, headdim=64, dstate=64, k=6, rounds=12, io="f32",
                          accept="uniform", seed=33, snapshot_mode="hj_only"), None
    data = generate(wl, k_schedule=ks)
    if case == "kmax16":
        data.rounds[0].accepted[:] = [16, 16, 9]           # a fully accepted round leaves kmax tokens pending
        data.rounds[1].accepted[:] = [16, 0, 16]
    if case == "mixed":
        data.rounds[0].accepted[:] = [0, 1, 2, 3, 4, 5, 6, 6, 0]
    run_parity(wl, data, fused=fused, reverify=True)


DEFER_CASES = {
    # matrix-core engine (bf16, tiled slots): pend_hi = 8, pend up to 12
    "cfg1": (CONFIGS["cfg1"].scaled(nheads=4, batch=5, rounds=40, snapshot_mode="defer"), None),
    "cfg1_all": (CONFIGS["cfg1"].scaled(nheads=2, batch=2, rounds=9, snapshot_mode="defer", accept="all"), None),
    "cfg1_none": (CONFIGS["cfg1"].scaled(nheads=2, batch=2, rounds=5, snapshot_mode="defer", accept="none"), None),
    "groups_n32_silu": (CONFIGS["cfg1"].scaled(nheads=4, headdim=64, dstate=32, ngroups=2, batch=5, rounds=24, conv_act="silu",
                                               snapshot_mode="defer"), None),
    "n128_k6": (CONFIGS["cfg1"].scaled(nheads=3, headdim=64, dstate=128, batch=2, k=6, rounds=20, snapshot_mode="defer"), None),
    "k8_is_single_snapshot": (CONFIGS["cfg1"].scaled(nheads=2, batch=3, k=8, rounds=10, snapshot_mode="defer"), None),
    "kmax5_varying_k": (CONFIGS["cfg1"].scaled(nheads=2, batch=3, k=4, kmax=5, rounds=16, snapshot_mode="defer"),
                        [5, 1, 5, 5, 2, 3, 5, 1, 1, 4, 5, 5, 2, 5, 3, 5]),
    # vector engine: the same shape forced, fp32 tokens, diagonal A
    "cfg1_vector": (CONFIGS["cfg1"].scaled(nheads=4, batch=3, rounds=24, snapshot_mode="defer", engine="vector"), None),
    "f32_k3": (Workload("df32", "scalar", batch=4, nheads=2, headdim=48, dstate=16, k=3, rounds=30, io="f32", accept="uniform",
                        ngroups=2, seed=35, snapshot_mode="defer"), None),
    "cfg2_k5": (CONFIGS["cfg2"].scaled(nheads=1000, batch=2, k=5, rounds=20, snapshot_mode="defer"), None),
}


@FUSED
@pytest.mark.parametrize("case", sorted(DEFER_CASES))
def test_deferred_advance_variant(case, fused):
    """SSMV_SNAP_DEFER: h_k is never stored and h_j only by a verify that meets pend > 16 - 2 kmax; until then the
    accepted tokens collect in the window ring behind the live slot.  Outputs, logical state and the integer model's
    bookkeeping must match the eager oracle on both engines; the schedules are long enough to reach the rounds that
    store, and for the ring to wrap."""
    wl, ks = DEFER_CASES[case]
    data = generate(wl, k_schedule=ks)
    run_parity(wl, data, fused=fused, reverify=True)
    bk = oracle.BookkeepingModel(wl.batch, wl.ring_len, wl.conv_width, mode="defer", kmax=wl.kmax_eff)
    moved, top = 0, 0
    for i, rd in enumerate(data.rounds):
        bk.verify(rd.x_raw.shape[1])
        before = list(bk.cur)
        bk.commit(rd.accepted)
        moved += sum(a != b for a, b in zip(before, bk.cur))
        top = max(top, max(bk.pend))
    if "none" not in case:
        assert moved > 0, "the schedule never reached a round that stores h_j"
        assert top > wl.kmax_eff or 2 * wl.kmax_eff == 16, "the window never held more than one round"


def test_deferred_advance_stores_a_state_only_when_the_window_fills():
    """Slot writes of SSMV_SNAP_DEFER on the matrix-core engine: the h_k slot is never written, the h_j slot exactly
    in the rounds that meet pend > 16 - 2 kmax, and then it holds the state at pos + pend."""
    wl = CONFIGS["cfg1"].scaled(nheads=2, batch=4, rounds=30, snapshot_mode="defer")
    data = generate(wl)
    hip = HipLayer(wl, data.layers[0])
    assert ssmv.ssmv_engine_of(hip.dims) == 1
    pend_hi = ssmv.SSMV_WINDOW - 2 * wl.kmax_eff
    stored = 0
    for rd in data.rounds:
        ints = hip.cache.ints()
        cur = torch.from_numpy(ints["cur_slot"]).long()
        pend = ints["pend"]
        seqs = torch.arange(wl.batch)
        hip.cache.state_view()[(cur + 1) % 3, seqs] = 123.0       # sentinels in both non-live slots
        hip.cache.state_view()[(cur + 2) % 3, seqs] = 321.0
        want_hj = hip.materialize()                                # state at pos + pend, before the round
        dx, ddt, dB, dC = (to_dev(v, wl.io) for v in (rd.x_raw, rd.dt[0], rd.B[0], rd.C[0]))
        hip.conv_verify(dx, ddt, dB, dC)
        sv = hip.cache.state_view()
        for b in range(wl.batch):
            c = int(cur[b])
            assert torch.all(sv[(c + 2) % 3, b] == 321.0)
            if pend[b] > pend_hi:
                stored += 1
                assert rel_err(to_host(untile_state(sv[(c + 1) % 3, b])), to_host(want_hj[b])) <= 1e-4
            else:
                assert torch.all(sv[(c + 1) % 3, b] == 123.0)
        hip.commit(torch.from_numpy(rd.accepted).to("cuda"))
    assert stored > 0
    ssmv.ssmv_check(hip.cache.c)


def test_single_snapshot_never_writes_the_third_slot():
    wl = CONFIGS["cfg1"].scaled(nheads=2, batch=2, rounds=6, snapshot_mode="hj_only")
    data = generate(wl)
    hip = HipLayer(wl, data.layers[0])
    hip.cache.state_view()[1:].fill_(123.0)                # slots 1, 2: sentinel
    untouched = None
    for rd in data.rounds:
        ints = hip.cache.ints()
        cur = torch.from_numpy(ints["cur_slot"]).long()
        third = (cur + 2) % 3
        before = hip.cache.state_view()[third, torch.arange(wl.batch)].clone()
        dx, ddt, dB, dC = (to_dev(v, wl.io) for v in (rd.x_raw, rd.dt[0], rd.B[0], rd.C[0]))
        hip.conv_verify(dx, ddt, dB, dC)
        after = hip.cache.state_view()[third, torch.arange(wl.batch)]
        assert torch.equal(before, after)
        hip.commit(torch.from_numpy(rd.accepted).to("cuda"))


def test_fused_launch_equals_the_two_separate_launches_bit_for_bit():
    """Same fp32 order and rounding in both paths: y, the stash, the ring and the snapshots must be identical."""
    for wl in (CONFIGS["cfg1"].scaled(nheads=3, batch=2, rounds=6, conv_act="silu"),
               CONFIGS["cfg2"].scaled(nheads=512, batch=2, rounds=6)):
        data = generate(wl)
        lp = data.layers[0]
        a, bb = HipLayer(wl, lp), HipLayer(wl, lp)
        for rd in data.rounds:
            dx, ddt, dB, dC = (to_dev(v, wl.io) for v in (rd.x_raw, rd.dt[0], rd.B[0], rd.C[0]))
            xc = a.conv(dx)
            y1 = a.verify(xc, ddt, dB, dC)
            y2, xc2 = bb.conv_verify(dx, ddt, dB, dC)
            assert torch.equal(y1, y2) and torch.equal(xc, xc2)
            acc = torch.from_numpy(rd.accepted).to("cuda")
            a.commit(acc)
            bb.commit(acc)
            for name in ("state", "conv_ring", "win_dt0", "win_dt1", "win_B0", "win_B1"):
                assert torch.equal(a.cache.buffers[name], bb.cache.buffers[name]), name


@pytest.mark.parametrize("snap", ["both", "hj_only", "defer"])
def test_commit_multi_matches_single_commits(snap):
    wl = Workload("cm", "scalar", batch=5, nheads=1, headdim=16, dstate=16, k=3, rounds=6 if snap != "defer" else 18, io="f32",
                  accept="uniform", seed=17, snapshot_mode=snap)
    data = generate(wl)
    lp = data.layers[0]
    n_layers = 40                                        # more than one launch covers
    multi = [HipLayer(wl, lp) for _ in range(n_layers)]
    single = HipLayer(wl, lp)
    for rd in data.rounds:
        dx, ddt, dB, dC = (to_dev(v, wl.io) for v in (rd.x_raw, rd.dt[0], rd.B[0], rd.C[0]))
        for layer in multi + [single]:
            layer.conv_verify(dx, ddt, dB, dC)
        acc = torch.from_numpy(rd.accepted).to("cuda")
        ssmv.ssm_commit_rollback_multi(single.dims, [m.cache.c for m in multi], acc)
        single.commit(acc)
        ref = single.cache.ints()
        for m in multi:
            got = m.cache.ints()
            for name in ("cur_slot", "pend", "pos", "conv_head", "last_k"):
                assert np.array_equal(got[name], ref[name]), name
            assert got["win_par"] == ref["win_par"] and got["err_flag"] == 0


def test_multistep_equals_single_steps_on_gpu():
    """I1 on the device: one k-token verify + full accept == k single-token rounds (same kernels, tolerance)."""
    wl = Workload("i1", "scalar", batch=2, nheads=2, headdim=64, dstate=64, k=4, rounds=1, io="f32",
                  accept="all", seed=13)
    data = generate(wl)
    rd, lp = data.rounds[0], data.layers[0]
    big, one = HipLayer(wl, lp), HipLayer(wl, lp)
    dx, ddt, dB, dC = (to_dev(a, wl.io) for a in (rd.x_raw, rd.dt[0], rd.B[0], rd.C[0]))
    y = big.verify(big.conv(dx), ddt, dB, dC)
    big.commit(torch.full((wl.batch,), wl.k, dtype=torch.int32, device="cuda"))
    ones = torch.ones(wl.batch, dtype=torch.int32, device="cuda")
    for t in range(wl.k):
        sl = slice(t, t + 1)
        yt = one.verify(one.conv(dx[:, sl].contiguous()), ddt[:, sl].contiguous(), dB[:, sl].contiguous(), dC[:, sl].contiguous())
        one.commit(ones)
        assert rel_err(to_host(yt[:, 0]), to_host(y[:, t])) <= 1e-5
    assert rel_err(to_host(one.materialize()), to_host(big.materialize())) <= 1e-5


def test_materialize_and_verify_do_not_mutate_the_cache():
    wl = Workload("mut", "scalar", batch=2, nheads=2, headdim=64, dstate=64, k=4, rounds=2, io="f32",
                  accept="uniform", seed=14)
    data = generate(wl)
    data.rounds[0].accepted[:] = [2, 1]                       # leave tokens pending
    lp = data.layers[0]
    hip = HipLayer(wl, lp)
    r0, r1 = data.rounds
    xc = hip.conv(to_dev(r0.x_raw, wl.io))
    hip.verify(xc, to_dev(r0.dt[0], wl.io), to_dev(r0.B[0], wl.io), to_dev(r0.C[0], wl.io))
    hip.commit(torch.from_numpy(r0.accepted).to("cuda"))
    ints0 = hip.cache.ints()
    live0 = hip.cache.state_view()[torch.from_numpy(ints0["cur_slot"]).long(), torch.arange(wl.batch)].clone()
    h_a = hip.materialize()
    xc = hip.conv(to_dev(r1.x_raw, wl.io))
    hip.verify(xc, to_dev(r1.dt[0], wl.io), to_dev(r1.B[0], wl.io), to_dev(r1.C[0], wl.io))
    h_b = hip.materialize()
    ints1 = hip.cache.ints()
    live1 = hip.cache.state_view()[torch.from_numpy(ints1["cur_slot"]).long(), torch.arange(wl.batch)]
    assert torch.equal(h_a, h_b) and torch.equal(live0, live1)
    for name in ("cur_slot", "pend", "pos", "conv_head"):
        assert np.array_equal(ints0[name], ints1[name])
    assert ints1["last_k"].tolist() == [wl.k] * wl.batch and ints1["win_par"] == ints0["win_par"]


def test_device_error_flag_paths():
    wl = Workload("err", "scalar", batch=3, nheads=1, headdim=16, dstate=16, k=3, rounds=1, io="f32",
                  accept="uniform", seed=15)
    data = generate(wl)
    lp, rd = data.layers[0], data.rounds[0]
    hip = HipLayer(wl, lp)
    # commit without verify: nothing changes, sticky flag
    hip.commit(torch.zeros(wl.batch, dtype=torch.int32, device="cuda"))
    with pytest.raises(ssmv.SsmvError) as ei:
        ssmv.ssmv_check(hip.cache.c)
    assert ei.value.code == ssmv.SSMV_ESEQUENCE
    ints = hip.cache.ints()
    assert ints["win_par"] == 0 and ints["cur_slot"].tolist() == [0, 0, 0] and ints["pos"].tolist() == [0, 0, 0]
    # out-of-range accepted: clamped exactly like the integer model, sticky flag
    hip.reset()
    ssmv.ssmv_check(hip.cache.c)
    xc = hip.conv(to_dev(rd.x_raw, wl.io))
    hip.verify(xc, to_dev(rd.dt[0], wl.io), to_dev(rd.B[0], wl.io), to_dev(rd.C[0], wl.io))
    bad = np.array([7, -2, 1], dtype=np.int32)
    hip.commit(torch.from_numpy(bad).to("cuda"))
    bk = oracle.BookkeepingModel(wl.batch, wl.ring_len, wl.conv_width, mode=wl.snapshot_mode, kmax=wl.kmax_eff)
    bk.verify(wl.k)
    bk.commit(bad)
    ints = hip.cache.ints()
    assert ints["cur_slot"].tolist() == bk.cur and ints["pend"].tolist() == bk.pend and ints["pos"].tolist() == bk.pos
    assert ints["conv_head"].tolist() == bk.conv_head and ints["err_flag"] == bk.err == 1


def test_commit_is_per_sequence_when_some_have_no_verify_pending():
    """The 'no verify pending' rule per sequence, against the integer model: last_k is cleared by hand for some
    sequences after a verify, then one commit covers all of them."""
    wl = Workload("mix", "scalar", batch=4, nheads=1, headdim=16, dstate=16, k=3, rounds=1, io="f32", accept="uniform", seed=17)
    data = generate(wl)
    lp, rd = data.layers[0], data.rounds[0]
    for mask in ([1, 0, 1, 0], [0, 1, 1, 1], [0, 0, 0, 0]):
        hip = HipLayer(wl, lp)
        xc = hip.conv(to_dev(rd.x_raw, wl.io))
        hip.verify(xc, to_dev(rd.dt[0], wl.io), to_dev(rd.B[0], wl.io), to_dev(rd.C[0], wl.io))
        lk = hip.cache.buffers["last_k"].view(torch.int32)
        lk[:wl.batch] = lk[:wl.batch] * torch.tensor(mask, dtype=torch.int32, device="cuda")
        acc = np.array([3, 1, 2, 0], dtype=np.int32)
        hip.commit(torch.from_numpy(acc).to("cuda"))
        bk = oracle.BookkeepingModel(wl.batch, wl.ring_len, wl.conv_width, mode=wl.snapshot_mode, kmax=wl.kmax_eff)
        bk.verify(wl.k)
        bk.last_k = [wl.k * m for m in mask]
        bk.commit(acc)
        ints = hip.cache.ints()
        assert ints["cur_slot"].tolist() == bk.cur and ints["pend"].tolist() == bk.pend and ints["pos"].tolist() == bk.pos
        assert ints["conv_head"].tolist() == bk.conv_head and ints["last_k"].tolist() == bk.last_k
        assert ints["win_par"] == bk.win_par and ints["err_flag"] == bk.err == 1


def test_first_conflict_bit_exact():
    rng = np.random.default_rng(16)
    for batch, k in [(1, 1), (7, 4), (300, 8), (1025, 16)]:
        draft = rng.integers(0, 3, size=(batch, k)).astype(np.int32)
        target = rng.integers(0, 3, size=(batch, k)).astype(np.int32)
        target[: batch // 3] = draft[: batch // 3]                      # some full matches
        out = torch.empty(batch, dtype=torch.int32, device="cuda")
        ssmv.ssmv_first_conflict(torch.from_numpy(draft).to("cuda"), torch.from_numpy(target).to("cuda"), batch, k, out)
        assert np.array_equal(out.cpu().numpy(), oracle.first_conflict(draft, target))


def test_copy_probe_copies():
    src = torch.randn(1 << 20, device="cuda")
    d0, d1 = torch.zeros_like(src), torch.zeros_like(src)
    ssmv.ssmv_copy_probe(src, d0, d1, src.numel() * 4)
    assert torch.equal(src, d0) and torch.equal(src, d1)
    d0.zero_()
    ssmv.ssmv_copy_probe(src, d0, None, src.numel() * 4)
    assert torch.equal(src, d0)
