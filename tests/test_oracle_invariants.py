"""Invariants of the oracle's verify/commit protocol and of the lazy cache policy (CPU only).

Section 4.2 of arXiv 2408.15237 (MultiStep, Algorithm 2):
  I1  multistep over k tokens equals k single steps,
  I2  multistep from a cached state equals the matching slice of one full scan
      over exactly the accepted tokens,
  I3  rollback (partial accept) then re-verify of the same remaining tokens
      reproduces the first verify's outputs and final state,
  O3==O1  the lazy three-slot cache (snapshot h_j / h_k, replay of pending
      tokens, conv ring) is observationally the eager definition,
  and the integer bookkeeping obeys its invariants on every acceptance sequence.
"""
import itertools

import numpy as np
import pytest
import torch

import oracle
from workload import Workload, generate

TINY = Workload("tiny", "scalar", batch=2, nheads=4, headdim=3, dstate=5, k=4, rounds=10, io="f32",
                accept="uniform", ngroups=2, seed=3)
TINY_DIAG = Workload("tinyd", "diag", batch=2, nheads=6, headdim=1, dstate=4, k=5, rounds=10, io="bf16",
                     accept="geometric", conv_act="silu", seed=4)


def _eager(wl, data, layer=0):
    lp = data.layers[layer]
    return oracle.EagerOracle(wl.a_mode, lp.A, lp.D, lp.conv_w, lp.conv_b, lp.h0, wl.io, wl.conv_act, wl.ngroups)


def _lazy(wl, data, layer=0):
    lp = data.layers[layer]
    return oracle.LazyMirror(wl.a_mode, lp.A, lp.D, lp.conv_w, lp.conv_b, lp.h0, wl.io, wl.kmax_eff, wl.ring_len,
                             wl.conv_act, wl.ngroups, mode=wl.snapshot_mode)


def _pend_limit(bk, k):
    """Largest pend the integer model may show after a commit."""
    return bk.WINDOW - k if bk.defer else (k if bk.hj_only else k - 1)


@pytest.mark.parametrize("wl", [TINY, TINY_DIAG], ids=lambda w: w.name)
def test_I1_multistep_equals_single_steps(wl):
    data = generate(wl, rounds=1)
    rd = data.rounds[0]
    big = _eager(wl, data)
    y, xc, snap = big.verify(rd.x_raw, rd.dt[0], rd.B[0], rd.C[0])
    one = _eager(wl, data)
    ones = np.ones(wl.batch, dtype=np.int32)
    for t in range(wl.k):
        y1, xc1, _ = one.verify(rd.x_raw[:, t:t + 1], rd.dt[0][:, t:t + 1], rd.B[0][:, t:t + 1], rd.C[0][:, t:t + 1])
        one.commit(ones)
        assert np.array_equal(y1[:, 0], y[:, t])
        assert np.array_equal(xc1[:, 0], xc[:, t])
        assert np.array_equal(one.h, snap[t + 1])


@pytest.mark.parametrize("wl", [TINY, TINY_DIAG], ids=lambda w: w.name)
def test_I2_schedule_equals_full_scan_of_accepted_tokens(wl):
    """Re-drafting after a rejection: every round feeds fresh tokens; the committed stream is the accepted ones."""
    data = generate(wl)
    lp = data.layers[0]
    eager = _eager(wl, data)
    acc_x = [[] for _ in range(wl.batch)]
    acc_dt = [[] for _ in range(wl.batch)]
    acc_B = [[] for _ in range(wl.batch)]
    acc_C = [[] for _ in range(wl.batch)]
    acc_y = [[] for _ in range(wl.batch)]
    for rd in data.rounds:
        y, _, _ = eager.verify(rd.x_raw, rd.dt[0], rd.B[0], rd.C[0])
        for b in range(wl.batch):
            a = int(rd.accepted[b])
            acc_x[b].append(rd.x_raw[b, :a]); acc_dt[b].append(rd.dt[0][b, :a])
            acc_B[b].append(rd.B[0][b, :a]); acc_C[b].append(rd.C[0][b, :a]); acc_y[b].append(y[b, :a])
        eager.commit(rd.accepted)
    W, Cx = wl.conv_width, wl.conv_channels
    for b in range(wl.batch):
        xs = np.concatenate(acc_x[b]); dts = np.concatenate(acc_dt[b])
        Bs = np.concatenate(acc_B[b]); Cs = np.concatenate(acc_C[b]); ys = np.concatenate(acc_y[b])
        L = xs.shape[0]
        assert L == eager.j[b] and L > 0
        # one pass: library conv over the whole accepted stream, then one scan from h0
        want_conv = torch.nn.functional.conv1d(
            torch.from_numpy(xs.astype(np.float64)).T[None], torch.from_numpy(lp.conv_w.astype(np.float64))[:, None, :],
            None if lp.conv_b is None else torch.from_numpy(lp.conv_b.astype(np.float64)), padding=W - 1, groups=Cx)[0, :, :L].T
        if wl.conv_act == "silu":
            want_conv = torch.nn.functional.silu(want_conv)
        raw = np.concatenate([np.zeros((1, W - 1, Cx)), xs[None]], axis=1)
        xc_full = oracle.conv_causal(raw, lp.conv_w, lp.conv_b, wl.conv_act, wl.io)
        tol = 1e-2 if wl.io == "bf16" else 3e-7
        assert np.allclose(xc_full[0], want_conv.numpy(), rtol=tol, atol=tol)
        y_full, snap = oracle.scan_tokens(wl.a_mode, lp.h0[b:b + 1], xc_full, dts[None], Bs[None], Cs[None], lp.A, lp.D)
        assert np.array_equal(y_full[0], ys)
        assert np.array_equal(snap[L, 0], eager.h[b])


@pytest.mark.parametrize("wl", [TINY, TINY_DIAG], ids=lambda w: w.name)
def test_I3_rollback_then_reverify_reproduces(wl):
    data = generate(wl, rounds=2)
    r0, r1 = data.rounds
    eager = _eager(wl, data)
    eager.verify(r0.x_raw, r0.dt[0], r0.B[0], r0.C[0])
    eager.commit(np.full(wl.batch, wl.k, dtype=np.int32))          # warm the conv history
    y, _, snap = eager.verify(r1.x_raw, r1.dt[0], r1.B[0], r1.C[0])
    for a in range(wl.k):
        e2 = _eager(wl, data)
        e2.verify(r0.x_raw, r0.dt[0], r0.B[0], r0.C[0]); e2.commit(np.full(wl.batch, wl.k, dtype=np.int32))
        e2.verify(r1.x_raw, r1.dt[0], r1.B[0], r1.C[0]); e2.commit(np.full(wl.batch, a, dtype=np.int32))
        assert np.array_equal(e2.h, snap[a])
        y2, _, snap2 = e2.verify(r1.x_raw[:, a:], r1.dt[0][:, a:], r1.B[0][:, a:], r1.C[0][:, a:])
        assert np.array_equal(y2, y[:, a:])
        assert np.array_equal(snap2[-1], snap[-1])


def _run_both(wl, data, accepted_per_round, ks=None):
    eager, lazy = _eager(wl, data), _lazy(wl, data)
    total = np.zeros(wl.batch, dtype=np.int64)
    for i, rd in enumerate(data.rounds):
        k = rd.x_raw.shape[1]
        ye, xce, _ = eager.verify(rd.x_raw, rd.dt[0], rd.B[0], rd.C[0])
        yl, xcl = lazy.verify(rd.x_raw, rd.dt[0], rd.B[0], rd.C[0])
        assert np.array_equal(xce, xcl)
        assert np.allclose(ye, yl, rtol=1e-12, atol=1e-13)
        # verify is idempotent and leaves the bookkeeping alone
        yl2, _ = lazy.verify(rd.x_raw, rd.dt[0], rd.B[0], rd.C[0])
        assert np.array_equal(yl, yl2)
        acc = np.asarray(accepted_per_round[i])
        eager.commit(acc); lazy.commit(acc)
        total += acc
        bk = lazy.bk
        assert np.allclose(lazy.materialize(), eager.h, rtol=1e-12, atol=1e-13)
        for b in range(wl.batch):
            assert bk.pos[b] + bk.pend[b] == total[b] == eager.j[b]
            assert bk.cur[b] in (0, 1, 2) and 0 <= bk.pend[b] <= _pend_limit(bk, wl.kmax_eff)
            assert bk.conv_head[b] == (wl.conv_width - 2 + total[b]) % wl.ring_len
            assert bk.last_k[b] == 0
        assert bk.win_par == (i + 1) % 2 and bk.err == 0
    return eager, lazy


TINY_HJ = TINY.scaled(name="tiny_hj", snapshot_mode="hj_only")
TINY_DIAG_HJ = TINY_DIAG.scaled(name="tinyd_hj", snapshot_mode="hj_only")
TINY_DEFER = TINY.scaled(name="tiny_defer", snapshot_mode="defer", rounds=24)
TINY_DIAG_DEFER = TINY_DIAG.scaled(name="tinyd_defer", snapshot_mode="defer", rounds=24)


@pytest.mark.parametrize("wl", [TINY, TINY_DIAG, TINY_HJ, TINY_DIAG_HJ, TINY_DEFER, TINY_DIAG_DEFER], ids=lambda w: w.name)
def test_lazy_policy_equals_eager_on_random_schedule(wl):
    data = generate(wl)
    _run_both(wl, data, [rd.accepted for rd in data.rounds])


@pytest.mark.parametrize("snap", ["both", "hj_only", "defer"])
def test_lazy_policy_with_varying_k_and_kmax(snap):
    wl = TINY.scaled(kmax=6, rounds=12, seed=9, snapshot_mode=snap)
    ks = [1, 6, 3, 6, 2, 5, 1, 1, 6, 4, 2, 6]
    data = generate(wl, k_schedule=ks)
    rng = np.random.default_rng(1)
    acc = [rng.integers(0, k + 1, size=wl.batch) for k in ks]
    _run_both(wl, data, acc)


@pytest.mark.parametrize("snap", ["both", "hj_only", "defer"])
def test_lazy_policy_all_accept_and_all_reject_streaks(snap):
    wl = TINY.scaled(rounds=9, snapshot_mode=snap)
    data = generate(wl)
    k = wl.k
    acc = [[k, k], [k, k], [0, 0], [0, 0], [k, 0], [0, k], [k - 1, 1], [k, k], [0, 0]]
    _run_both(wl, data, acc)


@pytest.mark.parametrize("snap", ["both", "hj_only", "defer"])
def test_bruteforce_every_acceptance_sequence(snap):
    """All (k+1)^rounds acceptance sequences for k<=3 over 4 rounds: lazy state == eager state, ints consistent."""
    for k in (1, 2, 3):
        wl = Workload("bf", "scalar", batch=1, nheads=2, headdim=2, dstate=3, k=k, rounds=4, io="f32",
                      accept="uniform", seed=20 + k, snapshot_mode=snap)
        data = generate(wl)
        for seq in itertools.product(range(k + 1), repeat=wl.rounds):
            _run_both(wl, data, [[a] for a in seq])


def test_bruteforce_deferred_advance_through_the_advance_round():
    """Deferred advance with kmax = 7 and 6 (pend_hi = 2 and 4): four and five rounds reach the rounds that store h_j and
    move the live slot, for every acceptance sequence; the window ring (16 entries) wraps on the way."""
    for k, rounds in ((7, 4), (6, 4)):
        wl = Workload("bfd", "scalar", batch=1, nheads=2, headdim=2, dstate=3, k=k, rounds=rounds, io="f32",
                      accept="uniform", seed=40 + k, snapshot_mode="defer")
        data = generate(wl)
        moved = 0
        for seq in itertools.product(range(k + 1), repeat=wl.rounds):
            _, lazy = _run_both(wl, data, [[a] for a in seq])
            moved += lazy.bk.cur[0] != 0
        assert moved > 0


def test_bookkeeping_slot_semantics_bruteforce():
    """Track, per slot, which token position its content stands for; the live slot must always stand for `pos`."""
    R = 8
    for k in (1, 2, 3):
        for seq in itertools.product(range(k + 1), repeat=5):
            bk = oracle.BookkeepingModel(1, R, 4)
            slot_pos = {0: 0}
            total = 0
            for a in seq:
                cur, pend, pos = bk.cur[0], bk.pend[0], bk.pos[0]
                bk.verify(k)
                if pend > 0:
                    slot_pos[(cur + 1) % 3] = pos + pend          # h_j written
                slot_pos[(cur + 2) % 3] = pos + pend + k          # h_k written
                assert (cur + 2) % 3 != cur and (cur + 1) % 3 != cur   # the source slot is never overwritten
                bk.commit([a])
                total += a
                assert slot_pos[bk.cur[0]] == bk.pos[0]
                assert bk.pos[0] + bk.pend[0] == total
                assert 0 <= bk.pend[0] < k
                assert bk.conv_head[0] == (2 + total) % R


def test_bookkeeping_slot_semantics_bruteforce_single_snapshot():
    """Single-snapshot variant: only h_j is ever written; the live slot must still stand for `pos`."""
    R = 8
    for k in (1, 2, 3):
        for seq in itertools.product(range(k + 1), repeat=5):
            bk = oracle.BookkeepingModel(1, R, 4, hj_only=True)
            slot_pos = {0: 0}
            total = 0
            for a in seq:
                cur, pend, pos = bk.cur[0], bk.pend[0], bk.pos[0]
                bk.verify(k)
                if pend > 0:
                    slot_pos[(cur + 1) % 3] = pos + pend          # h_j written, nothing else
                bk.commit([a])
                total += a
                assert slot_pos[bk.cur[0]] == bk.pos[0]
                assert bk.pos[0] + bk.pend[0] == total and 0 <= bk.pend[0] <= k
                assert bk.conv_head[0] == (2 + total) % R


def test_bookkeeping_slot_semantics_bruteforce_deferred_advance():
    """Deferred advance: h_j is written only by a verify that meets pend > pend_hi, and only then does the commit move
    the live slot; the live slot must always stand for `pos`, a verify must never need more than WINDOW tokens, and no
    window entry that is still pending may be overwritten by the round's own tokens."""
    R = 16
    for kmax, rounds in ((8, 4), (5, 6), (4, 7), (3, 7)):
        for seq in itertools.product(range(kmax + 1), repeat=rounds):
            bk = oracle.BookkeepingModel(1, R, 4, mode="defer", kmax=kmax)
            Wn = bk.WINDOW
            assert bk.pend_hi == Wn - 2 * kmax
            slot_pos = {0: 0}
            total = 0
            owner = {}                                            # window entry -> token index it holds
            for a in seq:
                cur, pend, pos = bk.cur[0], bk.pend[0], bk.pos[0]
                assert pend + kmax <= Wn                          # the verify fits the window
                for i in range(pend):                             # every pending token is still in its entry
                    assert owner[(pos + i) % Wn] == pos + i
                bk.verify(kmax)
                for t in range(kmax):                             # the round's tokens behind the pending ones
                    e = (pos + pend + t) % Wn
                    assert not (e in owner and pos <= owner[e] < pos + pend)
                    owner[e] = pos + pend + t
                if pend > bk.pend_hi:
                    slot_pos[(cur + 1) % 3] = pos + pend          # h_j written, nothing else
                bk.commit([a])
                total += a
                assert slot_pos[bk.cur[0]] == bk.pos[0]
                assert (bk.cur[0] != cur) == (pend > bk.pend_hi)
                assert bk.pos[0] + bk.pend[0] == total and 0 <= bk.pend[0] <= Wn - kmax
                assert bk.conv_head[0] == (2 + total) % R


def test_deferred_advance_with_the_smallest_window_is_the_single_snapshot_rule():
    """kmax = 8: pend_hi = 0, so h_j is stored whenever anything is pending - the single-snapshot integer rule."""
    rng = np.random.default_rng(5)
    a_bk = oracle.BookkeepingModel(3, 16, 4, mode="defer", kmax=8)
    b_bk = oracle.BookkeepingModel(3, 16, 4, hj_only=True)
    for _ in range(200):
        k = int(rng.integers(1, 9))
        acc = rng.integers(0, k + 1, size=3)
        a_bk.verify(k); b_bk.verify(k)
        a_bk.commit(acc); b_bk.commit(acc)
        for name in ("cur", "pend", "pos", "conv_head", "last_k", "win_par", "err"):
            assert getattr(a_bk, name) == getattr(b_bk, name), name


def test_bookkeeping_error_paths():
    bk = oracle.BookkeepingModel(2, 8, 4)
    bk.commit([0, 0])                               # commit without verify: no-op, sticky error
    assert bk.err == 1 and bk.win_par == 0 and bk.cur == [0, 0]
    bk = oracle.BookkeepingModel(2, 8, 4)
    bk.verify(3)
    bk.commit([7, -2])                              # out of range: clamped to [0, k], sticky error
    assert bk.err == 1 and bk.pend == [0, 0] and bk.pos == [3, 0] and bk.cur == [2, 0]
    assert bk.conv_head == [(2 + 3) % 8, 2]


@pytest.mark.parametrize("wl", [TINY, TINY_DIAG], ids=lambda w: w.name)
def test_I2_from_a_given_conv_history(wl):
    """Section 4.3 footnote: the conv part of the cache is the last W-1 raw inputs, oldest first.  A schedule started
    from a random history must equal ONE library convolution over (history ++ accepted stream), whose first outputs
    see the history in that order; a reversed or shifted history fails this."""
    data = generate(wl)
    lp = data.layers[0]
    W, Cx = wl.conv_width, wl.conv_channels
    rng = np.random.default_rng(77)
    init = oracle.round_io(rng.standard_normal((wl.batch, W - 1, Cx)), wl.io)
    eager = oracle.EagerOracle(wl.a_mode, lp.A, lp.D, lp.conv_w, lp.conv_b, lp.h0, wl.io, wl.conv_act, wl.ngroups, conv_init=init)
    lazy = oracle.LazyMirror(wl.a_mode, lp.A, lp.D, lp.conv_w, lp.conv_b, lp.h0, wl.io, wl.kmax_eff, wl.ring_len,
                             wl.conv_act, wl.ngroups, conv_init=init)
    got_xc = [[] for _ in range(wl.batch)]
    acc_x = [[] for _ in range(wl.batch)]
    for rd in data.rounds:
        _, xc, _ = eager.verify(rd.x_raw, rd.dt[0], rd.B[0], rd.C[0])
        yl, xcl = lazy.verify(rd.x_raw, rd.dt[0], rd.B[0], rd.C[0])
        assert np.array_equal(xc, xcl)
        for b in range(wl.batch):
            a = int(rd.accepted[b])
            got_xc[b].append(xc[b, :a]); acc_x[b].append(rd.x_raw[b, :a])
        eager.commit(rd.accepted); lazy.commit(rd.accepted)
        assert np.allclose(lazy.materialize(), eager.h, rtol=1e-12, atol=1e-13)
    for b in range(wl.batch):
        xs = np.concatenate([init[b]] + acc_x[b])                       # oldest first, then the accepted stream
        L = xs.shape[0] - (W - 1)
        assert L > 0
        want = torch.nn.functional.conv1d(
            torch.from_numpy(xs).T[None], torch.from_numpy(lp.conv_w.astype(np.float64))[:, None, :],
            None if lp.conv_b is None else torch.from_numpy(lp.conv_b.astype(np.float64)), groups=Cx)[0].T
        assert want.shape[0] == L
        if wl.conv_act == "silu":
            want = torch.nn.functional.silu(want)
        tol = 1e-2 if wl.io == "bf16" else 3e-7
        assert np.allclose(np.concatenate(got_xc[b]), want.numpy(), rtol=tol, atol=tol)
    # the history matters and its order matters: the first outputs change when it is reversed
    rd = data.rounds[0]
    e_rev = oracle.EagerOracle(wl.a_mode, lp.A, lp.D, lp.conv_w, lp.conv_b, lp.h0, wl.io, wl.conv_act, wl.ngroups,
                               conv_init=init[:, ::-1])
    e_fwd = oracle.EagerOracle(wl.a_mode, lp.A, lp.D, lp.conv_w, lp.conv_b, lp.h0, wl.io, wl.conv_act, wl.ngroups, conv_init=init)
    assert not np.allclose(e_rev.verify(rd.x_raw, rd.dt[0], rd.B[0], rd.C[0])[1][:, 0], e_fwd.verify(rd.x_raw, rd.dt[0], rd.B[0], rd.C[0])[1][:, 0])


def _compositions(n):
    """All ways to write n as an ordered sum of positive integers."""
    if n == 0:
        yield ()
        return
    for first in range(1, n + 1):
        for rest in _compositions(n - first):
            yield (first,) + rest


@pytest.mark.parametrize("replay", [False, True], ids=["carry", "replay"])
@pytest.mark.parametrize("wl", [TINY, TINY_DIAG.scaled(k=4), TINY_HJ, TINY_DEFER], ids=lambda w: w.name)
def test_round_fed_by_several_calls_equals_one_call(wl, replay):
    """Section 4.3, draft side: a round whose k tokens arrive over several calls leaves the cache exactly where one
    k-token call would, for every way of splitting k <= 4, over rounds with ragged acceptance in between - whether the
    calls carry the state through the h_k slot or every call recomputes from the live slot (replay_round)."""
    if wl.snapshot_mode != "both" and not replay:
        pytest.skip("carrying the state needs the h_k slot")
    data = generate(wl.scaled(rounds=8 if wl.snapshot_mode == "defer" else 4))
    lp = data.layers[0]
    mk = lambda: oracle.LazyMirror(wl.a_mode, lp.A, lp.D, lp.conv_w, lp.conv_b, lp.h0, wl.io, wl.kmax_eff, wl.ring_len,
                                   wl.conv_act, wl.ngroups, mode=wl.snapshot_mode)
    for split in _compositions(wl.k):
        one, many = mk(), mk()
        eager = _eager(wl, data)
        for rd in data.rounds:
            y1, xc1 = one.verify(rd.x_raw, rd.dt[0], rd.B[0], rd.C[0])
            ye, _, _ = eager.verify(rd.x_raw, rd.dt[0], rd.B[0], rd.C[0])
            t0, ys, xcs = 0, [], []
            slots_before = many.slots.copy()
            for ci, n in enumerate(split):
                s = slice(t0, t0 + n)
                last = ci == len(split) - 1
                y, xc = many.verify(rd.x_raw[:, s], rd.dt[0][:, s], rd.B[0][:, s], rd.C[0][:, s], tok0=t0,
                                    replay_round=replay, last_call=replay and last)
                if replay:                                    # idempotent, and no slot is touched before the last call
                    y2, _ = many.verify(rd.x_raw[:, s], rd.dt[0][:, s], rd.B[0][:, s], rd.C[0][:, s], tok0=t0,
                                        replay_round=True, last_call=last)
                    assert np.array_equal(y, y2)
                    assert last or np.array_equal(many.slots, slots_before)
                ys.append(y); xcs.append(xc)
                t0 += n
                assert many.bk.last_k == [t0] * wl.batch
            assert np.array_equal(np.concatenate(xcs, axis=1), xc1)
            assert np.allclose(np.concatenate(ys, axis=1), y1, rtol=1e-13, atol=1e-14)
            assert np.allclose(y1, ye, rtol=1e-12, atol=1e-13)
            assert np.array_equal(many.ring, one.ring) and np.array_equal(many.win_xc, one.win_xc)
            assert np.array_equal(many.win_dt, one.win_dt) and np.array_equal(many.win_B, one.win_B)
            assert np.allclose(many.slots, one.slots, rtol=1e-13, atol=1e-14)
            for m in (one, many):
                m.commit(rd.accepted)
            eager.commit(rd.accepted)
            for name in ("cur", "pend", "pos", "conv_head", "last_k", "win_par", "err"):
                assert getattr(many.bk, name) == getattr(one.bk, name), name
            assert np.allclose(many.materialize(), eager.h, rtol=1e-12, atol=1e-13)


def test_commit_is_per_sequence_when_some_have_no_verify_pending():
    """A sequence whose last_k is 0 is left untouched and raises the sticky error; the others commit as usual; the
    batch-wide window parity follows sequence 0.  Every mix of (verified, not verified) over three sequences."""
    for mask in itertools.product((0, 1), repeat=3):
        for a in range(4):
            bk = oracle.BookkeepingModel(3, 8, 4)
            ref = oracle.BookkeepingModel(1, 8, 4)
            bk.verify(3)
            bk.last_k = [3 * m for m in mask]
            bk.commit([a, a, a])
            ref.verify(3); ref.commit([a])
            for b, m in enumerate(mask):
                if m:
                    assert (bk.cur[b], bk.pend[b], bk.pos[b], bk.conv_head[b]) == (ref.cur[0], ref.pend[0], ref.pos[0], ref.conv_head[0])
                else:
                    assert (bk.cur[b], bk.pend[b], bk.pos[b], bk.conv_head[b]) == (0, 0, 0, 2)
                assert bk.last_k[b] == 0
            assert bk.err == (0 if all(mask) else 1)
            assert bk.win_par == mask[0]
