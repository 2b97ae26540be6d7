"""Python face of the fp64 CPU oracle (TEST INFRASTRUCTURE ONLY).

Three pieces, all independent of the HIP path:

* ``EagerOracle``  - the definition: keeps the true state after the accepted
  tokens and the full list of committed raw conv inputs; ``verify`` runs the
  recurrence token by token (C, fp64) keeping every intermediate state,
  ``commit`` indexes the one after the accepted prefix (Section 4.2,
  MultiStep and Algorithm 2 of arXiv 2408.15237, read eagerly).
* ``BookkeepingModel`` - pure-integer model of the cache bookkeeping that
  Algorithm 2's "return h_k if k'=k else h_j" and the lazily advanced single
  cached state imply, for a three-slot state cache and a ping-pong window of
  pending tokens.
* ``LazyMirror`` - an fp64 mirror of that lazy three-slot policy (snapshot
  h_j / h_k, replay of accepted-but-unfolded tokens, conv ring with a moving
  head), used on the CPU only to show that the lazy policy is observationally
  the eager oracle.
"""
from __future__ import annotations

import ctypes
from typing import List, Optional

import numpy as np

from .build import build as _build

F32, BF16 = 0, 1
A_SCALAR, A_DIAG = 0, 1
ACT_NONE, ACT_SILU = 0, 1

_IO = {"f32": F32, "bf16": BF16}
_MODE = {"scalar": A_SCALAR, "diag": A_DIAG}
_ACT = {"none": ACT_NONE, "silu": ACT_SILU}

_lib = None
_dp = ctypes.POINTER(ctypes.c_double)


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build())
        lib.ssmo_threads.restype = ctypes.c_int
        lib.ssmo_round_bf16.restype = ctypes.c_double
        lib.ssmo_round_bf16.argtypes = [ctypes.c_double]
        lib.ssmo_round_array.restype = None
        lib.ssmo_round_array.argtypes = [_dp, _dp, ctypes.c_size_t, ctypes.c_int]
        lib.ssmo_conv.restype = None
        lib.ssmo_conv.argtypes = [ctypes.c_int] * 4 + [_dp, _dp, _dp, ctypes.c_int, ctypes.c_int, _dp]
        lib.ssmo_scan.restype = None
        lib.ssmo_scan.argtypes = [ctypes.c_int] * 7 + [_dp] * 9
        _lib = lib
    return _lib


def _c(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_dp)


def oracle_threads() -> int:
    return int(_load().ssmo_threads())


def round_io(a, io: str) -> np.ndarray:
    """Round fp64 values to the I/O storage type (single rounding, ties to even)."""
    a = _c(a)
    out = np.empty_like(a)
    _load().ssmo_round_array(_p(a), _p(out), a.size, _IO[io])
    return out


def conv_causal(raw, wgt, bias, act: str, io: str) -> np.ndarray:
    """raw [batch][W-1+k][Cx] (history then new tokens) -> xc [batch][k][Cx]."""
    raw, wgt = _c(raw), _c(wgt)
    bias = None if bias is None else _c(bias)
    batch, L, Cx = raw.shape
    W = wgt.shape[1]
    assert wgt.shape[0] == Cx
    k = L - (W - 1)
    xc = np.empty((batch, k, Cx), dtype=np.float64)
    _load().ssmo_conv(batch, k, Cx, W, _p(raw), _p(wgt), _p(bias), _ACT[act], _IO[io], _p(xc))
    return xc


def scan_tokens(a_mode: str, h_in, x, dt, Bm, Cm, A, D):
    """Run k tokens from h_in.  Returns (y [batch][k][H*P], h_snap [k+1][batch][H][P][N])."""
    h_in, x, dt, Bm, Cm, A, D = map(_c, (h_in, x, dt, Bm, Cm, A, D))
    batch, H, P, N = h_in.shape
    k = x.shape[1]
    G = Bm.shape[2]
    assert x.shape == (batch, k, H * P) and dt.shape == (batch, k, H)
    assert Bm.shape == (batch, k, G, N) and Cm.shape == (batch, k, G, N)
    assert A.shape == ((H, N) if a_mode == "diag" else (H,)) and D.shape == (H,)
    assert H % G == 0
    y = np.empty((batch, k, H * P), dtype=np.float64)
    snap = np.empty((k + 1, batch, H, P, N), dtype=np.float64)
    _load().ssmo_scan(_MODE[a_mode], batch, H, P, N, G, k, _p(h_in), _p(x), _p(dt), _p(Bm), _p(Cm),
                      _p(A), _p(D), _p(y), _p(snap))
    return y, snap


def softplus(x) -> np.ndarray:
    """log(1 + exp(x)), the map from a raw step-size projection to the positive step dt of Section 2.2
    (evaluated as max(x,0) + log1p(exp(-|x|)) so that no exponential overflows)."""
    x = _c(x)
    return np.maximum(x, 0.0) + np.log1p(np.exp(-np.abs(x)))


def step_size(dt_raw, dt_bias=None, use_softplus: bool = False) -> np.ndarray:
    """dt = softplus(dt_raw + dt_bias) (bias broadcast over the last axis); identity pieces when not asked for."""
    dt = _c(dt_raw)
    if dt_bias is not None:
        dt = dt + _c(dt_bias)
    return softplus(dt) if use_softplus else dt


def silu_gate(y, z) -> np.ndarray:
    """y * z * sigmoid(z): the output gate of a Mamba block."""
    y, z = _c(y), _c(z)
    return y * z / (1.0 + np.exp(-z))


def rmsnorm_gated(y, z, weight, group_size: int, eps: float) -> np.ndarray:
    """The norm behind the recurrence in a Mamba-2 block: g = y * silu(z) (g = y when z is None); per row and per
    group of `group_size` adjacent channels out = g / sqrt(mean(g^2) + eps) * weight."""
    g = _c(y) if z is None else silu_gate(y, z)
    rows, ch = g.reshape(-1, g.shape[-1]).shape
    gg = g.reshape(rows, ch // group_size, group_size)
    ms = np.mean(gg * gg, axis=-1, keepdims=True)
    return (gg / np.sqrt(ms + eps)).reshape(g.shape) * _c(weight)


def first_conflict(draft, target) -> np.ndarray:
    """Length of the longest prefix on which draft and target agree (Algorithm 2, FirstConflict)."""
    draft = np.asarray(draft)
    target = np.asarray(target)
    out = np.zeros(draft.shape[0], dtype=np.int32)
    for b in range(draft.shape[0]):
        n = 0
        while n < draft.shape[1] and draft[b, n] == target[b, n]:
            n += 1
        out[b] = n
    return out


class EagerOracle:
    """O1: the plain definition.  No slots, no laziness, unbounded conv history."""

    def __init__(self, a_mode: str, A, D, conv_w, conv_b, h0, io: str, act: str = "none",
                 ngroups: int = 1, conv_init=None, dt_bias=None, dt_softplus: bool = False):
        self.a_mode, self.io, self.act, self.G = a_mode, io, act, ngroups
        self.dt_bias = None if dt_bias is None else _c(dt_bias)
        self.dt_softplus = dt_softplus
        self.A, self.D = _c(A), _c(D)
        self.conv_w = _c(conv_w)
        self.conv_b = None if conv_b is None else _c(conv_b)
        self.h = _c(h0).copy()
        self.batch, self.H, self.P, self.N = self.h.shape
        self.Cx, self.W = self.conv_w.shape
        assert self.Cx == self.H * self.P
        init = np.zeros((self.batch, self.W - 1, self.Cx)) if conv_init is None else _c(conv_init)
        assert init.shape == (self.batch, self.W - 1, self.Cx)
        self.hist: List[np.ndarray] = [init[b].copy() for b in range(self.batch)]
        self.j = np.zeros(self.batch, dtype=np.int64)
        self._last = None

    def verify(self, x_raw, dt, Bm, Cm, z=None):
        """Returns (y, xc, h_snap); h_snap[t] is the state after t of the new tokens.  With z, y is gated."""
        x_raw = _c(x_raw)
        dt = step_size(dt, self.dt_bias, self.dt_softplus)
        W = self.W
        raw = np.stack([np.concatenate([self.hist[b][-(W - 1):], x_raw[b]], axis=0)
                        for b in range(self.batch)])
        xc = conv_causal(raw, self.conv_w, self.conv_b, self.act, self.io)
        y, snap = scan_tokens(self.a_mode, self.h, xc, dt, Bm, Cm, self.A, self.D)
        if z is not None:
            y = silu_gate(y, z)
        self._last = (x_raw, snap)
        return y, xc, snap

    def commit(self, accepted) -> None:
        x_raw, snap = self._last
        k = x_raw.shape[1]
        for b in range(self.batch):
            a = int(accepted[b])
            assert 0 <= a <= k
            self.h[b] = snap[a, b]
            self.hist[b] = np.concatenate([self.hist[b], x_raw[b, :a]], axis=0)
            self.j[b] += a
        self._last = None


class BookkeepingModel:
    """O2: integer model of the lazy cache.

    Per sequence: ``cur`` (live slot of 3), ``pend`` (accepted tokens not yet
    folded into the live slot), ``pos`` (tokens folded), ``conv_head`` (ring index
    of the newest committed raw input), ``last_k`` (k of the un-committed verify).
    Global: ``win_par`` (which half of the pending-token window is current),
    ``err`` (sticky).  Verify writes h_j to slot (cur+1)%3 when pend>0 and h_k to
    slot (cur+2)%3 and touches no integer except last_k.

    mode "hj_only": the single-snapshot variant.  h_k is never stored; every accepted token stays pending,
    also after a fully accepted round, and is replayed by the next verify.
    mode "defer": h_k is never stored and h_j only when it has to be.  A verify can replay up to WINDOW - k
    tokens, so the live slot stays where it is, and the accepted tokens pile up behind it, for as long as the
    NEXT round is sure to fit: pend + a + kmax <= WINDOW for every a <= kmax, i.e. pend <= WINDOW - 2 kmax = pend_hi.
    Only a verify that meets pend > pend_hi stores h_j (the state after the pending tokens), and its commit moves
    the live slot there.  The pending tokens of a sequence sit in a ring of WINDOW entries, token q of the sequence
    (counted from its start) at entry q mod WINDOW.
    """

    WINDOW = 16

    def __init__(self, batch: int, ring_len: int, conv_width: int = 4, hj_only: bool = False, mode: str = None, kmax: int = 0):
        assert ring_len & (ring_len - 1) == 0
        self.batch, self.R = batch, ring_len
        self.mode = mode if mode is not None else ("hj_only" if hj_only else "both")
        assert self.mode in ("both", "hj_only", "defer")
        self.hj_only = self.mode == "hj_only"
        self.defer = self.mode == "defer"
        self.pend_hi = 0
        if self.defer:
            assert 1 <= kmax and 2 * kmax <= self.WINDOW, "defer mode: the window must hold two rounds"
            self.pend_hi = self.WINDOW - 2 * kmax
        self.cur = [0] * batch
        self.pend = [0] * batch
        self.pos = [0] * batch
        self.conv_head = [conv_width - 2] * batch
        self.last_k = [0] * batch
        self.win_par = 0
        self.err = 0

    def verify(self, k: int, tok0: int = 0) -> None:
        """tok0 > 0: a later call of a round that several calls feed (draft side); the round then holds tok0+k tokens."""
        self.last_k = [tok0 + k] * self.batch

    def commit(self, accepted) -> None:
        """Per sequence: one with no verify pending (last_k == 0) is left as it is and the sticky error is set.
        The window parity is one value for the whole batch; it follows sequence 0."""
        flip = self.last_k[0] != 0
        for b in range(self.batch):
            lk = self.last_k[b]
            if lk == 0:
                self.err = 1      # commit without a verify: nothing to commit for this sequence
                continue
            a = int(accepted[b])
            if a < 0 or a > lk:
                self.err = 1
                a = min(max(a, 0), lk)
            if self.defer:
                if self.pend[b] > self.pend_hi:       # this round's verify stored h_j: move there
                    self.cur[b] = (self.cur[b] + 1) % 3
                    self.pos[b] += self.pend[b]
                    self.pend[b] = a
                else:                                 # the live slot stays; the window grows
                    self.pend[b] += a
            elif a == lk and not self.hj_only:
                self.cur[b] = (self.cur[b] + 2) % 3
                self.pos[b] += self.pend[b] + a
                self.pend[b] = 0
            elif self.pend[b] > 0:
                self.cur[b] = (self.cur[b] + 1) % 3
                self.pos[b] += self.pend[b]
                self.pend[b] = a
            else:
                self.pend[b] = a
            self.conv_head[b] = (self.conv_head[b] + a) & (self.R - 1)
            self.last_k[b] = 0
        if flip:
            self.win_par ^= 1


class LazyMirror:
    """O3: fp64 mirror of the lazy three-slot policy (CPU only; proves lazy == eager)."""

    def __init__(self, a_mode: str, A, D, conv_w, conv_b, h0, io: str, kmax: int, ring_len: int,
                 act: str = "none", ngroups: int = 1, conv_init=None, hj_only: bool = False, mode: str = None):
        self.a_mode, self.io, self.act, self.G = a_mode, io, act, ngroups
        self.A, self.D = _c(A), _c(D)
        self.conv_w = _c(conv_w)
        self.conv_b = None if conv_b is None else _c(conv_b)
        h0 = _c(h0)
        self.batch, self.H, self.P, self.N = h0.shape
        self.Cx, self.W = self.conv_w.shape
        self.kmax, self.R = kmax, ring_len
        assert ring_len >= self.W - 1 + kmax
        self.slots = np.zeros((3,) + h0.shape)
        self.slots[0] = h0
        self.ring = np.zeros((self.batch, ring_len, self.Cx))
        if conv_init is not None:
            self.ring[:, : self.W - 1] = _c(conv_init)
        self.bk = BookkeepingModel(self.batch, ring_len, self.W, hj_only=hj_only, mode=mode, kmax=kmax)
        self.hj_only, self.defer = self.bk.hj_only, self.bk.defer
        # both / hj_only: two halves of kmax entries (pending tokens in half win_par, the round's in the other);
        # defer: one ring of WINDOW entries per sequence (kept as "half 0"), token q of the sequence at entry q mod WINDOW
        went = self.bk.WINDOW if self.defer else kmax
        self.win_xc = np.zeros((2, self.batch, went, self.Cx))
        self.win_dt = np.zeros((2, self.batch, went, self.H))
        self.win_B = np.zeros((2, self.batch, went, ngroups, self.N))

    def _entries(self, b: int, first: int, count: int, of_round: bool):
        """(half, entry indices) of `count` window tokens of sequence b: the pending ones from `first` on, or, with
        of_round, the ones the current round has been fed from its token `first` on."""
        bk = self.bk
        if self.defer:
            base = bk.pos[b] + (bk.pend[b] if of_round else 0) + first
            return 0, [(base + i) % bk.WINDOW for i in range(count)]
        return (bk.win_par ^ 1 if of_round else bk.win_par), list(range(first, first + count))

    def _scan_window(self, b: int, g: np.ndarray, count: int, of_round: bool) -> np.ndarray:
        """g advanced over `count` window tokens (no outputs)."""
        if count == 0:
            return g
        half, idx = self._entries(b, 0, count, of_round)
        zeros_c = np.zeros((1, count, self.G, self.N))
        _, snap = scan_tokens(self.a_mode, g[None], self.win_xc[half, b][idx][None], self.win_dt[half, b][idx][None],
                              self.win_B[half, b][idx][None], zeros_c, self.A, self.D)
        return snap[count, 0]

    def _replayed(self, b: int) -> np.ndarray:
        """State of sequence b at pos+pend: live slot with the pending tokens folded in."""
        bk = self.bk
        return self._scan_window(b, self.slots[bk.cur[b], b], bk.pend[b], of_round=False)

    def verify(self, x_raw, dt, Bm, Cm, tok0: int = 0, replay_round: bool = False, last_call: bool = False):
        """tok0 > 0: a later call of a round that several calls feed (the draft side of Section 4.3 produces its
        tokens one call at a time).  By default it continues from the state the earlier calls left in the h_k slot,
        advances that slot in place, replays nothing, and appends its tokens to the round's stash and ring behind the
        tok0 earlier ones.  With replay_round every call of the round instead starts from the live slot and recomputes:
        the pending tokens, then the round's tok0 earlier tokens out of the round's stash, then its own; no slot is
        written before the call that says last_call, which writes h_j and h_k as one call with all tokens would."""
        x_raw, dt, Bm, Cm = map(_c, (x_raw, dt, Bm, Cm))
        assert not last_call or replay_round
        bk, W, R = self.bk, self.W, self.R
        k = x_raw.shape[1]
        assert 1 <= k and 0 <= tok0 and tok0 + k <= self.kmax
        assert tok0 == 0 or replay_round or not (self.hj_only or self.defer)
        raw = np.empty((self.batch, W - 1 + k, self.Cx))
        for b in range(self.batch):
            head = (bk.conv_head[b] + tok0) & (R - 1)  # newest raw input fed so far
            for t in range(k):                        # append after the head; old committed entries stay
                self.ring[b, (head + 1 + t) & (R - 1)] = x_raw[b, t]
            for i in range(W - 1 + k):                # oldest needed entry is head-(W-2)
                raw[b, i] = self.ring[b, (head - (W - 2) + i) & (R - 1)]
        xc = conv_causal(raw, self.conv_w, self.conv_b, self.act, self.io)
        y = np.empty((self.batch, k, self.Cx))
        for b in range(self.batch):
            cur = bk.cur[b]
            stores = not replay_round or last_call
            if tok0 == 0 or replay_round:
                g = self._replayed(b)
                if bk.pend[b] > bk.pend_hi and stores:               # (pend_hi = 0 unless the advance is deferred)
                    self.slots[(cur + 1) % 3, b] = g                 # snapshot h_j
                if replay_round and tok0 > 0:                        # the round's earlier tokens, again, no outputs
                    g = self._scan_window(b, g, tok0, of_round=True)
            else:
                g = self.slots[(cur + 2) % 3, b]                     # where the earlier calls of the round stopped
            yb, snap = scan_tokens(self.a_mode, g[None], xc[b:b + 1], dt[b:b + 1], Bm[b:b + 1], Cm[b:b + 1],
                                   self.A, self.D)
            y[b] = yb[0]
            if not (self.hj_only or self.defer) and stores:
                self.slots[(cur + 2) % 3, b] = snap[k, 0]            # snapshot h_k
        for b in range(self.batch):
            half, idx = self._entries(b, tok0, k, of_round=True)
            self.win_xc[half, b, idx] = xc[b]
            self.win_dt[half, b, idx] = dt[b]
            self.win_B[half, b, idx] = Bm[b]
        bk.verify(k, tok0)
        return y, xc

    def commit(self, accepted) -> None:
        self.bk.commit(accepted)

    def materialize(self) -> np.ndarray:
        return np.stack([self._replayed(b) for b in range(self.batch)])
