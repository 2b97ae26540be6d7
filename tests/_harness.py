"""Shared helpers of the GPU parity tests: run a seeded workload through the HIP library (C ABI)
and through the fp64 oracle, round by round, and compare.

Error metrics (per tensor), both held to the same bound: the element-wise relative error
max_i |g_i - r_i| / max(|r_i|, rms(r)) (the rms floor keeps near-cancelled dot products from dividing
by ~0) and the tensor-wide max|g - r| / max|r|.  Bounds: 1e-5 for fp32 I/O, 2e-2 for bf16 I/O
with fp32 state.  Integers (slot, pending count, position, ring head, parity) must be equal.
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2408_15237_amd as ssmv
from workload import Workload, WorkloadData

TOL = {"f32": 1e-5, "bf16": 2e-2}
TORCH_IO = {"f32": torch.float32, "bf16": torch.bfloat16}


def rel_err(got, ref) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    floor = np.sqrt(np.mean(ref * ref))
    den = np.maximum(np.abs(ref), max(floor, 1e-30))
    return float(np.max(np.abs(got - ref) / den))


def max_err(got, ref) -> float:
    """max|g - r| / max|r| over the whole tensor."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    return float(np.max(np.abs(got - ref)) / max(float(np.max(np.abs(ref))), 1e-30))


def check_close(got, ref, tol: float, what: str):
    """Asserts both metrics; returns (element-wise floored error, tensor-wide error)."""
    e, m = rel_err(got, ref), max_err(got, ref)
    assert e <= tol and m <= tol, "%s: error %.3g (floored relative), %.3g (max|g-r|/max|r|) > %.3g" % (what, e, m, tol)
    return e, m


def to_dev(a, io: str):
    """float32 container holding io-representable values -> device tensor of the io type (exact)."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda").to(TORCH_IO[io]).contiguous()


def to_host(t) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def untile_state(t):
    """A (..., P, N) view of raw slot memory of the matrix-core engine -> the (..., P, N) state it stands for.  Inside a
    (sequence, head) block, tile (p/16, n/16) is 256 consecutive floats and the four floats n%16 in [4g, 4g+4) of row
    p%16 are the float4 number 16 g + p%16 of the tile."""
    lead, (P, N) = t.shape[:-2], t.shape[-2:]
    v = t.reshape(*lead, P // 16, N // 16, 4, 16, 4)          # tile row, tile column, g, p%16, n%4
    n = len(lead)
    return v.permute(*range(n), n, n + 3, n + 1, n + 2, n + 4).reshape(*lead, P, N)


def dims_of(wl: Workload):
    return ssmv.make_dims(wl.batch, wl.nheads, wl.headdim, wl.dstate, ngroups=wl.ngroups, kmax=wl.kmax_eff,
                          ring_len=wl.ring_len, io=wl.io, a_mode=wl.a_mode, conv_act=wl.conv_act,
                          snapshot_mode=wl.snapshot_mode, engine=wl.engine)


class HipLayer:
    """One layer of the HIP path: device parameters, its cache, and the three calls of a round."""

    def __init__(self, wl: Workload, lp, conv_init=None):
        self.wl = wl
        self.dims = dims_of(wl)
        self.cache = ssmv.LayerCache.allocate(self.dims)
        self.A = torch.from_numpy(lp.A).to("cuda").contiguous()
        self.D = torch.from_numpy(lp.D).to("cuda").contiguous()
        self.conv_w = to_dev(lp.conv_w, wl.io)
        self.conv_b = None if lp.conv_b is None else to_dev(lp.conv_b, wl.io)
        self.h0 = torch.from_numpy(lp.h0).to("cuda").contiguous()
        self.conv_init = None if conv_init is None else to_dev(conv_init, wl.io)
        self.reset()

    def reset(self):
        ssmv.ssmv_cache_reset(self.dims, self.cache.c, self.h0, self.conv_init)

    def conv(self, x_raw):
        k = x_raw.shape[1]
        xc = torch.empty_like(x_raw)
        ssmv.conv1d_state_update(self.dims, self.cache.c, x_raw, self.conv_w, self.conv_b, k, xc)
        return xc

    def verify(self, xc, dt, Bm, Cm):
        k = xc.shape[1]
        y = torch.empty_like(xc)
        ssmv.ssm_verify_multistep(self.dims, self.cache.c, xc, dt, Bm, Cm, self.A, self.D, k, y)
        return y

    def conv_verify(self, x_raw, dt, Bm, Cm):
        """conv roll + verification in one launch; returns (y, xc read back from the stash window)."""
        k = x_raw.shape[1]
        y = torch.empty_like(x_raw)
        ssmv.ssm_conv_verify_multistep(self.dims, self.cache.c, x_raw, self.conv_w, self.conv_b, dt, Bm, Cm, self.A, self.D, k, y)
        return y, self.stashed_xc(k)

    def stashed_xc(self, k):
        """This round's conv outputs as the verify kernel stashed them (the half that commit makes current)."""
        wl = self.wl
        ints = self.cache.ints()
        if wl.snapshot_mode == "defer":                   # one ring per sequence: token q of the sequence at entry q % 16
            Wn = ssmv.SSMV_WINDOW
            n = wl.batch * Wn * wl.conv_channels
            t = self.cache.buffers["win_xc0"].view(TORCH_IO[wl.io])[:n].view(wl.batch, Wn, wl.conv_channels)
            first = ints["pos"] + ints["pend"]
            idx = torch.from_numpy(np.stack([(int(first[b]) + np.arange(k)) % Wn for b in range(wl.batch)])).to("cuda")
            return torch.gather(t, 1, idx[:, :, None].expand(-1, -1, wl.conv_channels)).clone()
        par = ints["win_par"]
        buf = self.cache.buffers["win_xc%d" % (par ^ 1)]
        n = wl.batch * wl.kmax_eff * wl.conv_channels
        t = buf.view(TORCH_IO[wl.io])[:n].view(wl.batch, wl.kmax_eff, wl.conv_channels)
        return t[:, :k].clone()

    def commit(self, accepted_dev):
        ssmv.ssm_commit_rollback(self.dims, self.cache.c, accepted_dev)

    def materialize(self):
        wl = self.wl
        h = torch.empty((wl.batch, wl.nheads, wl.headdim, wl.dstate), dtype=torch.float32, device="cuda")
        ssmv.ssmv_materialize(self.dims, self.cache.c, self.A, h)
        return h


def eager_oracle(wl: Workload, lp, conv_init=None):
    return oracle.EagerOracle(wl.a_mode, lp.A, lp.D, lp.conv_w, lp.conv_b, lp.h0, wl.io, wl.conv_act, wl.ngroups,
                              conv_init=conv_init)


def run_parity(wl: Workload, data: WorkloadData, layer: int = 0, x_override=None, check_state_every: int = 1,
               conv_init=None, reverify: bool = False, fused: bool = False):
    """Full parity of one layer over all rounds of `data`.  Returns the worst errors seen."""
    lp = data.layers[layer]
    tol = TOL[wl.io]
    hip = HipLayer(wl, lp, conv_init=conv_init)
    ora = eager_oracle(wl, lp, conv_init=conv_init)
    bk = oracle.BookkeepingModel(wl.batch, wl.ring_len, wl.conv_width, mode=wl.snapshot_mode, kmax=wl.kmax_eff)
    worst = {"y": 0.0, "xc": 0.0, "h": 0.0, "y_max": 0.0, "h_max": 0.0}
    for i, rd in enumerate(data.rounds):
        x_raw = rd.x_raw if x_override is None else x_override[i]
        k = x_raw.shape[1]
        y_ref, xc_ref, _ = ora.verify(x_raw, rd.dt[layer], rd.B[layer], rd.C[layer])
        d_x, d_dt = to_dev(x_raw, wl.io), to_dev(rd.dt[layer], wl.io)
        d_B, d_C = to_dev(rd.B[layer], wl.io), to_dev(rd.C[layer], wl.io)
        if fused:
            y, xc = hip.conv_verify(d_x, d_dt, d_B, d_C)
            if reverify:
                y2, xc2 = hip.conv_verify(d_x, d_dt, d_B, d_C)
                assert torch.equal(y, y2) and torch.equal(xc, xc2), "fused verify is not idempotent (round %d)" % i
        else:
            xc = hip.conv(d_x)
            y = hip.verify(xc, d_dt, d_B, d_C)
            if reverify:                                   # verify twice: must be idempotent
                y2 = hip.verify(xc, d_dt, d_B, d_C)
                assert torch.equal(y, y2), "verify is not idempotent (round %d)" % i
        bk.verify(k)
        e_xc, _ = check_close(to_host(xc), xc_ref, tol, "round %d: conv output" % i)
        e_y, m_y = check_close(to_host(y), y_ref, tol, "round %d: y" % i)
        worst["y_max"] = max(worst["y_max"], m_y)
        acc = rd.accepted
        hip.commit(torch.from_numpy(acc.astype(np.int32)).to("cuda"))
        ora.commit(acc)
        bk.commit(acc)
        ints = hip.cache.ints()
        assert ints["cur_slot"].tolist() == bk.cur, "round %d: cur_slot" % i
        assert ints["pend"].tolist() == bk.pend, "round %d: pend" % i
        assert ints["pos"].tolist() == bk.pos, "round %d: pos" % i
        assert ints["conv_head"].tolist() == bk.conv_head, "round %d: conv_head" % i
        assert ints["last_k"].tolist() == bk.last_k, "round %d: last_k" % i
        assert ints["win_par"] == bk.win_par and ints["err_flag"] == bk.err == 0, "round %d: parity/err" % i
        if check_state_every and (i % check_state_every == 0 or i == len(data.rounds) - 1):
            e_h, m_h = check_close(to_host(hip.materialize()), ora.h, tol, "round %d: state" % i)
            worst["h"], worst["h_max"] = max(worst["h"], e_h), max(worst["h_max"], m_h)
        worst["y"], worst["xc"] = max(worst["y"], e_y), max(worst["xc"], e_xc)
    ssmv.ssmv_check(hip.cache.c)
    return worst
