"""Pins of the CPU oracle against things other than itself.

The paper (arXiv 2408.15237) prints no worked numeric example of the multi-step
kernel, so the oracle is pinned to what the mathematics fixes:
  * the closed form of the recurrence for a scalar (and, element-wise, a
    diagonal) A  (Section 2.1 Eq. 1 with A_bar = exp(Delta*A), B_bar = Delta*B),
  * the geometric series for constant inputs,
  * the linear-attention special case A=0, Delta=1 (Section 2.1: the RNN form of
    linearized attention; Section 2.2: "N'=1 and identity discretization"),
  * a brute-force evaluation of Eq. 1 with explicit diagonal matrices,
  * library routines: torch conv1d for the conv, torch's bf16 cast for rounding.
Every pin is also run against deliberately wrong variants of the recurrence
(planted on the CPU, in this file) to show that it would catch them.
"""
import numpy as np
import pytest
import torch

import oracle


def _draw(seed, batch=2, H=4, P=3, N=5, G=2, k=6, mode="scalar"):
    r = np.random.default_rng(seed)
    d = dict(
        h0=r.standard_normal((batch, H, P, N)) * 0.3,
        x=r.standard_normal((batch, k, H * P)),
        dt=np.logaddexp(0, r.standard_normal((batch, k, H)) - 1.0),
        B=r.standard_normal((batch, k, G, N)),
        C=r.standard_normal((batch, k, G, N)),
        A=-np.exp(r.uniform(0, np.log(16), size=(H, N) if mode == "diag" else (H,))),
        D=r.standard_normal(H),
    )
    return d


def _oracle_scan(mode, d):
    return oracle.scan_tokens(mode, d["h0"], d["x"], d["dt"], d["B"], d["C"], d["A"], d["D"])


# ---- deliberately wrong recurrences (python loops; tiny sizes only) -----------------------------
def _mutant_scan(kind):
    def scan(mode, d):
        h0, x, dt, Bm, Cm, A, D = (d[n] for n in ("h0", "x", "dt", "B", "C", "A", "D"))
        batch, H, P, N = h0.shape
        k, G = x.shape[1], Bm.shape[2]
        snap = np.zeros((k + 1,) + h0.shape)
        snap[0] = h0
        y = np.zeros((batch, k, H * P))
        for b in range(batch):
            for hd in range(H):
                g = hd * G // H
                if kind == "group_modulo":
                    g = hd % G
                for t in range(k):
                    for p in range(P):
                        xv = x[b, t, hd * P + p]
                        acc = 0.0
                        for n in range(N):
                            a = A[hd, n] if mode == "diag" else A[hd]
                            dec = np.exp(dt[b, t, hd] * a)
                            Bv, Cv = Bm[b, t, g, n], Cm[b, t, g, n]
                            if kind == "sign_A":
                                dec = np.exp(-dt[b, t, hd] * a)
                            if kind == "swap_BC":
                                Bv, Cv = Cv, Bv
                            inp = dt[b, t, hd] * Bv * xv
                            if kind == "no_dt_on_B":
                                inp = Bv * xv
                            hprev = snap[t, b, hd, p, n]
                            hn = dec * hprev + inp
                            if kind == "decay_input_too":
                                hn = dec * (hprev + inp)
                            snap[t + 1, b, hd, p, n] = hn
                            acc += Cv * (hprev if kind == "y_from_old_state" else hn)
                        y[b, t, hd * P + p] = acc + (0.0 if kind == "drop_D" else D[hd] * xv)
        return y, snap
    return scan


MUTANTS = ["sign_A", "swap_BC", "no_dt_on_B", "decay_input_too", "y_from_old_state", "drop_D", "group_modulo"]


# ---- pin 1: closed form -------------------------------------------------------------------------
def _closed_form(mode, d):
    h0, x, dt, Bm, Cm, A, D = (d[n] for n in ("h0", "x", "dt", "B", "C", "A", "D"))
    batch, H, P, N = h0.shape
    k, G = x.shape[1], Bm.shape[2]
    rep = H // G
    Bh = np.repeat(Bm, rep, axis=2)                      # [b,k,H,N]: head hd -> group hd // (H/G)
    Ch = np.repeat(Cm, rep, axis=2)
    xh = x.reshape(batch, k, H, P)
    Acoef = A[None, None, :, :] if mode == "diag" else A[None, None, :, None]   # [1,1,H,N|1]
    S = np.cumsum(dt, axis=1)                            # [b,k,H]
    ys, hs = [], []
    for T in range(k):
        # h_T = e^{A S_T} h0 + sum_{t<=T} e^{A (S_T - S_t)} dt_t x_t (x) B_t
        decay0 = np.exp(Acoef[:, 0] * S[:, T, :, None])                       # [b,H,N|1]
        hT = decay0[:, :, None, :] * h0
        w = np.exp(Acoef * (S[:, T:T + 1, :] - S[:, :T + 1, :])[..., None])   # [b,T+1,H,N|1]
        hT = hT + np.einsum("bthn,bthp->bhpn", w * dt[:, :T + 1, :, None] * Bh[:, :T + 1], xh[:, :T + 1])
        yT = np.einsum("bhn,bhpn->bhp", Ch[:, T], hT) + D[None, :, None] * xh[:, T]
        hs.append(hT)
        ys.append(yT.reshape(batch, H * P))
    return np.stack(ys, axis=1), np.stack([h0] + hs, axis=0)


def _agrees(got, want, rtol=1e-11):
    (y, s), (y2, s2) = got, want
    return bool(np.allclose(y, y2, rtol=rtol, atol=1e-12) and np.allclose(s, s2, rtol=rtol, atol=1e-12))


@pytest.mark.parametrize("mode", ["scalar", "diag"])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_closed_form(mode, seed):
    d = _draw(seed, mode=mode)
    assert _agrees(_oracle_scan(mode, d), _closed_form(mode, d))


@pytest.mark.parametrize("kind", MUTANTS)
def test_closed_form_catches_planted_mistakes(kind):
    d = _draw(3, mode="scalar")
    assert _agrees(_mutant_scan("none")("scalar", d), _closed_form("scalar", d))      # the harness itself is sound
    assert not _agrees(_mutant_scan(kind)("scalar", d), _closed_form("scalar", d))


# ---- pin 2: constant input -> geometric series ---------------------------------------------------
@pytest.mark.parametrize("mode", ["scalar", "diag"])
def test_constant_input_geometric_series(mode):
    batch, H, P, N, k = 1, 2, 2, 3, 40
    r = np.random.default_rng(5)
    delta = 0.07
    x1 = r.standard_normal(H * P)
    B1 = r.standard_normal((1, N))
    C1 = r.standard_normal((1, N))
    A = -np.exp(r.uniform(0, 2, size=(H, N) if mode == "diag" else (H,)))
    D = r.standard_normal(H)
    h0 = r.standard_normal((batch, H, P, N))
    d = dict(h0=h0, x=np.tile(x1, (batch, k, 1)), dt=np.full((batch, k, H), delta),
             B=np.tile(B1, (batch, k, 1, 1)), C=np.tile(C1, (batch, k, 1, 1)), A=A, D=D)
    y, snap = _oracle_scan(mode, d)
    a = np.exp(delta * (A if mode == "diag" else A[:, None]))           # [H,N|1]
    T = k
    drive = delta * B1[0][None, None, :] * x1.reshape(H, P)[:, :, None]  # [H,P,N]
    want = a[:, None, :] ** T * h0[0] + drive * (1 - a[:, None, :] ** T) / (1 - a[:, None, :])
    assert np.allclose(snap[T, 0], want, rtol=1e-10, atol=1e-13)
    y_want = np.einsum("n,hpn->hp", C1[0], want) + D[:, None] * x1.reshape(H, P)
    assert np.allclose(y[0, T - 1], y_want.reshape(-1), rtol=1e-10, atol=1e-13)


# ---- pin 3: linear attention special case -------------------------------------------------------
def _linear_attention(d):
    x, Bm, Cm = d["x"], d["B"], d["C"]
    batch, k, G, N = Bm.shape
    H = d["D"].shape[0]
    P = x.shape[2] // H
    out = np.zeros_like(x)
    for b in range(batch):
        for hd in range(H):
            g = hd * G // H
            scores = np.tril(Cm[b, :, g] @ Bm[b, :, g].T)               # [k,k], causal
            out[b, :, hd * P:(hd + 1) * P] = scores @ x[b, :, hd * P:(hd + 1) * P]
    return out


def _linatt_inputs(seed):
    d = _draw(seed, batch=2, H=4, P=3, N=5, G=2, k=7)
    d["A"] = np.zeros_like(d["A"])
    d["dt"] = np.ones_like(d["dt"])
    d["D"] = np.zeros_like(d["D"])
    d["h0"] = np.zeros_like(d["h0"])
    return d


def test_linear_attention_special_case():
    d = _linatt_inputs(7)
    y, _ = _oracle_scan("scalar", d)
    assert np.allclose(y, _linear_attention(d), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("kind", ["swap_BC", "y_from_old_state", "group_modulo"])
def test_linear_attention_catches_planted_mistakes(kind):
    d = _linatt_inputs(7)
    y, _ = _mutant_scan(kind)("scalar", d)
    assert not np.allclose(y, _linear_attention(d), rtol=1e-9, atol=1e-9)


# ---- pin 4: brute force of Eq. 1 with explicit matrices ------------------------------------------
@pytest.mark.parametrize("mode", ["scalar", "diag"])
def test_bruteforce_matrix_form(mode):
    d = _draw(11, batch=1, H=2, P=2, N=3, G=1, k=4, mode=mode)
    y, snap = _oracle_scan(mode, d)
    for hd in range(2):
        for p in range(2):
            h = d["h0"][0, hd, p].copy()                                  # state vector in R^N
            for t in range(4):
                dt = d["dt"][0, t, hd]
                a = d["A"][hd] if mode == "diag" else np.full(3, d["A"][hd])
                Abar = np.diag(np.exp(dt * a))                           # discrete A as a diagonal matrix
                Bbar = dt * d["B"][0, t, 0]
                xv = d["x"][0, t, hd * 2 + p]
                h = Abar @ h + Bbar * xv
                assert np.allclose(snap[t + 1, 0, hd, p], h, rtol=1e-12, atol=1e-14)
                assert np.isclose(y[0, t, hd * 2 + p], d["C"][0, t, 0] @ h + d["D"][hd] * xv, rtol=1e-12, atol=1e-14)


# ---- pin 5: conv against the library routine ----------------------------------------------------
@pytest.mark.parametrize("act", ["none", "silu"])
@pytest.mark.parametrize("use_bias", [True, False])
def test_conv_matches_torch_conv1d(act, use_bias):
    r = np.random.default_rng(13)
    batch, L, Cx, W = 2, 9, 6, 4
    seq = r.standard_normal((batch, L, Cx))
    wgt = r.standard_normal((Cx, W))
    bias = r.standard_normal(Cx) if use_bias else None
    raw = np.concatenate([np.zeros((batch, W - 1, Cx)), seq], axis=1)
    got = oracle.conv_causal(raw, wgt, bias, act, "f32")
    xt = torch.from_numpy(seq).permute(0, 2, 1)                           # [b,C,L]
    want = torch.nn.functional.conv1d(xt, torch.from_numpy(wgt)[:, None, :],
                                      None if bias is None else torch.from_numpy(bias),
                                      padding=W - 1, groups=Cx)[..., :L]
    if act == "silu":
        want = torch.nn.functional.silu(want)
    want = want.permute(0, 2, 1).to(torch.float32).to(torch.float64).numpy()
    assert np.allclose(got, want, rtol=3e-7, atol=1e-7)


def test_conv_tap_order_is_pinned():
    # one-hot weights: tap w of a width-4 causal conv selects the input 3-w steps back
    batch, Cx, W, k = 1, 1, 4, 5
    seq = np.arange(1.0, 1.0 + W - 1 + k).reshape(1, -1, 1)               # raw[i] = i+1
    for w in range(W):
        wgt = np.zeros((Cx, W))
        wgt[0, w] = 1.0
        got = oracle.conv_causal(seq, wgt, None, "none", "f32")[0, :, 0]
        assert np.array_equal(got, seq[0, w:w + k, 0])


# ---- pin 6: rounding against the library cast ----------------------------------------------------
def test_bf16_rounding_matches_torch_cast():
    r = np.random.default_rng(17)
    v = np.concatenate([
        r.standard_normal(20000).astype(np.float32),
        (r.standard_normal(2000) * 1e-30).astype(np.float32),
        (r.standard_normal(2000) * 1e30).astype(np.float32),
        np.float32([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -1.0 - 2.0 ** -8, 0.0, 2.0 ** -133, 2.0 ** -134,
                    3 * 2.0 ** -134, 1e-40, -1e-40, 3.38e38]),
    ])
    want = torch.from_numpy(v).to(torch.bfloat16).to(torch.float64).numpy()
    got = oracle.round_io(v.astype(np.float64), "bf16")
    assert np.array_equal(got, want)


def test_bf16_rounding_is_single_step():
    # 1 + 2^-8 + 2^-30 lies just above a tie: one rounding goes up; rounding via fp32 first would tie to even (down)
    x = 1.0 + 2.0 ** -8 + 2.0 ** -30
    assert oracle.round_io(np.array([x]), "bf16")[0] == 1.0 + 2.0 ** -7
    assert oracle.round_io(np.array([x]), "f32")[0] == np.float64(np.float32(x))


def test_first_conflict_examples():
    draft = np.array([[1, 2, 3, 4], [1, 2, 3, 4], [9, 2, 3, 4], [1, 2, 3, 4]])
    target = np.array([[1, 2, 3, 4], [1, 2, 7, 4], [1, 2, 3, 4], [1, 2, 3, 5]])
    assert oracle.first_conflict(draft, target).tolist() == [4, 2, 0, 3]


# ---- the pieces of a whole Mamba block around the recurrence: step-size transform and output gate ----

def test_softplus_closed_forms_and_library():
    """softplus(0) = ln 2; softplus(x) - softplus(-x) = x; softplus(x) -> x for large x and -> exp(x) for very
    negative x (no overflow on either side); and torch's softplus in fp64 as the library routine."""
    assert oracle.softplus(0.0) == pytest.approx(np.log(2.0), rel=1e-15)
    x = np.linspace(-30, 30, 241)
    np.testing.assert_allclose(oracle.softplus(x) - oracle.softplus(-x), x, rtol=0, atol=1e-13)
    assert oracle.softplus(800.0) == 800.0 and np.isfinite(oracle.softplus(-800.0))
    np.testing.assert_allclose(oracle.softplus(-40.0), np.exp(-40.0), rtol=1e-12)
    ref = torch.nn.functional.softplus(torch.from_numpy(x), beta=1.0, threshold=1e9).numpy()
    np.testing.assert_allclose(oracle.softplus(x), ref, rtol=1e-13)
    # planted mistakes: log(1+exp(x)) without the bias term / with the wrong sign
    assert not np.allclose(np.log1p(np.exp(-x)), ref)
    assert not np.allclose(np.maximum(x, 0) - np.log1p(np.exp(-np.abs(x))), ref)


def test_step_size_bias_is_added_before_the_softplus():
    r = np.random.default_rng(5)
    raw, bias = r.standard_normal((2, 3, 4)), r.standard_normal(4)
    got = oracle.step_size(raw, bias, True)
    ref = torch.nn.functional.softplus(torch.from_numpy(raw) + torch.from_numpy(bias), threshold=1e9).numpy()
    np.testing.assert_allclose(got, ref, rtol=1e-13)
    assert not np.allclose(oracle.softplus(raw) + bias, ref)                 # bias after the softplus: caught
    np.testing.assert_array_equal(oracle.step_size(raw), raw)                # nothing asked for: identity
    np.testing.assert_allclose(oracle.step_size(raw, bias), raw + bias, rtol=0, atol=0)


def test_silu_gate_library_and_limits():
    r = np.random.default_rng(6)
    y, z = r.standard_normal((3, 5, 8)), r.standard_normal((3, 5, 8)) * 3
    ref = (torch.from_numpy(y) * torch.nn.functional.silu(torch.from_numpy(z))).numpy()
    np.testing.assert_allclose(oracle.silu_gate(y, z), ref, rtol=1e-13, atol=1e-15)
    np.testing.assert_array_equal(oracle.silu_gate(y, np.zeros_like(z)), np.zeros_like(y))      # silu(0) = 0
    np.testing.assert_allclose(oracle.silu_gate(y, np.full_like(z, 50.0)), 50.0 * y, rtol=1e-12)  # silu(z) -> z
    assert not np.allclose(y / (1 + np.exp(-z)), ref)                        # sigmoid gate instead of SiLU: caught


def test_eager_oracle_block_pieces_compose_with_the_plain_scan():
    """EagerOracle with a step-size transform and a gate = the plain scan on the transformed dt, gated afterwards:
    the transform acts on dt only (not on x, B or the skip term) and the gate on y only (not on the state)."""
    d = _draw(11)
    r = np.random.default_rng(12)
    H, P = d["D"].shape[0], d["h0"].shape[2]
    conv_w = np.zeros((H * P, 4)); conv_w[:, 3] = 1.0                        # identity conv: xc = x
    bias = r.standard_normal(H) * 0.3
    raw = r.standard_normal(d["dt"].shape) - 1.0
    z = r.standard_normal(d["x"].shape)
    blk = oracle.EagerOracle("scalar", d["A"], d["D"], conv_w, None, d["h0"], "f32", dt_bias=bias, dt_softplus=True)
    y, _, snap = blk.verify(d["x"], raw, d["B"], d["C"], z=z)
    dt = np.logaddexp(0.0, raw + bias)                                       # softplus through another routine
    y_ref, snap_ref = oracle.scan_tokens("scalar", d["h0"], oracle.round_io(d["x"], "f32"), dt, d["B"], d["C"], d["A"], d["D"])
    np.testing.assert_allclose(snap, snap_ref, rtol=1e-12, atol=1e-14)       # the gate leaves the state alone
    np.testing.assert_allclose(y, y_ref * z / (1 + np.exp(-z)), rtol=1e-12, atol=1e-14)


# ---- hand-worked examples stored as text fixtures -------------------------------------------------------

def _read_fixture(name):
    import os
    out = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, val = line.split(":", 1)
        out[key.strip()] = [[float(v) for v in part.split()] for part in val.split("|")]
    return out


def test_hand_worked_examples():
    f = _read_fixture("recurrence_halving_decay.txt")
    k = len(f["dt"][0])
    A = np.array([f["A_over_ln2"][0][0] * np.log(2.0)])
    Bm = np.tile(np.array(f["B"][0]), (1, k, 1, 1))
    Cm = np.tile(np.array(f["C"][0]), (1, k, 1, 1))
    y, snap = oracle.scan_tokens("scalar", np.array(f["h0"][0]).reshape(1, 1, 1, 2), np.array(f["x"][0]).reshape(1, k, 1),
                                 np.array(f["dt"][0]).reshape(1, k, 1), Bm, Cm, A, np.array(f["D"][0]))
    np.testing.assert_allclose(y.reshape(-1), f["y"][0], rtol=1e-13)
    np.testing.assert_allclose(snap[1:].reshape(k, 2), np.array(f["h_after"]), rtol=1e-13)
    np.testing.assert_allclose(snap[0].reshape(-1), f["h0"][0], rtol=0)
    c = _read_fixture("conv_width4.txt")
    raw = np.array(c["history"][0] + c["x"][0]).reshape(1, -1, 1)
    xc = oracle.conv_causal(raw, np.array(c["taps"][0]).reshape(1, 4), np.array(c["bias"][0]), "none", "f32")
    np.testing.assert_allclose(xc.reshape(-1), c["xc"][0], rtol=0, atol=0)


def test_rmsnorm_gated_library_and_invariants():
    r = np.random.default_rng(8)
    y, z, w = r.standard_normal((3, 5, 64)), r.standard_normal((3, 5, 64)), r.standard_normal(64)
    # one group: torch's rms_norm on the gated values
    g = torch.from_numpy(y) * torch.nn.functional.silu(torch.from_numpy(z))
    ref = torch.nn.functional.rms_norm(g, (64,), torch.from_numpy(w), eps=1e-5).numpy()
    np.testing.assert_allclose(oracle.rmsnorm_gated(y, z, w, 64, 1e-5), ref, rtol=1e-12, atol=1e-14)
    # groups are normalised one by one
    ref4 = torch.nn.functional.rms_norm(g.reshape(3, 5, 4, 16), (16,), None, eps=1e-5).reshape(3, 5, 64).numpy() * w
    np.testing.assert_allclose(oracle.rmsnorm_gated(y, z, w, 16, 1e-5), ref4, rtol=1e-12, atol=1e-14)
    # without eps the output does not depend on the scale of y and has unit mean square per group (weight 1)
    out = oracle.rmsnorm_gated(y, None, np.ones(64), 16, 0.0)
    np.testing.assert_allclose(oracle.rmsnorm_gated(7.5 * y, None, np.ones(64), 16, 0.0), out, rtol=1e-12)
    np.testing.assert_allclose(np.mean(out.reshape(3, 5, 4, 16) ** 2, axis=-1), 1.0, rtol=1e-12)
    # planted mistakes: mean over the whole row instead of the group; variance (mean removed) instead of mean square
    assert not np.allclose(oracle.rmsnorm_gated(y, z, w, 64, 1e-5), ref4)
    gv = g.numpy().reshape(3, 5, 4, 16)
    assert not np.allclose((gv / np.sqrt(gv.var(axis=-1, keepdims=True) + 1e-5)).reshape(3, 5, 64) * w, ref4)
