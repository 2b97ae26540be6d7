"""GPU parity of the chunked prefill (ssm_prefill_chunked): the prompt goes through the oracle token by token
(EagerOracle.verify with k = L, then a commit of all L), through the GPU chunk by chunk on the matrix cores; then
both decode speculatively from what the prefill left (state, conv ring, integers)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2408_15237_amd as ssmv
from workload import Workload, generate

from _harness import HipLayer, TOL, eager_oracle, rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu

# (name, headdim, dstate, nheads, ngroups, batch, io, conv_act, L)
CASES = [
    ("p32n32_f32", 32, 32, 3, 1, 2, "f32", "none", 70),
    ("p64n64_bf16_groups", 64, 64, 4, 2, 3, "bf16", "silu", 200),
    ("p128n64_bf16", 128, 64, 2, 1, 2, "bf16", "none", 130),
    ("p64n128_f32", 64, 128, 2, 1, 1, "f32", "none", 97),
    ("one_chunk_exact", 32, 64, 2, 1, 2, "f32", "none", 32),
    ("one_past_a_chunk", 32, 64, 2, 1, 2, "f32", "none", 33),
    ("shorter_than_the_conv", 32, 32, 2, 1, 2, "f32", "none", 2),
    ("single_token", 64, 32, 2, 1, 2, "bf16", "none", 1),
    # bf16 tensors run on the bf16 matrix cores: every compiled tile shape, lengths that are no multiple of a chunk
    ("p32n32_bf16", 32, 32, 3, 1, 2, "bf16", "none", 70),
    ("p32n64_bf16", 32, 64, 2, 1, 2, "bf16", "silu", 45),
    ("p32n128_bf16", 32, 128, 2, 1, 2, "bf16", "none", 100),
    ("p64n32_bf16", 64, 32, 2, 1, 2, "bf16", "none", 77),
    ("p64n128_bf16", 64, 128, 2, 2, 2, "bf16", "none", 66),
    ("p128n32_bf16", 128, 32, 2, 1, 2, "bf16", "none", 40),
    ("p128n128_bf16", 128, 128, 2, 1, 1, "bf16", "none", 97),
]


# the same with the deferred advance: the prompt leaves pos = L, so the window ring starts at entry L % 16, and the decode
# runs long enough to reach the rounds that store a state (matrix-core engine, vector engine with bf16 and with fp32 tensors)
DEFER_CASES = [
    ("defer_p128n64_bf16", 128, 64, 2, 1, 3, "bf16", "none", 77, "defer", "auto"),
    ("defer_p64n32_bf16_groups", 64, 32, 4, 2, 3, "bf16", "silu", 45, "defer", "auto"),
    ("defer_p64n64_bf16_vector", 64, 64, 2, 1, 2, "bf16", "none", 50, "defer", "vector"),
    ("defer_p32n32_f32", 32, 32, 3, 1, 2, "f32", "none", 70, "defer", "auto"),
]


@pytest.mark.parametrize("case", CASES + DEFER_CASES, ids=[c[0] for c in CASES + DEFER_CASES])
def test_prefill_then_speculative_decoding(case):
    name, P, N, H, G, batch, io, act, L = case[:9]
    snap, engine = (case[9], case[10]) if len(case) > 9 else ("both", "auto")
    tol = TOL[io]
    dec = Workload(name, "scalar", batch=batch, nheads=H, headdim=P, dstate=N, k=4, rounds=6 if snap == "both" else 24, io=io,
                   accept="uniform", ngroups=G, conv_act=act, seed=31, snapshot_mode=snap, engine=engine)
    prompt = generate(dec.scaled(k=L, kmax=L, rounds=1, seed=32))       # only its draws are used: one "round" of L tokens
    data = generate(dec)
    lp = data.layers[0]
    rng = np.random.default_rng(33)
    conv_init = np.asarray(rng.standard_normal((batch, 3, H * P)), dtype=np.float32)
    from workload import round_to_io
    conv_init = round_to_io(conv_init, io)                               # a non-trivial history ahead of the prompt
    hip = HipLayer(dec, lp, conv_init=conv_init)
    ora = eager_oracle(dec, lp, conv_init=conv_init)
    pr = prompt.rounds[0]

    y_ref, _, _ = ora.verify(pr.x_raw, pr.dt[0], pr.B[0], pr.C[0])
    ora.commit(np.full(batch, L))
    d_x = to_dev(pr.x_raw, io)
    y = torch.empty_like(d_x)
    ints0 = hip.cache.ints()
    ssmv.ssm_prefill_chunked(hip.dims, hip.cache.c, d_x, hip.conv_w, hip.conv_b, to_dev(pr.dt[0], io), to_dev(pr.B[0], io),
                             to_dev(pr.C[0], io), hip.A, hip.D, L, y)
    e_y = rel_err(to_host(y), y_ref)
    assert e_y <= tol, "prompt outputs: %.3g > %.3g" % (e_y, tol)
    ints = hip.cache.ints()
    assert ints["pos"].tolist() == [L] * batch and ints["pend"].tolist() == [0] * batch
    assert ints["cur_slot"].tolist() == ints0["cur_slot"].tolist() and ints["last_k"].tolist() == [0] * batch
    assert ints["conv_head"].tolist() == [(int(c) + L) & (dec.ring_len - 1) for c in ints0["conv_head"]]
    assert ints["err_flag"] == 0
    e_h = rel_err(to_host(hip.materialize()), ora.h)
    assert e_h <= tol, "state after the prompt: %.3g" % e_h

    # decode from there: the ring must continue the prompt, the slots and integers must be consistent
    bk = oracle.BookkeepingModel(batch, dec.ring_len, dec.conv_width, mode=dec.snapshot_mode, kmax=dec.kmax_eff)
    bk.pos = [L] * batch
    bk.conv_head = ints["conv_head"].tolist()
    for i, rd in enumerate(data.rounds):
        y_r, _, _ = ora.verify(rd.x_raw, rd.dt[0], rd.B[0], rd.C[0])
        y_g, _ = hip.conv_verify(to_dev(rd.x_raw, io), to_dev(rd.dt[0], io), to_dev(rd.B[0], io), to_dev(rd.C[0], io))
        assert rel_err(to_host(y_g), y_r) <= tol, "decode round %d" % i
        hip.commit(torch.from_numpy(rd.accepted.astype(np.int32)).to("cuda"))
        ora.commit(rd.accepted)
        bk.verify(dec.k)
        bk.commit(rd.accepted)
        got = hip.cache.ints()
        assert got["cur_slot"].tolist() == bk.cur and got["pend"].tolist() == bk.pend and got["pos"].tolist() == bk.pos
        assert got["conv_head"].tolist() == bk.conv_head and got["err_flag"] == 0
    assert rel_err(to_host(hip.materialize()), ora.h) <= tol
    ssmv.ssmv_check(hip.cache.c)


@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_prefill_in_two_pieces_equals_one(io):
    """A prompt fed as two calls (the second continues from the state and ring the first left).  The chunk boundaries
    of the two runs differ, so the results agree to rounding: fp32 products for fp32 tensors, head + tail products
    (2^-17 per product) and bf16 outputs for bf16 tensors."""
    y_tol, h_tol = (1e-5, 1e-5) if io == "f32" else (TOL["bf16"], 1e-4)
    dec = Workload("two", "scalar", batch=2, nheads=2, headdim=64, dstate=64, k=4, rounds=1, io=io, accept="uniform", seed=41)
    L1, L2 = 45, 52
    prompt = generate(dec.scaled(k=L1 + L2, kmax=L1 + L2, rounds=1, seed=42))
    lp, pr = prompt.layers[0], prompt.rounds[0]
    one, two = HipLayer(dec, lp), HipLayer(dec, lp)
    dev = lambda a: to_dev(a, io)
    y1 = torch.empty_like(dev(pr.x_raw))
    ssmv.ssm_prefill_chunked(one.dims, one.cache.c, dev(pr.x_raw), one.conv_w, one.conv_b, dev(pr.dt[0]), dev(pr.B[0]), dev(pr.C[0]),
                             one.A, one.D, L1 + L2, y1)
    ys = []
    for sl in (slice(0, L1), slice(L1, L1 + L2)):
        n = sl.stop - sl.start
        y = torch.empty_like(dev(pr.x_raw[:, sl]))
        ssmv.ssm_prefill_chunked(two.dims, two.cache.c, dev(pr.x_raw[:, sl]), two.conv_w, two.conv_b, dev(pr.dt[0][:, sl]),
                                 dev(pr.B[0][:, sl]), dev(pr.C[0][:, sl]), two.A, two.D, n, y)
        ys.append(y)
    assert rel_err(to_host(torch.cat(ys, dim=1)), to_host(y1)) <= y_tol
    assert rel_err(to_host(two.materialize()), to_host(one.materialize())) <= h_tol
    a, b = one.cache.ints(), two.cache.ints()
    assert a["pos"].tolist() == b["pos"].tolist() == [L1 + L2] * 2 and a["conv_head"].tolist() == b["conv_head"].tolist()


def test_prefill_flags_a_cache_with_pending_tokens():
    dec = Workload("flag", "scalar", batch=2, nheads=2, headdim=32, dstate=32, k=4, rounds=1, io="f32", accept="uniform", seed=43)
    data = generate(dec)
    hip = HipLayer(dec, data.layers[0])
    rd = data.rounds[0]
    dev = lambda a: to_dev(a, "f32")
    hip.conv_verify(dev(rd.x_raw), dev(rd.dt[0]), dev(rd.B[0]), dev(rd.C[0]))
    hip.commit(torch.tensor([2, 0], dtype=torch.int32, device="cuda"))          # sequence 0 now has pending tokens
    y = torch.empty_like(dev(rd.x_raw))
    ssmv.ssm_prefill_chunked(hip.dims, hip.cache.c, dev(rd.x_raw), hip.conv_w, hip.conv_b, dev(rd.dt[0]), dev(rd.B[0]), dev(rd.C[0]),
                             hip.A, hip.D, 4, y)
    with pytest.raises(ssmv.SsmvError) as ei:
        ssmv.ssmv_check(hip.cache.c)
    assert ei.value.code == ssmv.SSMV_ESEQUENCE


def test_prefill_full_layer_shape_every_head_of_two_sequences():
    """The bench's launch shape (cfg3 layer: 32 heads x 128 x 64, bf16 I/O, 2048 prompt tokens) at batch 4; the oracle
    runs the token-by-token scan over every head of two sequences (eight heads at a time: it keeps every
    intermediate state)."""
    from workload import CONFIGS, round_to_io
    io = "bf16"
    L = 2048
    dec = CONFIGS["cfg3"].scaled(batch=4, rounds=1)
    lp = generate(dec).layers[0]
    rng = np.random.default_rng(51)
    B_, H, P, N = dec.batch, dec.nheads, dec.headdim, dec.dstate
    x = round_to_io(rng.standard_normal((B_, L, H * P), dtype=np.float32), io)
    dt = round_to_io(np.logaddexp(0, rng.standard_normal((B_, L, H), dtype=np.float32) - 4.0), io)
    Bm = round_to_io(rng.standard_normal((B_, L, 1, N), dtype=np.float32) / np.sqrt(N), io)
    Cm = round_to_io(rng.standard_normal((B_, L, 1, N), dtype=np.float32) / np.sqrt(N), io)
    hip = HipLayer(dec, lp)
    y = torch.empty((B_, L, H * P), dtype=torch.bfloat16, device="cuda")
    ssmv.ssm_prefill_chunked(hip.dims, hip.cache.c, to_dev(x, io), hip.conv_w, hip.conv_b, to_dev(dt, io), to_dev(Bm, io),
                             to_dev(Cm, io), hip.A, hip.D, L, y)
    y_h, h_g = to_host(y), to_host(hip.materialize())
    seqs = [0, 3]
    worst_y = worst_h = 0.0
    for h0_ in range(0, H, 8):
        heads = list(range(h0_, h0_ + 8))
        ch = np.concatenate([np.arange(h * P, (h + 1) * P) for h in heads])
        ora = oracle.EagerOracle("scalar", lp.A[heads], lp.D[heads], lp.conv_w[ch], lp.conv_b[ch], lp.h0[seqs][:, heads], io)
        y_ref, _, _ = ora.verify(x[seqs][:, :, ch], dt[seqs][:, :, heads], Bm[seqs], Cm[seqs])
        ora.commit(np.full(len(seqs), L))
        e_y, e_h = rel_err(y_h[seqs][:, :, ch], y_ref), rel_err(h_g[seqs][:, heads], ora.h)
        assert e_y <= TOL[io] and e_h <= TOL[io], "heads %d..%d: y %.3g, state %.3g" % (heads[0], heads[-1], e_y, e_h)
        worst_y, worst_h = max(worst_y, e_y), max(worst_h, e_h)
        del ora, y_ref
    print("prefill cfg3 shape, L=2048: y error %.3g, state error %.3g" % (worst_y, worst_h))
    assert hip.cache.ints()["pos"].tolist() == [L] * B_ and hip.cache.ints()["err_flag"] == 0


BLOCK_CASES = [
    ("bf16_p64", 64, 64, 3, 1, 3, "bf16", 150),
    ("f32", 32, 32, 2, 1, 2, "f32", 75),
    ("bf16_small_n", 128, 32, 2, 1, 2, "bf16", 90),
    ("bf16_p128", 128, 64, 2, 1, 3, "bf16", 130),
]


@pytest.mark.parametrize("case", BLOCK_CASES, ids=[c[0] for c in BLOCK_CASES])
def test_prefill_with_block_pieces_and_ragged_lengths(case):
    """softplus(dt + dt_bias), the SiLU gate and per-sequence prompt lengths.  Each sequence is its own oracle run of
    its own length (the oracle commits a whole batch with one k); outputs behind a sequence's length stay untouched."""
    from workload import round_to_io
    name, P, N, H, G, batch, io, L = case
    tol = TOL[io]
    dec = Workload(name, "scalar", batch=batch, nheads=H, headdim=P, dstate=N, k=4, rounds=3, io=io, accept="uniform", ngroups=G, seed=61)
    prompt = generate(dec.scaled(k=L, kmax=L, rounds=1, seed=62))
    data = generate(dec)
    lp, pr = data.layers[0], prompt.rounds[0]
    rng = np.random.default_rng(63)
    bias = rng.uniform(-0.5, 0.5, size=H).astype(np.float32)
    dt_raw = round_to_io(rng.standard_normal((batch, L, H)) - 4.0, io)
    z = round_to_io(rng.standard_normal((batch, L, H * P)), io)
    lens = np.array([L, 0, 37][:batch] if batch >= 3 else [L - 5, 1], dtype=np.int32)
    hip = HipLayer(dec, lp)
    d_bias = torch.from_numpy(bias).to("cuda")
    y = torch.full((batch, L, H * P), 7.0, dtype=torch.bfloat16 if io == "bf16" else torch.float32, device="cuda")
    ssmv.ssm_prefill_block(hip.dims, hip.cache.c, x_raw=to_dev(pr.x_raw, io), conv_wgt=hip.conv_w, conv_bias=hip.conv_b,
                           dt=to_dev(dt_raw, io), dt_bias=d_bias, dt_softplus=True, Bm=to_dev(pr.B[0], io), Cm=to_dev(pr.C[0], io),
                           z=to_dev(z, io), A=hip.A, D=hip.D, L=L, y_out=y, seq_len=torch.from_numpy(lens).to("cuda"))
    y_h = to_host(y)
    h_g = to_host(hip.materialize())
    oras = []
    for b in range(batch):
        n = int(lens[b])
        ora = oracle.EagerOracle("scalar", lp.A, lp.D, lp.conv_w, lp.conv_b, lp.h0[b:b + 1], io, dec.conv_act, G,
                                 dt_bias=bias, dt_softplus=True)
        if n > 0:
            y_ref, _, _ = ora.verify(pr.x_raw[b:b + 1, :n], dt_raw[b:b + 1, :n], pr.B[0][b:b + 1, :n], pr.C[0][b:b + 1, :n], z=z[b:b + 1, :n])
            ora.commit([n])
            assert rel_err(y_h[b, :n], y_ref[0]) <= tol, "sequence %d" % b
        assert np.all(y_h[b, n:] == 7.0), "sequence %d: outputs behind its length were written" % b
        assert rel_err(h_g[b:b + 1], ora.h) <= tol, "sequence %d: state" % b
        oras.append(ora)
    ints = hip.cache.ints()
    assert ints["pos"].tolist() == lens.tolist() and ints["err_flag"] == 0
    assert ints["conv_head"].tolist() == [(2 + int(n)) & (dec.ring_len - 1) for n in lens]
    # decode one round from there through the general call
    rd = data.rounds[0]
    ex_dt = round_to_io(rng.standard_normal((batch, dec.k, H)) - 4.0, io)
    y_g = torch.empty_like(to_dev(rd.x_raw, io))
    ssmv.ssm_block_multistep(hip.dims, hip.cache.c, x_raw=to_dev(rd.x_raw, io), conv_wgt=hip.conv_w, conv_bias=hip.conv_b,
                             dt=to_dev(ex_dt, io), dt_bias=d_bias, dt_softplus=True, Bm=to_dev(rd.B[0], io), Cm=to_dev(rd.C[0], io),
                             A=hip.A, D=hip.D, k=dec.k, y_out=y_g)
    for b in range(batch):
        y_r, _, _ = oras[b].verify(rd.x_raw[b:b + 1], ex_dt[b:b + 1], rd.B[0][b:b + 1], rd.C[0][b:b + 1])
        assert rel_err(to_host(y_g)[b:b + 1], y_r) <= tol, "decode after prefill, sequence %d" % b


@pytest.mark.parametrize("io", ["bf16", "f32"])
def test_prefill_strong_decay_and_accuracy_of_the_state(io):
    """Decay of up to e^-30 per token: factors inside a chunk underflow, and the masked upper triangle of the chunk's
    matrix would overflow if it were computed and multiplied instead of selected away.  Then a mild decay, where the state
    integrates hundreds of tokens: with bf16 tensors the matrix cores multiply bf16 numbers, and the state must still be
    stay far more accurate than one bf16 pass would leave it: an fp32 operand enters as bf16 head + bf16 tail, which drops
    2^-17 of it (8e-6 per product; the worst of 16 k state elements a few times that), against 2^-9 (2e-3) for the head
    alone.  The bound below sits between the two."""
    from workload import round_to_io
    for scale, L in ((60.0, 96), (0.2, 300)):
        dec = Workload("decay", "scalar", batch=2, nheads=2, headdim=128, dstate=64, k=4, rounds=1, io=io, accept="uniform", seed=71)
        prompt = generate(dec.scaled(k=L, kmax=L, rounds=1, seed=72))
        lp, pr = prompt.layers[0], prompt.rounds[0]
        lp.A[:] = lp.A * scale
        lp.conv_w[:] = np.array([0.0, 0.0, 0.0, 1.0], dtype=lp.conv_w.dtype)      # conv = identity: no fp32-vs-fp64 rounding ties in
        if lp.conv_b is not None:                                                  # the bf16 conv output, the error seen is the scan's
            lp.conv_b[:] = 0.0
        hip = HipLayer(dec, lp)
        ora = eager_oracle(dec, lp)
        y_ref, _, _ = ora.verify(pr.x_raw, pr.dt[0], pr.B[0], pr.C[0])
        ora.commit(np.full(2, L))
        d_x = to_dev(pr.x_raw, io)
        y = torch.empty_like(d_x)
        ssmv.ssm_prefill_chunked(hip.dims, hip.cache.c, d_x, hip.conv_w, hip.conv_b, to_dev(pr.dt[0], io), to_dev(pr.B[0], io),
                                 to_dev(pr.C[0], io), hip.A, hip.D, L, y)
        y_h, h_g = to_host(y), to_host(hip.materialize())
        assert np.all(np.isfinite(y_h)) and np.all(np.isfinite(h_g))
        e_y, e_h = rel_err(y_h, y_ref), rel_err(h_g, ora.h)
        print("A x %g, %s: y error %.3g, state error %.3g" % (scale, io, e_y, e_h))
        assert e_y <= TOL[io]
        assert e_h <= (1e-4 if io == "bf16" else 1e-5), "state after the prompt: %.3g" % e_h
