"""The C-ABI library without a GPU: it loads, exports every symbol the header declares, and rejects
bad arguments on the host before any HIP call (so these error paths run on a CPU-only machine)."""
import ctypes
import os
import re

import pytest

import paper_2408_15237_amd as ssmv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "ssmv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^(?:int|const char \*)\s*(\w+)\s*\(", text, flags=re.M)
    assert len(names) >= 12
    return names


def test_library_exports_every_declared_symbol():
    lib = ssmv.load_library()
    declared = _declared()
    for name in declared:
        assert hasattr(lib, name), "libssmv.so does not export %s" % name
    assert sorted(declared) == sorted(ssmv.EXPORTS)
    assert "gfx950" in ssmv.ssmv_version()


def test_constants_match_header():
    text = open(os.path.join(ROOT, "include", "ssmv.h")).read()
    for name in ("SSMV_KMAX_LIMIT", "SSMV_CONV_WIDTH", "SSMV_CACHE_NPTR"):
        m = re.search(r"#define\s+%s\s+(\d+)" % name, text)
        assert int(m.group(1)) == getattr(ssmv, name)
    assert ctypes.sizeof(ssmv.ssmv_dims) == 14 * 4
    assert ctypes.sizeof(ssmv.ssmv_cache) == 15 * 8


def test_engine_choice_is_a_function_of_the_dimensions():
    mk = ssmv.make_dims
    assert ssmv.ssmv_engine_of(mk(32, 32, 128, 64, kmax=4, io="bf16")) == 1
    assert ssmv.ssmv_engine_of(mk(16, 32, 128, 64, kmax=8, io="bf16")) == 1
    assert ssmv.ssmv_engine_of(mk(1, 80, 64, 128, kmax=8, io="bf16")) == 1
    assert ssmv.ssmv_engine_of(mk(32, 32, 128, 64, kmax=4, io="bf16", engine="vector")) == 0
    assert ssmv.ssmv_engine_of(mk(32, 32, 128, 64, kmax=9, io="bf16")) == 0                           # 8 + 9 tokens in a launch
    assert ssmv.ssmv_engine_of(mk(32, 32, 128, 64, kmax=8, io="bf16", snapshot_mode="hj_only")) == 1  # 8 + 8
    assert ssmv.ssmv_engine_of(mk(32, 32, 128, 64, kmax=9, io="bf16", snapshot_mode="hj_only")) == 0
    assert ssmv.ssmv_engine_of(mk(32, 32, 128, 64, kmax=4, io="bf16", snapshot_mode="defer")) == 1    # 12 + 4
    assert ssmv.ssmv_engine_of(mk(32, 32, 128, 64, kmax=8, io="bf16", snapshot_mode="defer")) == 1
    assert ssmv.ssmv_engine_of(mk(32, 32, 128, 64, kmax=4, io="f32")) == 0
    assert ssmv.ssmv_engine_of(mk(32, 32, 32, 64, kmax=4, io="bf16")) == 0                            # headdim not a multiple of 64
    assert ssmv.ssmv_engine_of(mk(32, 32, 128, 16, kmax=4, io="bf16")) == 0
    assert ssmv.ssmv_engine_of(mk(1, 8192, 1, 16, kmax=8, io="bf16", a_mode="diag")) == 0
    d = mk(2, 4, 16, 16, kmax=4, io="f32")
    d.engine = 7
    assert _code(ssmv.ssmv_engine_of, d) == ssmv.SSMV_EINVAL


def test_cache_sizes():
    d = ssmv.make_dims(32, 32, 128, 64, kmax=4, io="bf16")
    s = ssmv.ssmv_cache_sizes(d)
    S = 32 * 32 * 128 * 64 * 4
    assert s[0] == 3 * S and s[1] == 32 * 8 * 4096 * 2 and s[2] == s[3] == 32 * 4 * 4096 * 2
    assert s[4] == s[5] == 32 * 4 * 32 * 2 and s[6] == s[7] == 32 * 4 * 64 * 2
    assert s[8:] == [256] * 7                       # every size is rounded up to 256-byte granules
    d = ssmv.make_dims(1, 8192, 1, 16, kmax=8, io="f32", a_mode="diag")
    s = ssmv.ssmv_cache_sizes(d)
    assert s[0] == 3 * 8192 * 16 * 4 and s[1] == 16 * 8192 * 4
    d = ssmv.make_dims(1, 1, 3, 16, kmax=1, io="bf16")
    assert ssmv.ssmv_cache_sizes(d) == [768, 256] + [256] * 13
    # deferred advance: one window ring of 16 entries per sequence, the second arrays one granule
    d = ssmv.make_dims(32, 32, 128, 64, kmax=4, io="bf16", snapshot_mode="defer")
    s = ssmv.ssmv_cache_sizes(d)
    assert s[2] == 32 * 16 * 4096 * 2 and s[4] == 32 * 16 * 32 * 2 and s[6] == 32 * 16 * 64 * 2 and s[3] == s[5] == s[7] == 256


def _code(fn, *a, **kw):
    with pytest.raises(ssmv.SsmvError) as ei:
        fn(*a, **kw)
    return ei.value.code


def test_dims_validation():
    mk = ssmv.make_dims
    sizes = ssmv.ssmv_cache_sizes
    assert _code(sizes, mk(0, 4, 16, 16)) == ssmv.SSMV_EINVAL
    assert _code(sizes, mk(1, 4, 16, 17)) == ssmv.SSMV_EUNSUPPORTED
    assert _code(sizes, mk(1, 4, 16, 16, kmax=17)) == ssmv.SSMV_EUNSUPPORTED
    assert _code(sizes, mk(1, 4, 16, 16, kmax=0)) == ssmv.SSMV_EINVAL
    assert _code(sizes, mk(1, 4, 16, 16, ngroups=3)) == ssmv.SSMV_EINVAL
    assert _code(sizes, mk(1, 4, 16, 16, ring_len=6)) == ssmv.SSMV_EINVAL          # not a power of two
    assert _code(sizes, mk(1, 4, 16, 16, kmax=8, ring_len=8)) == ssmv.SSMV_EINVAL  # < W-1+kmax
    assert _code(sizes, mk(1, 4, 16, 16, conv_width=3)) == ssmv.SSMV_EUNSUPPORTED
    assert _code(sizes, mk(1, 4, 16, 16, conv_channels=65)) == ssmv.SSMV_EINVAL
    assert _code(sizes, mk(1, 4, 2, 16, a_mode="diag")) == ssmv.SSMV_EINVAL        # diag needs headdim 1
    assert _code(sizes, mk(1, 4, 1, 128, a_mode="diag")) == ssmv.SSMV_EUNSUPPORTED
    assert _code(sizes, mk(1, 4, 16, 16, io=7)) == ssmv.SSMV_EINVAL
    assert _code(sizes, mk(1, 4, 16, 16, snapshot_mode=3)) == ssmv.SSMV_EINVAL
    assert _code(sizes, mk(1, 4, 16, 16, kmax=9, snapshot_mode="defer")) == ssmv.SSMV_EUNSUPPORTED   # two rounds must fit the window
    assert "dstate" in ssmv.load_library().ssmv_last_error().decode() or True


def _fake_cache(base=0x10000):
    c = ssmv.ssmv_cache()
    c.state, c.conv_ring = base, base + 0x100
    for i in range(2):
        c.win_xc[i], c.win_dt[i], c.win_B[i] = base + 0x200 + i * 0x10, base + 0x300 + i * 0x10, base + 0x400 + i * 0x10
    c.cur_slot, c.pend, c.pos, c.conv_head = base + 0x500, base + 0x510, base + 0x520, base + 0x530
    c.last_k, c.win_par, c.err_flag = base + 0x540, base + 0x550, base + 0x560
    return c


def test_argument_validation_precedes_any_gpu_work():
    """Every call below must fail on the host; none of these pointers is ever dereferenced."""
    d = ssmv.make_dims(2, 4, 16, 16, kmax=4, io="f32")
    c = _fake_cache()
    P = 0x20000      # plausible, aligned, never touched
    # NULL and misaligned tensors
    assert _code(ssmv.ssm_verify_multistep, d, c, None, P, P, P, P, P, 4, P, 0) == ssmv.SSMV_EINVAL
    assert _code(ssmv.ssm_verify_multistep, d, c, P, P, P, P, P, P + 4, 4, P, 0) == ssmv.SSMV_EALIGN
    assert _code(ssmv.ssm_verify_multistep, d, c, P, P, P, P, P, P, 4, None, 0) == ssmv.SSMV_EINVAL
    # k outside [1, kmax]
    assert _code(ssmv.ssm_verify_multistep, d, c, P, P, P, P, P, P, 0, P, 0) == ssmv.SSMV_EINVAL
    assert _code(ssmv.ssm_verify_multistep, d, c, P, P, P, P, P, P, 5, P, 0) == ssmv.SSMV_EINVAL
    assert _code(ssmv.conv1d_state_update, d, c, P, P, None, 9, P, 0) == ssmv.SSMV_EINVAL
    assert _code(ssmv.conv1d_state_update, d, c, P, None, None, 2, P, 0) == ssmv.SSMV_EINVAL
    assert _code(ssmv.conv1d_state_update, d, c, P, P, P + 2, 2, P, 0) == ssmv.SSMV_EALIGN
    # the general call: exactly one of x_raw / xc, tok0 + k within kmax, flag values, no multi-call rounds without h_k
    blk = dict(dt=P, Bm=P, Cm=P, A=P, D=P, y_out=P, stream=0)
    assert _code(ssmv.ssm_block_multistep, d, c, k=4, **blk) == ssmv.SSMV_EINVAL
    assert _code(ssmv.ssm_block_multistep, d, c, k=4, xc=P, x_raw=P, conv_wgt=P, **blk) == ssmv.SSMV_EINVAL
    assert _code(ssmv.ssm_block_multistep, d, c, k=4, x_raw=P, **blk) == ssmv.SSMV_EINVAL          # no conv weights
    assert _code(ssmv.ssm_block_multistep, d, c, k=2, tok0=3, xc=P, **blk) == ssmv.SSMV_EINVAL
    assert _code(ssmv.ssm_block_multistep, d, c, k=1, tok0=-1, xc=P, **blk) == ssmv.SSMV_EINVAL
    assert _code(ssmv.ssm_block_multistep, d, c, k=1, tok0=1, xc=P, k_seq=P, **blk) == ssmv.SSMV_EUNSUPPORTED
    # a later call of a round must bring raw inputs: conv1d_state_update cannot append behind the round's earlier tokens
    assert _code(ssmv.ssm_block_multistep, d, c, k=1, tok0=1, xc=P, **blk) == ssmv.SSMV_EUNSUPPORTED
    # replayed rounds: flag values; last_call only with replay_round; only on the matrix-core engine
    assert _code(ssmv.ssm_block_multistep, d, c, k=1, x_raw=P, conv_wgt=P, last_call=True, **blk) == ssmv.SSMV_EINVAL
    assert _code(ssmv.ssm_block_multistep, d, c, k=1, x_raw=P, conv_wgt=P, replay_round=True, **blk) == ssmv.SSMV_EUNSUPPORTED
    d_mx = ssmv.make_dims(2, 4, 64, 64, kmax=4, io="bf16")
    ssmv.ssmv_set_tuning(4, 4)
    try:
        assert _code(ssmv.ssm_block_multistep, d_mx, c, k=1, x_raw=P, conv_wgt=P, replay_round=True, **blk) == ssmv.SSMV_EUNSUPPORTED
    finally:
        ssmv.ssmv_set_tuning(0, 0)
    assert _code(ssmv.ssm_block_multistep, d, c, k=1, xc=P, dt_softplus=2, **blk) == ssmv.SSMV_EINVAL
    assert _code(ssmv.ssm_block_multistep, d, c, k=1, xc=P, z=P + 2, **blk) == ssmv.SSMV_EALIGN
    d_hj = ssmv.make_dims(2, 4, 16, 16, kmax=4, io="f32", snapshot_mode="hj_only")
    assert _code(ssmv.ssm_block_multistep, d_hj, c, k=1, tok0=1, xc=P, **blk) == ssmv.SSMV_EUNSUPPORTED
    d_df = ssmv.make_dims(2, 4, 16, 16, kmax=4, io="f32", snapshot_mode="defer")       # no h_k slot to carry a round in either
    assert _code(ssmv.ssm_block_multistep, d_df, c, k=1, tok0=1, x_raw=P, conv_wgt=P, **blk) == ssmv.SSMV_EUNSUPPORTED
    assert _code(ssmv.ssmv_materialize_block, d, c, P, None, 3, P, 0) == ssmv.SSMV_EINVAL
    # prefill: length, mode and shape
    assert _code(ssmv.ssm_prefill_chunked, d, c, P, P, None, P, P, P, P, P, 0, P, 0) == ssmv.SSMV_EINVAL
    assert _code(ssmv.ssm_prefill_chunked, d, c, P, P, None, P, P, P, P, P, 8, P, 0) == ssmv.SSMV_EUNSUPPORTED      # 16 x 16
    d_ok = ssmv.make_dims(2, 4, 64, 64, kmax=4, io="bf16")
    assert _code(ssmv.ssm_prefill_chunked, d_ok, c, P, P, None, P, P, P, P, P, 8, None, 0) == ssmv.SSMV_EINVAL
    assert _code(ssmv.ssm_prefill_chunked, d_ok, c, P + 2, P, None, P, P, P, P, P, 8, P, 0) == ssmv.SSMV_EALIGN
    pf = dict(x_raw=P, conv_wgt=P, dt=P, Bm=P, Cm=P, A=P, D=P, y_out=P, stream=0)
    assert _code(ssmv.ssm_prefill_block, d_ok, c, L=8, dt_softplus=2, **pf) == ssmv.SSMV_EINVAL
    assert _code(ssmv.ssm_prefill_block, d_ok, c, L=8, z=P + 4, **pf) == ssmv.SSMV_EALIGN
    assert _code(ssmv.ssm_prefill_block, d_ok, c, L=8, seq_len=P + 2, **pf) == ssmv.SSMV_EALIGN
    # 32-bit token offsets: the widest token row decides, here B and C (8 groups x 128) against 4 x 64 channels
    d_wide = ssmv.make_dims(1, 8, 32, 128, ngroups=8, kmax=4, io="bf16")
    assert _code(ssmv.ssm_prefill_chunked, d_wide, c, P, P, None, P, P, P, P, P, 3000000, P, 0) == ssmv.SSMV_EUNSUPPORTED
    d_diag = ssmv.make_dims(1, 64, 1, 16, a_mode="diag")
    assert _code(ssmv.ssm_prefill_chunked, d_diag, c, P, P, None, P, P, P, P, P, 8, P, 0) == ssmv.SSMV_EUNSUPPORTED
    # broken cache struct
    bad = _fake_cache()
    bad.pend = None
    assert _code(ssmv.ssm_commit_rollback, d, bad, P, 0) == ssmv.SSMV_EINVAL
    bad = _fake_cache()
    bad.state = 0x10008
    assert _code(ssmv.ssmv_materialize, d, bad, P, P, 0) == ssmv.SSMV_EALIGN
    assert _code(ssmv.ssm_commit_rollback, d, c, None, 0) == ssmv.SSMV_EINVAL
    assert _code(ssmv.ssmv_cache_reset, d, bad, None, None, 0) == ssmv.SSMV_EALIGN
    # gated norm
    assert _code(ssmv.ssmv_gated_rmsnorm, P, None, P, 4, 64, 48, 1e-5, "bf16", P, 0) == ssmv.SSMV_EINVAL         # 64 % 48
    assert _code(ssmv.ssmv_gated_rmsnorm, P, None, P, 4, 64, 4, 1e-5, "bf16", P, 0) == ssmv.SSMV_EUNSUPPORTED    # group < one vector
    assert _code(ssmv.ssmv_gated_rmsnorm, P, None, P, 0, 64, 64, 1e-5, "bf16", P, 0) == ssmv.SSMV_EINVAL
    assert _code(ssmv.ssmv_gated_rmsnorm, P, P + 4, P, 4, 64, 64, 1e-5, "bf16", P, 0) == ssmv.SSMV_EALIGN
    assert _code(ssmv.ssmv_gated_rmsnorm, P, None, None, 4, 64, 64, 1e-5, "f32", P, 0) == ssmv.SSMV_EINVAL
    # helpers
    assert _code(ssmv.ssmv_first_conflict, None, P, 2, 2, P, 0) == ssmv.SSMV_EINVAL
    assert _code(ssmv.ssmv_first_conflict, P, P, 0, 2, P, 0) == ssmv.SSMV_EINVAL
    assert _code(ssmv.ssmv_copy_probe, P, P, None, 24, 0) == ssmv.SSMV_EINVAL
    assert _code(ssmv.ssmv_copy_probe, P, P + 8, None, 32, 0) == ssmv.SSMV_EALIGN
    assert _code(ssmv.ssmv_set_tuning, 3, 0) == ssmv.SSMV_EINVAL
    assert _code(ssmv.ssmv_set_tuning, 0, 3) == ssmv.SSMV_EINVAL
    # a launch shape that is not built for this state size is refused before launch
    ssmv.ssmv_set_tuning(8, 4)
    try:
        d256 = ssmv.make_dims(1, 2, 8, 256, kmax=2, io="f32")
        assert _code(ssmv.ssm_verify_multistep, d256, c, P, P, P, P, P, P, 2, P, 0) == ssmv.SSMV_EUNSUPPORTED
    finally:
        ssmv.ssmv_set_tuning(0, 0)
    assert len(ssmv.load_library().ssmv_last_error()) > 0
