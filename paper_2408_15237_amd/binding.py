"""ctypes binding of libssmv (declared in include/ssmv.h).

Argument marshalling only: every step of the path runs in the HIP kernels behind
the C ABI.  torch is used for device memory (``torch.empty(device="cuda")``,
``.data_ptr()``) and for the current HIP stream, nothing else.  There is no CPU
fallback: if the library cannot be loaded, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Dict, List, Optional

PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG, "libssmv.so")

SSMV_OK, SSMV_EINVAL, SSMV_EUNSUPPORTED, SSMV_EALIGN, SSMV_ESEQUENCE, SSMV_EHIP = 0, -1, -2, -3, -4, -5
SSMV_F32, SSMV_BF16 = 0, 1
SSMV_A_SCALAR, SSMV_A_DIAG = 0, 1
SSMV_ACT_NONE, SSMV_ACT_SILU = 0, 1
SSMV_SNAP_BOTH, SSMV_SNAP_HJ_ONLY, SSMV_SNAP_DEFER = 0, 1, 2
SSMV_WINDOW = 16
SSMV_KMAX_LIMIT = 16
SSMV_CONV_WIDTH = 4
SSMV_CACHE_NPTR = 15

IO_CODES = {"f32": SSMV_F32, "bf16": SSMV_BF16}
MODE_CODES = {"scalar": SSMV_A_SCALAR, "diag": SSMV_A_DIAG}
ACT_CODES = {"none": SSMV_ACT_NONE, "silu": SSMV_ACT_SILU}
SNAP_CODES = {"both": SSMV_SNAP_BOTH, "hj_only": SSMV_SNAP_HJ_ONLY, "defer": SSMV_SNAP_DEFER}
SSMV_ENGINE_AUTO, SSMV_ENGINE_VECTOR = 0, 1
ENGINE_CODES = {"auto": SSMV_ENGINE_AUTO, "vector": SSMV_ENGINE_VECTOR}

EXPORTS = [
    "ssmv_cache_sizes", "ssmv_cache_reset", "conv1d_state_update", "ssm_verify_multistep",
    "ssm_conv_verify_multistep", "ssm_block_multistep", "ssmv_materialize_block", "ssm_prefill_chunked", "ssm_prefill_block", "ssm_commit_rollback", "ssm_commit_rollback_multi", "ssmv_materialize", "ssmv_first_conflict", "ssmv_gated_rmsnorm", "ssmv_check",
    "ssmv_set_tuning", "ssmv_copy_probe", "ssmv_stream_probe", "ssmv_engine_of", "ssmv_last_error", "ssmv_version",
]


class ssmv_step_args(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in (
        "x_raw", "xc", "conv_wgt", "conv_bias", "dt", "dt_bias", "Bm", "Cm", "z", "A", "D", "k_seq", "y_out")] + [
        (n, ctypes.c_int32) for n in ("k", "tok0", "dt_softplus", "replay_round", "last_call")]


class ssmv_prefill_args(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in (
        "x_raw", "conv_wgt", "conv_bias", "dt", "dt_bias", "Bm", "Cm", "z", "A", "D", "seq_len", "y_out")] + [
        (n, ctypes.c_int32) for n in ("L", "dt_softplus")]


class SsmvError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("ssmv status %d: %s" % (code, msg))
        self.code = code


class ssmv_dims(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "batch", "nheads", "headdim", "dstate", "ngroups", "conv_width", "conv_channels", "kmax",
        "ring_len", "io_dtype", "a_mode", "conv_act", "snapshot_mode", "engine")]


class ssmv_cache(ctypes.Structure):
    _fields_ = [
        ("state", ctypes.c_void_p),
        ("conv_ring", ctypes.c_void_p),
        ("win_xc", ctypes.c_void_p * 2),
        ("win_dt", ctypes.c_void_p * 2),
        ("win_B", ctypes.c_void_p * 2),
        ("cur_slot", ctypes.c_void_p),
        ("pend", ctypes.c_void_p),
        ("pos", ctypes.c_void_p),
        ("conv_head", ctypes.c_void_p),
        ("last_k", ctypes.c_void_p),
        ("win_par", ctypes.c_void_p),
        ("err_flag", ctypes.c_void_p),
    ]


_lib = None


def load_library(build_if_missing: bool = True) -> ctypes.CDLL:
    """Load the in-tree libssmv.so; build it first only if no built library is there."""
    global _lib
    if _lib is not None:
        return _lib
    path = os.environ.get("SSMV_LIBRARY") or LIB_PATH     # another build of the same library (a sanitizer or profiling build)
    if not os.path.exists(path):
        if not build_if_missing or path != LIB_PATH:
            raise SsmvError(SSMV_EHIP, "libssmv.so is not built (%s)" % path)
        from .build import build
        build()
    lib = ctypes.CDLL(path)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    dp, cp = ctypes.POINTER(ssmv_dims), ctypes.POINTER(ssmv_cache)
    lib.ssmv_cache_sizes.argtypes = [dp, ctypes.POINTER(sz)]
    lib.ssmv_engine_of.argtypes = [dp]
    lib.ssmv_cache_reset.argtypes = [dp, cp, vp, vp, vp]
    lib.conv1d_state_update.argtypes = [dp, cp, vp, vp, vp, i32, vp, vp]
    lib.ssm_verify_multistep.argtypes = [dp, cp, vp, vp, vp, vp, vp, vp, i32, vp, vp]
    lib.ssm_conv_verify_multistep.argtypes = [dp, cp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp]
    lib.ssm_commit_rollback.argtypes = [dp, cp, vp, vp]
    lib.ssm_prefill_chunked.argtypes = [dp, cp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp]
    lib.ssm_prefill_block.argtypes = [dp, cp, ctypes.POINTER(ssmv_prefill_args), vp]
    lib.ssm_commit_rollback_multi.argtypes = [dp, cp, i32, vp, vp]
    lib.ssmv_materialize.argtypes = [dp, cp, vp, vp, vp]
    lib.ssm_block_multistep.argtypes = [dp, cp, ctypes.POINTER(ssmv_step_args), vp]
    lib.ssmv_materialize_block.argtypes = [dp, cp, vp, vp, i32, vp, vp]
    lib.ssmv_first_conflict.argtypes = [vp, vp, i32, i32, vp, vp]
    lib.ssmv_gated_rmsnorm.argtypes = [vp, vp, vp, i32, i32, i32, ctypes.c_float, i32, vp, vp]
    lib.ssmv_check.argtypes = [cp, vp]
    lib.ssmv_set_tuning.argtypes = [i32, i32]
    lib.ssmv_copy_probe.argtypes = [vp, vp, vp, sz, vp]
    lib.ssmv_stream_probe.argtypes = [i32, vp, vp, vp, sz, i32, i32, vp]
    for name in EXPORTS[:-2]:
        getattr(lib, name).restype = ctypes.c_int
    lib.ssmv_last_error.restype = ctypes.c_char_p
    lib.ssmv_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _ck(code: int) -> None:
    if code != SSMV_OK:
        raise SsmvError(code, load_library().ssmv_last_error().decode())


def _ptr(t) -> Optional[int]:
    """Device (or raw integer) pointer of an argument; None passes NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        s = torch.cuda.current_stream().cuda_stream
        return s if s else None
    return stream if stream else None


def make_dims(batch, nheads, headdim, dstate, ngroups=1, kmax=4, ring_len=None, io="bf16", a_mode="scalar",
              conv_act="none", conv_width=SSMV_CONV_WIDTH, conv_channels=None, snapshot_mode="both", engine="auto") -> ssmv_dims:
    if ring_len is None:
        ring_len = 1
        while ring_len < conv_width - 1 + kmax:
            ring_len *= 2
    return ssmv_dims(batch, nheads, headdim, dstate, ngroups, conv_width,
                     nheads * headdim if conv_channels is None else conv_channels, kmax, ring_len,
                     IO_CODES[io] if isinstance(io, str) else io,
                     MODE_CODES[a_mode] if isinstance(a_mode, str) else a_mode,
                     ACT_CODES[conv_act] if isinstance(conv_act, str) else conv_act,
                     SNAP_CODES[snapshot_mode] if isinstance(snapshot_mode, str) else snapshot_mode,
                     ENGINE_CODES[engine] if isinstance(engine, str) else engine)


# ---- the C entry points, same names, torch tensors (or raw pointers) in place of pointers ----------

def ssmv_engine_of(dims: ssmv_dims) -> int:
    rc = load_library().ssmv_engine_of(ctypes.byref(dims))
    if rc < 0:
        _ck(rc)
    return rc


def ssmv_cache_sizes(dims: ssmv_dims) -> List[int]:
    out = (ctypes.c_size_t * SSMV_CACHE_NPTR)()
    _ck(load_library().ssmv_cache_sizes(ctypes.byref(dims), out))
    return list(out)


def ssmv_cache_reset(dims, cache: ssmv_cache, h0=None, conv_init=None, stream=None) -> None:
    _ck(load_library().ssmv_cache_reset(ctypes.byref(dims), ctypes.byref(cache), _ptr(h0), _ptr(conv_init), _stream(stream)))


def conv1d_state_update(dims, cache, x_raw, wgt, bias, k: int, xc_out, stream=None) -> None:
    _ck(load_library().conv1d_state_update(ctypes.byref(dims), ctypes.byref(cache), _ptr(x_raw), _ptr(wgt), _ptr(bias),
                                           k, _ptr(xc_out), _stream(stream)))


def ssm_verify_multistep(dims, cache, xc, dt, Bm, Cm, A, D, k: int, y_out, stream=None) -> None:
    _ck(load_library().ssm_verify_multistep(ctypes.byref(dims), ctypes.byref(cache), _ptr(xc), _ptr(dt), _ptr(Bm), _ptr(Cm),
                                            _ptr(A), _ptr(D), k, _ptr(y_out), _stream(stream)))


def ssm_conv_verify_multistep(dims, cache, x_raw, wgt, bias, dt, Bm, Cm, A, D, k: int, y_out, stream=None) -> None:
    _ck(load_library().ssm_conv_verify_multistep(ctypes.byref(dims), ctypes.byref(cache), _ptr(x_raw), _ptr(wgt), _ptr(bias),
                                                 _ptr(dt), _ptr(Bm), _ptr(Cm), _ptr(A), _ptr(D), k, _ptr(y_out), _stream(stream)))


def ssm_block_multistep(dims, cache, *, dt, Bm, Cm, A, D, k: int, y_out, x_raw=None, xc=None, conv_wgt=None, conv_bias=None,
                        dt_bias=None, dt_softplus: bool = False, z=None, tok0: int = 0, k_seq=None, replay_round: bool = False,
                        last_call: bool = False, stream=None) -> None:
    a = ssmv_step_args(_ptr(x_raw), _ptr(xc), _ptr(conv_wgt), _ptr(conv_bias), _ptr(dt), _ptr(dt_bias), _ptr(Bm), _ptr(Cm),
                       _ptr(z), _ptr(A), _ptr(D), _ptr(k_seq), _ptr(y_out), k, tok0, int(dt_softplus), int(replay_round), int(last_call))
    _ck(load_library().ssm_block_multistep(ctypes.byref(dims), ctypes.byref(cache), ctypes.byref(a), _stream(stream)))


def ssmv_materialize_block(dims, cache, A, dt_bias, dt_softplus: bool, h_out, stream=None) -> None:
    _ck(load_library().ssmv_materialize_block(ctypes.byref(dims), ctypes.byref(cache), _ptr(A), _ptr(dt_bias), int(dt_softplus),
                                              _ptr(h_out), _stream(stream)))


def ssm_prefill_chunked(dims, cache, x_raw, wgt, bias, dt, Bm, Cm, A, D, L: int, y_out, stream=None) -> None:
    _ck(load_library().ssm_prefill_chunked(ctypes.byref(dims), ctypes.byref(cache), _ptr(x_raw), _ptr(wgt), _ptr(bias), _ptr(dt),
                                           _ptr(Bm), _ptr(Cm), _ptr(A), _ptr(D), L, _ptr(y_out), _stream(stream)))


def ssm_prefill_block(dims, cache, *, x_raw, conv_wgt, dt, Bm, Cm, A, D, L: int, y_out, conv_bias=None, dt_bias=None,
                      dt_softplus: bool = False, z=None, seq_len=None, stream=None) -> None:
    a = ssmv_prefill_args(_ptr(x_raw), _ptr(conv_wgt), _ptr(conv_bias), _ptr(dt), _ptr(dt_bias), _ptr(Bm), _ptr(Cm), _ptr(z), _ptr(A),
                          _ptr(D), _ptr(seq_len), _ptr(y_out), L, int(dt_softplus))
    _ck(load_library().ssm_prefill_block(ctypes.byref(dims), ctypes.byref(cache), ctypes.byref(a), _stream(stream)))


def ssm_commit_rollback_multi(dims, caches, accepted, stream=None) -> None:
    """`caches`: a ctypes array (ssmv_cache * n) or a sequence of ssmv_cache structs."""
    if not isinstance(caches, ctypes.Array):
        caches = (ssmv_cache * len(caches))(*caches)
    _ck(load_library().ssm_commit_rollback_multi(ctypes.byref(dims), caches, len(caches), _ptr(accepted), _stream(stream)))


def ssm_commit_rollback(dims, cache, accepted, stream=None) -> None:
    _ck(load_library().ssm_commit_rollback(ctypes.byref(dims), ctypes.byref(cache), _ptr(accepted), _stream(stream)))


def ssmv_materialize(dims, cache, A, h_out, stream=None) -> None:
    _ck(load_library().ssmv_materialize(ctypes.byref(dims), ctypes.byref(cache), _ptr(A), _ptr(h_out), _stream(stream)))


def ssmv_first_conflict(draft, target, batch: int, k: int, accepted, stream=None) -> None:
    _ck(load_library().ssmv_first_conflict(_ptr(draft), _ptr(target), batch, k, _ptr(accepted), _stream(stream)))


def ssmv_gated_rmsnorm(y, z, weight, rows: int, channels: int, group_size: int, eps: float, io, out, stream=None) -> None:
    _ck(load_library().ssmv_gated_rmsnorm(_ptr(y), _ptr(z), _ptr(weight), rows, channels, group_size, eps,
                                          IO_CODES[io] if isinstance(io, str) else io, _ptr(out), _stream(stream)))


def ssmv_check(cache, stream=None) -> None:
    _ck(load_library().ssmv_check(ctypes.byref(cache), _stream(stream)))


def ssmv_set_tuning(rows_per_lane: int = 0, waves_per_group: int = 0) -> None:
    _ck(load_library().ssmv_set_tuning(rows_per_lane, waves_per_group))


def ssmv_copy_probe(src, dst0, dst1, n_bytes: int, stream=None) -> None:
    _ck(load_library().ssmv_copy_probe(_ptr(src), _ptr(dst0), _ptr(dst1), n_bytes, _stream(stream)))


PROBE_MODES = {"read": 0, "write": 1, "r1w1": 2, "r1w2": 3, "empty": 4}


def ssmv_stream_probe(mode, src, dst0, dst1, n_bytes: int, piece_kib: int = 32, grid: int = 0, stream=None) -> None:
    _ck(load_library().ssmv_stream_probe(PROBE_MODES[mode] if isinstance(mode, str) else mode, _ptr(src), _ptr(dst0), _ptr(dst1),
                                         n_bytes, piece_kib, grid, _stream(stream)))


def ssmv_version() -> str:
    return load_library().ssmv_version().decode()


# ---- device memory for one layer's cache -----------------------------------------------------------

_FIELDS = ["state", "conv_ring", "win_xc0", "win_xc1", "win_dt0", "win_dt1", "win_B0", "win_B1",
           "cur_slot", "pend", "pos", "conv_head", "last_k", "win_par", "err_flag"]


@dataclass
class LayerCache:
    """Caller-side owner of the device buffers of one ssmv_cache (torch tensors) plus the C struct."""
    dims: ssmv_dims
    buffers: Dict[str, "object"]
    c: ssmv_cache

    @staticmethod
    def allocate(dims: ssmv_dims, device="cuda") -> "LayerCache":
        import torch
        sizes = ssmv_cache_sizes(dims)
        bufs = {}
        for name, nbytes in zip(_FIELDS, sizes):
            # 8-byte granules keep int64 views legal; torch device allocations are 256-byte aligned
            bufs[name] = torch.zeros((nbytes + 7) // 8, dtype=torch.int64, device=device)
        c = ssmv_cache()
        c.state = bufs["state"].data_ptr()
        c.conv_ring = bufs["conv_ring"].data_ptr()
        for i in range(2):
            c.win_xc[i] = bufs["win_xc%d" % i].data_ptr()
            c.win_dt[i] = bufs["win_dt%d" % i].data_ptr()
            c.win_B[i] = bufs["win_B%d" % i].data_ptr()
        for name in ("cur_slot", "pend", "pos", "conv_head", "last_k", "win_par", "err_flag"):
            setattr(c, name, bufs[name].data_ptr())
        return LayerCache(dims=dims, buffers=bufs, c=c)

    # views for tests and tools (host copies)
    def ints(self) -> Dict[str, "object"]:
        import torch
        b = self.dims.batch
        out = {}
        for name in ("cur_slot", "pend", "conv_head", "last_k"):
            out[name] = self.buffers[name].view(torch.int32)[:b].cpu().numpy()
        out["pos"] = self.buffers["pos"][:b].cpu().numpy()
        out["win_par"] = int(self.buffers["win_par"].view(torch.int32)[0].item())
        out["err_flag"] = int(self.buffers["err_flag"].view(torch.int32)[0].item())
        return out

    def state_view(self):
        import torch
        d = self.dims
        n = 3 * d.batch * d.nheads * d.headdim * d.dstate
        return self.buffers["state"].view(torch.float32)[:n].view(3, d.batch, d.nheads, d.headdim, d.dstate)
