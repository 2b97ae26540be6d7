"""Seeded input generator (numpy PCG64) shared by the oracle tests, the GPU tests and the bench.

It draws shapes and values only.  Nothing here evaluates the recurrence, the
convolution or the cache bookkeeping; the one numeric operation performed is
rounding the draws to the I/O storage type so that the oracle and the GPU path
consume bit-identical numbers.

Draw order (fixed, so a seed names one data set):
  per layer:  A, D, conv weight, conv bias, h0
  if layers > 1:  the hand-off projection Wp
  per round:  x_raw (layer 0 only), then per layer dt, B, C, then accepted[batch]

Distributions: x ~ N(0,1); B, C ~ N(0,1)/sqrt(dstate); dt = softplus(N(0,1) - 4);
scalar mode A = -exp(U(0, ln 16)); diag mode A[c,n] = -(n+1) + U(-0.25, 0.25) per
channel; D ~ N(0,1); h0 ~ N(0, std 0.1); conv weight ~ N(0,1)/sqrt(W); conv
bias ~ N(0, std 0.1).  Accepted lengths: uniform integer in [0,k], or geometric
with per-token reject probability p truncated to [0,k].
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

from .configs import Workload


def round_to_io(a: np.ndarray, io: str) -> np.ndarray:
    """Round an array to the I/O storage type and return it as float32 (exact container)."""
    a32 = np.asarray(a, dtype=np.float32)
    if io == "f32":
        return a32
    if io == "bf16":
        return torch.from_numpy(a32).to(torch.bfloat16).to(torch.float32).numpy()
    raise ValueError(io)


@dataclass
class LayerParams:
    A: np.ndarray          # fp32 [H] (scalar) or [H][N] (diag); negative
    D: np.ndarray          # fp32 [H]
    conv_w: np.ndarray     # io-rounded, float32 container [Cx][W]
    conv_b: Optional[np.ndarray]   # io-rounded [Cx] or None
    h0: np.ndarray         # fp32 [batch][H][P][N]


@dataclass
class RoundInputs:
    x_raw: np.ndarray                 # io-rounded [batch][k][Cx]   (input of layer 0)
    dt: List[np.ndarray]              # per layer, io-rounded [batch][k][H]
    B: List[np.ndarray]               # per layer, io-rounded [batch][k][G][N]
    C: List[np.ndarray]               # per layer, io-rounded [batch][k][G][N]
    accepted: np.ndarray              # int32 [batch] in [0,k]


@dataclass
class WorkloadData:
    wl: Workload
    layers: List[LayerParams]
    rounds: List[RoundInputs] = field(default_factory=list)
    Wp: Optional[np.ndarray] = None   # io-rounded [Cx][Cx] hand-off projection (layers > 1)


def draw_accepted(rng: np.random.Generator, wl: Workload, k: int) -> np.ndarray:
    if wl.accept == "uniform":
        return rng.integers(0, k + 1, size=wl.batch).astype(np.int32)
    if wl.accept == "geometric":
        g = rng.geometric(wl.accept_p, size=wl.batch) - 1
        return np.minimum(g, k).astype(np.int32)
    if wl.accept == "all":
        return np.full(wl.batch, k, dtype=np.int32)
    if wl.accept == "none":
        return np.zeros(wl.batch, dtype=np.int32)
    raise ValueError(wl.accept)


def _softplus(z: np.ndarray) -> np.ndarray:
    return np.logaddexp(0.0, z)


def _draw_layer(rng: np.random.Generator, wl: Workload) -> LayerParams:
    H, P, N, W, Cx = wl.nheads, wl.headdim, wl.dstate, wl.conv_width, wl.conv_channels
    if wl.a_mode == "scalar":
        A = -np.exp(rng.uniform(0.0, np.log(16.0), size=H))
    elif wl.a_mode == "diag":
        A = -(np.arange(N, dtype=np.float64)[None, :] + 1.0) + rng.uniform(-0.25, 0.25, size=(H, 1))
    else:
        raise ValueError(wl.a_mode)
    D = rng.standard_normal(H)
    conv_w = rng.standard_normal((Cx, W)) / np.sqrt(W)
    conv_b = rng.standard_normal(Cx) * 0.1
    h0 = rng.standard_normal((wl.batch, H, P, N)) * 0.1
    return LayerParams(
        A=A.astype(np.float32),
        D=D.astype(np.float32),
        conv_w=round_to_io(conv_w, wl.io),
        conv_b=round_to_io(conv_b, wl.io) if wl.conv_bias else None,
        h0=h0.astype(np.float32),
    )


def _draw_round(rng: np.random.Generator, wl: Workload, k: int) -> RoundInputs:
    Bsz, H, N, G, Cx = wl.batch, wl.nheads, wl.dstate, wl.ngroups, wl.conv_channels
    x_raw = round_to_io(rng.standard_normal((Bsz, k, Cx)), wl.io)
    dts, Bs, Cs = [], [], []
    for _ in range(wl.layers):
        dts.append(round_to_io(_softplus(rng.standard_normal((Bsz, k, H)) - 4.0), wl.io))
        Bs.append(round_to_io(rng.standard_normal((Bsz, k, G, N)) / np.sqrt(N), wl.io))
        Cs.append(round_to_io(rng.standard_normal((Bsz, k, G, N)) / np.sqrt(N), wl.io))
    acc = draw_accepted(rng, wl, k)
    return RoundInputs(x_raw=x_raw, dt=dts, B=Bs, C=Cs, accepted=acc)


def generate(wl: Workload, rounds: Optional[int] = None, k_schedule=None) -> WorkloadData:
    """Draw every parameter and every round's inputs for `wl`.

    `k_schedule`, if given, is a list of per-round draft counts (each <= wl.kmax_eff)
    replacing the constant wl.k; the draw order is otherwise unchanged.
    """
    rng = np.random.default_rng(wl.seed)
    n_rounds = wl.rounds if rounds is None else rounds
    layers = [_draw_layer(rng, wl) for _ in range(wl.layers)]
    data = WorkloadData(wl=wl, layers=layers)
    if wl.layers > 1:
        Cx = wl.conv_channels
        data.Wp = round_to_io(rng.standard_normal((Cx, Cx)) / np.sqrt(Cx), wl.io)
    for r in range(n_rounds):
        k = wl.k if k_schedule is None else int(k_schedule[r])
        assert 1 <= k <= wl.kmax_eff
        data.rounds.append(_draw_round(rng, wl, k))
    return data


@dataclass
class BlockExtras:
    """Inputs of the optional block pieces, drawn from a stream of their own (seed + 1000003) so that the
    data sets above do not change: per layer a step-size bias, per round and layer a raw step-size projection
    (the step is softplus(raw + bias)), per round a gate input z."""
    dt_bias: List[np.ndarray]            # per layer [nheads] float32
    dt_raw: List[List[np.ndarray]]       # [round][layer] [batch][k][nheads], io-representable
    z: List[np.ndarray]                  # [round] [batch][k][conv_channels], io-representable


def block_extras(data: WorkloadData) -> BlockExtras:
    """raw ~ N(0,1) - 4 and bias ~ U(-0.5, 0.5): softplus(raw + bias) has the spread of the plain workloads' dt;
    z ~ N(0,1)."""
    wl = data.wl
    rng = np.random.Generator(np.random.PCG64(wl.seed + 1000003))
    bias = [rng.uniform(-0.5, 0.5, size=wl.nheads).astype(np.float32) for _ in range(wl.layers)]
    dt_raw, z = [], []
    for rd in data.rounds:
        k = rd.x_raw.shape[1]
        dt_raw.append([round_to_io(rng.standard_normal((wl.batch, k, wl.nheads)) - 4.0, wl.io) for _ in range(wl.layers)])
        z.append(round_to_io(rng.standard_normal((wl.batch, k, wl.conv_channels)), wl.io))
    return BlockExtras(dt_bias=bias, dt_raw=dt_raw, z=z)
