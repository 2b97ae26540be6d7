"""The synthetic configurations the build is measured and parity-tested on.

Every field is a shape, a count or the name of a distribution; nothing here
computes anything.  `cfg0`..`cfg4` follow the five benchmark configurations
(tiny fp32 layer, 8B-shaped Mamba-2-style layer at batch 1, Mamba-1-style
diagonal-A layer, the 8B shape at batch 32, and a 24-layer stack).
"""
from __future__ import annotations

from dataclasses import dataclass, replace


@dataclass(frozen=True)
class Workload:
    name: str
    a_mode: str          # "scalar": A[H], one decay per head; "diag": A[H][N] with headdim == 1
    batch: int
    nheads: int
    headdim: int
    dstate: int
    k: int               # draft tokens per verify round
    rounds: int
    io: str              # "f32" | "bf16"  (state is always fp32 on the GPU, fp64 in the oracle)
    accept: str          # "uniform" in [0,k] | "geometric" (per-token reject prob p, truncated to [0,k])
    accept_p: float = 0.3
    ngroups: int = 1
    conv_width: int = 4
    conv_act: str = "none"   # "none" | "silu"
    conv_bias: bool = True
    snapshot_mode: str = "both"   # "both": h_j and h_k as Algorithm 2 | "hj_only": single-snapshot variant | "defer": h_j only when the window fills up
    engine: str = "auto"     # "auto": the library picks the kernel | "vector": the vector-ALU kernel and row-major state
    kmax: int = 0        # 0 -> k
    layers: int = 1
    seed: int = 0

    @property
    def conv_channels(self) -> int:
        return self.nheads * self.headdim

    @property
    def kmax_eff(self) -> int:
        return self.kmax if self.kmax > 0 else self.k

    @property
    def ring_len(self) -> int:
        need = self.conv_width - 1 + self.kmax_eff
        r = 1
        while r < need:
            r *= 2
        return r

    @property
    def state_elems(self) -> int:
        return self.nheads * self.headdim * self.dstate

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


CONFIGS = {
    # Tiny single layer, fp32.
    "cfg0": Workload("cfg0", "scalar", batch=1, nheads=4, headdim=16, dstate=16, k=4, rounds=8,
                     io="f32", accept="uniform"),
    # Mamba-2-style layer shaped like an 8B hybrid, batch 1.
    "cfg1": Workload("cfg1", "scalar", batch=1, nheads=32, headdim=128, dstate=64, k=4, rounds=64,
                     io="bf16", accept="uniform"),
    # Mamba-1-style diagonal A per channel.
    "cfg2": Workload("cfg2", "diag", batch=1, nheads=8192, headdim=1, dstate=16, k=8, rounds=64,
                     io="bf16", accept="geometric", accept_p=0.3),
    # Batched verification of the cfg1 shape, ragged acceptance per sequence.
    "cfg3": Workload("cfg3", "scalar", batch=32, nheads=32, headdim=128, dstate=64, k=4, rounds=64,
                     io="bf16", accept="uniform"),
    # 24 layers of the cfg1 shape applied in sequence.
    "cfg4": Workload("cfg4", "scalar", batch=16, nheads=32, headdim=128, dstate=64, k=8, rounds=32,
                     io="bf16", accept="uniform", layers=24),
}


def get_workload(name: str) -> Workload:
    return CONFIGS[name]
