"""GPU parity on seeded random corners of the supported space: shapes (also three 64-row tiles per head, a single
state column tile, odd batches), groups, draft counts from 1 to kmax, every snapshot mode, both engines, both conv
activations, fused and split conv.  Each case is a full run_parity: every y, conv output, the logical state every few
rounds and every integer against the eager fp64 oracle and the integer model."""
import numpy as np
import pytest

import paper_2408_15237_amd as ssmv
from workload import Workload, generate

from _harness import run_parity

pytestmark = pytest.mark.gpu


def _cases():
    rng = np.random.default_rng(20240815)
    out = []
    for i in range(28):
        io = "bf16" if i % 4 else "f32"
        headdim = int(rng.choice([64, 128, 192] if io == "bf16" else [16, 48, 64]))
        dstate = int(rng.choice([32, 64, 128] if io == "bf16" else [16, 32, 64]))
        ngroups = int(rng.choice([1, 1, 2]))
        nheads = ngroups * int(rng.integers(1, 4))
        snap = ["both", "hj_only", "defer"][i % 3]
        kmax = int(rng.integers(1, 9))
        k_sched = [int(rng.integers(1, kmax + 1)) for _ in range(int(rng.integers(10, 22)))]
        k_sched[int(rng.integers(0, len(k_sched)))] = kmax
        out.append(dict(
            wl=Workload("rnd%d" % i, "scalar", batch=int(rng.integers(1, 6)), nheads=nheads, headdim=headdim, dstate=dstate, k=k_sched[0],
                        kmax=kmax, rounds=len(k_sched), io=io, accept=str(rng.choice(["uniform", "geometric", "all"])), accept_p=0.35,
                        ngroups=ngroups, conv_act=str(rng.choice(["none", "silu"])), conv_bias=bool(rng.integers(0, 2)),
                        snapshot_mode=snap, engine="vector" if (io == "bf16" and i % 7 == 3) else "auto", seed=100 + i),
            ks=k_sched, fused=bool(i % 2)))
    return out


CASES = _cases()


@pytest.mark.parametrize("case", CASES, ids=[c["wl"].name + "_" + c["wl"].snapshot_mode + "_" + c["wl"].io for c in CASES])
def test_random_corner(case):
    wl = case["wl"]
    data = generate(wl, k_schedule=case["ks"])
    worst = run_parity(wl, data, fused=case["fused"], reverify=True, check_state_every=3)
    assert worst["y"] >= 0.0


def test_the_cases_reach_both_engines_and_all_modes():
    engines = set()
    for c in CASES:
        wl = c["wl"]
        d = ssmv.make_dims(wl.batch, wl.nheads, wl.headdim, wl.dstate, ngroups=wl.ngroups, kmax=wl.kmax_eff, ring_len=wl.ring_len,
                           io=wl.io, conv_act=wl.conv_act, snapshot_mode=wl.snapshot_mode, engine=wl.engine)
        engines.add((ssmv.ssmv_engine_of(d), wl.snapshot_mode))
    assert engines == {(e, m) for e in (0, 1) for m in ("both", "hj_only", "defer")}
