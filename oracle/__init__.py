"""fp64 CPU oracle of the multi-step SSM verification path.

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports this.
"""
from .reference import (  # noqa: F401
    EagerOracle, BookkeepingModel, LazyMirror, first_conflict,
    conv_causal, scan_tokens, round_io, oracle_threads, softplus, step_size, silu_gate, rmsnorm_gated,
)
