"""MI355X-native multi-step speculative verification through a selective state-space layer.

The product is the C-ABI library ``libssmv.so`` (hand-written HIP for gfx950, declared in
``include/ssmv.h``); this package is its thin ctypes binding.
"""
from .binding import (  # noqa: F401
    SsmvError, ssmv_dims, ssmv_cache, ssmv_step_args, LayerCache, make_dims, load_library, LIB_PATH, EXPORTS,
    ssmv_engine_of, ssmv_stream_probe, ssmv_cache_sizes, ssmv_cache_reset, conv1d_state_update, ssm_verify_multistep, ssm_conv_verify_multistep, ssm_commit_rollback,
    ssm_commit_rollback_multi, ssm_block_multistep, ssmv_materialize_block, ssm_prefill_chunked, ssm_prefill_block, ssmv_prefill_args,
    ssmv_materialize, ssmv_first_conflict, ssmv_gated_rmsnorm, ssmv_check, ssmv_set_tuning, ssmv_copy_probe, ssmv_version,
    SSMV_OK, SSMV_EINVAL, SSMV_EUNSUPPORTED, SSMV_EALIGN, SSMV_ESEQUENCE, SSMV_EHIP,
    SSMV_F32, SSMV_BF16, SSMV_A_SCALAR, SSMV_A_DIAG, SSMV_ACT_NONE, SSMV_ACT_SILU,
    SSMV_SNAP_BOTH, SSMV_SNAP_HJ_ONLY, SSMV_SNAP_DEFER, SSMV_WINDOW,
    SSMV_KMAX_LIMIT, SSMV_CONV_WIDTH, SSMV_CACHE_NPTR,
)
