// Stand-ins for the kernel launchers of libssmv, for the host-only sanitizer build of the argument-validation layer
// (csrc/api.hip): every launch "succeeds" without touching a GPU, every shape query says yes.  Test infrastructure only.
#include "ssmv_internal.h"

namespace ssmv {
int launch_verify_scalar(const VerifyParams &, VerifyShape, hipStream_t) { return 0; }
int launch_verify_diag(const VerifyParams &, VerifyShape, hipStream_t) { return 0; }
size_t verify_lds_bytes(const VerifyParams &, bool) { return 0; }
bool verify_shape_supported(int N, int R, bool diag)
{
    if (N != 16 && N != 32 && N != 64 && N != 128 && N != 256) return false;
    if (R != 1 && R != 2 && R != 4 && R != 8) return false;
    return R * ((N / lanes_per_row(N)) / 4) <= (diag ? 4 : 8);
}
int launch_verify_mfma(const VerifyParams &, hipStream_t) { return 0; }
bool verify_mfma_supported(int N, int P) { return (N == 32 || N == 64 || N == 128) && P >= 64 && P % 64 == 0; }
int launch_conv(const ConvParams &, hipStream_t) { return 0; }
int launch_prefill(const PrefillParams &, hipStream_t) { return 0; }
int launch_prefill_bf16(const PrefillParams &, hipStream_t) { return 0; }
bool prefill_shape_supported(int P, int N) { return (P == 32 || P == 64 || P == 128) && (N == 32 || N == 64 || N == 128); }
int launch_commit(const CommitParams &, hipStream_t) { return 0; }
int launch_reset(const ResetParams &, hipStream_t) { return 0; }
int launch_first_conflict(const int32_t *, const int32_t *, int, int, int32_t *, hipStream_t) { return 0; }
int launch_copy_probe(const void *, void *, void *, size_t, hipStream_t) { return 0; }
int launch_stream_probe(int, const void *, void *, void *, size_t, int, int, hipStream_t) { return 0; }
int launch_gated_rmsnorm(const void *, const void *, const float *, int, int, int, float, int, void *, hipStream_t) { return 0; }
}  // namespace ssmv
