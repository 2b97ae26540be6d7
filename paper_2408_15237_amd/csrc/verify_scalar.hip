// Scalar-A (Mamba-2 style: one decay per head) instantiations of the fused verification kernel.
#include "verify_impl.h"

namespace ssmv {

int launch_verify_scalar(const VerifyParams &p, VerifyShape shape, hipStream_t stream)
{
    return launch_verify_any<false>(p, shape, stream);
}

size_t verify_lds_bytes(const VerifyParams &p, bool diag)
{
    return (diag ? verify_lds_floats<true>(p.lds_tokens, p.k, p.N, p.rows_wg, p.z != nullptr)
                 : verify_lds_floats<false>(p.lds_tokens, p.k, p.N, p.rows_wg, p.z != nullptr)) * sizeof(float);
}

bool verify_shape_supported(int N, int R, bool diag)
{
    if (N != 16 && N != 32 && N != 64 && N != 128 && N != 256) return false;
    if (R != 1 && R != 2 && R != 4 && R != 8) return false;
    const int V = (N / lanes_per_row(N)) / 4;
    return R * V <= (diag ? 4 : 8);
}

}  // namespace ssmv
