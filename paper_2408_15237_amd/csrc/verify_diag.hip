// Diagonal-A (Mamba-1 style: A[channel][n], headdim 1) instantiations of the fused verification kernel.
#include "verify_impl.h"

namespace ssmv {

int launch_verify_diag(const VerifyParams &p, VerifyShape shape, hipStream_t stream)
{
    return launch_verify_any<true>(p, shape, stream);
}

}  // namespace ssmv
