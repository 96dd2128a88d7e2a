// Fused kernels of the MLP half of a layer (Eq. 5 with the skip of Eq. 4 in the prologue).
#include "astl_mlp.h"
#include "profile.h"

namespace gswa {

bool astl_mlp_supported(int, int) { return false; }

size_t astl_mlp_bwd_ws_bytes(long, int, int) { return 0; }

hipError_t launch_astl_mlp_fwd(long, int, int, float, const bf16_t *, const bf16_t *, const bf16_t *, const bf16_t *,
                               const bf16_t *, const bf16_t *, const bf16_t *, const bf16_t *, bf16_t *, bf16_t *,
                               hipStream_t)
{
    return hipErrorNotSupported;
}

hipError_t launch_astl_mlp_bwd(long, int, int, float, const bf16_t *, const bf16_t *, const bf16_t *, const bf16_t *,
                               const bf16_t *, const bf16_t *, const bf16_t *, bf16_t *, float *, float *, float *,
                               float *, float *, float *, long, int, void *, hipStream_t)
{
    return hipErrorNotSupported;
}

} // namespace gswa
