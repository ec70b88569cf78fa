// MLP gradients: placeholder until the MFMA kernels land.
#include "common.h"

namespace lsgd {

bool mlp_shape_supported(const lsgd_mlp_batch& b, const char** why)
{
    (void)b;
    *why = "MLP gradient kernels are not built yet";
    return false;
}
size_t mlp_scratch_bytes(int W, const lsgd_mlp_batch& b) { (void)W; (void)b; return 0; }
hipError_t launch_mlp_grad_loss(const uint16_t*, const float*, float*, float*, int, int64_t, int64_t,
                                const lsgd_mlp_batch&, const DeviceState&, hipStream_t)
{
    return hipErrorNotSupported;
}

} // namespace lsgd
