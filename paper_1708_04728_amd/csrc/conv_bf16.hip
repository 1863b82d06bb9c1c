// bf16 convolution forward (bf16 storage, fp32 accumulation).  Not implemented yet.
#include "dr_internal.h"

namespace dr {

int launch_conv_bf16(const ConvGeom&, const uint16_t*, const uint16_t*, const float*, const uint16_t*, uint16_t*, hipStream_t)
{
    return fail(DR_ERR_UNSUPPORTED, "convolution: bf16 kernels are not available in this build");
}

}  // namespace dr
