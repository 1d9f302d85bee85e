// bf16 backward (placeholder until the kernel lands): reports "not supported".
#include "sb_kernels.h"

namespace sb {

hipError_t launch_bwd_bf16(const uint16_t*, const uint16_t*, const uint16_t*, const float*,
                           const uint16_t*, float*, float*, float*, int, int, int, int, hipStream_t)
{
    return hipErrorNotSupported;
}

}  // namespace sb
