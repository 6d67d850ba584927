// Instantiations of the fused step for 3-bit first-moment codes, signed linear codebook.
#include "solo_step.h"

namespace solo {
template <>
hipError_t launch_step<3, false>(uint32_t bits_v, uint32_t block_size, bool bf16, const StepArgs &args,
                          hipStream_t stream)
{
    return launch_step_impl<3, false>(bits_v, block_size, bf16, args, stream);
}
template <>
hipError_t launch_multi<3, false>(uint32_t bits_v, uint32_t block_size, bool bf16, const MultiArgs &args,
                          hipStream_t stream)
{
    return launch_multi_impl<3, false>(bits_v, block_size, bf16, args, stream);
}
}  // namespace solo
