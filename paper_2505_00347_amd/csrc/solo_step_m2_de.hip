// Instantiations of the fused step for 2-bit first-moment codes, dynamic-exponent codebook.
#include "solo_step.h"

namespace solo {
template <>
hipError_t launch_step<2, true>(uint32_t bits_v, uint32_t block_size, bool bf16, const StepArgs &args,
                          hipStream_t stream)
{
    return launch_step_impl<2, true>(bits_v, block_size, bf16, args, stream);
}
template <>
hipError_t launch_multi<2, true>(uint32_t bits_v, uint32_t block_size, bool bf16, const MultiArgs &args,
                          hipStream_t stream)
{
    return launch_multi_impl<2, true>(bits_v, block_size, bf16, args, stream);
}
}  // namespace solo
