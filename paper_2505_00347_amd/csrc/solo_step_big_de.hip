// Instantiations of the fused step for blocks of 2048 elements, dynamic-exponent codebook.
#include "solo_step_big.h"

namespace solo {
template <>
hipError_t launch_big<2, true>(uint32_t bits_v, bool bf16, const StepArgs &args, hipStream_t stream)
{
    return launch_big_impl<2, true>(bits_v, bf16, args, stream);
}
template <>
hipError_t launch_big<3, true>(uint32_t bits_v, bool bf16, const StepArgs &args, hipStream_t stream)
{
    return launch_big_impl<3, true>(bits_v, bf16, args, stream);
}
template <>
hipError_t launch_big<4, true>(uint32_t bits_v, bool bf16, const StepArgs &args, hipStream_t stream)
{
    return launch_big_impl<4, true>(bits_v, bf16, args, stream);
}
template <>
hipError_t launch_multi_big<2, true>(uint32_t bits_v, bool bf16, const MultiArgs &args, uint32_t count, bool ragged,
                                     hipStream_t stream)
{
    return launch_multi_big_impl<2, true>(bits_v, bf16, args, count, ragged, stream);
}
template <>
hipError_t launch_multi_big<3, true>(uint32_t bits_v, bool bf16, const MultiArgs &args, uint32_t count, bool ragged,
                                     hipStream_t stream)
{
    return launch_multi_big_impl<3, true>(bits_v, bf16, args, count, ragged, stream);
}
template <>
hipError_t launch_multi_big<4, true>(uint32_t bits_v, bool bf16, const MultiArgs &args, uint32_t count, bool ragged,
                                     hipStream_t stream)
{
    return launch_multi_big_impl<4, true>(bits_v, bf16, args, count, ragged, stream);
}
}  // namespace solo
