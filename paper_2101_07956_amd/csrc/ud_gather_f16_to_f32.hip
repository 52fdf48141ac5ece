// Instantiations of the chunked gather for table dtype UD_F16_TO_F32 (one translation
// unit per dtype so that they compile in parallel).
#include "ud_gather_kernel.hpp"

namespace ud {
hipError_t launch_chunked_f16_to_f32(const GatherArgs &a, const Plan &p, hipStream_t s)
{
    return launch_chunked<UD_F16_TO_F32>(a, p, s);
}
} // namespace ud
