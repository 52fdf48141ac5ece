// Instantiations of the chunked gather for table dtype UD_F16 (one translation
// unit per dtype so that they compile in parallel).
#include "ud_gather_kernel.hpp"

namespace ud {
hipError_t launch_chunked_f16(const GatherArgs &a, const Plan &p, hipStream_t s)
{
    return launch_chunked<UD_F16>(a, p, s);
}
} // namespace ud
