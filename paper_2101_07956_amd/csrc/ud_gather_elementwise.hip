// One lane per output element: lane g = i*D + j copies element j of row idx[i].
// This is the thread layout of the unmodified indexing kernel that Section 4.5
// (Figure 4) of PyTorch-Direct starts from: rows straddle wavefronts and memory
// lines.  It is kept as the comparison point for the tuning table and as the
// fallback that works for any pointer alignment.
#include "ud_gather_kernel.hpp"

namespace ud {

template <int DT>
__global__ __launch_bounds__(kBlockThreads) void gather_elementwise(GatherArgs a)
{
    const int64_t total = a.M * a.D;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlockThreads;
    for (int64_t g = static_cast<int64_t>(blockIdx.x) * kBlockThreads + threadIdx.x; g < total; g += stride) {
        const int64_t i = g / a.D;
        const int64_t j = g - i * a.D;
        const int64_t r = load_id(a.idx, a.itype, i);
        if (r < 0 || r >= a.N) {
            if (j == 0)
                atomicMin(a.err, static_cast<unsigned long long>(i));
            continue;
        }
        const int64_t src = r * a.D + j;
        if constexpr (DT == UD_F32)
            static_cast<uint32_t *>(a.out)[g] = reinterpret_cast<const uint32_t *>(a.table)[src];
        else if constexpr (DT == UD_F16)
            static_cast<uint16_t *>(a.out)[g] = reinterpret_cast<const uint16_t *>(a.table)[src];
        else
            static_cast<uint32_t *>(a.out)[g] = widen_half(reinterpret_cast<const uint16_t *>(a.table)[src]);
    }
}

hipError_t launch_elementwise(const GatherArgs &a, int dtype, const Plan &p, hipStream_t s)
{
    const int64_t total = a.M * a.D;
    int64_t blocks = (total + kBlockThreads - 1) / kBlockThreads;
    if (blocks > p.max_blocks)
        blocks = p.max_blocks;
    if (blocks < 1)
        return hipSuccess;
    const dim3 grid(static_cast<unsigned>(blocks)), block(kBlockThreads);
    switch (dtype) {
    case UD_F32:
        hipLaunchKernelGGL(gather_elementwise<UD_F32>, grid, block, 0, s, a);
        break;
    case UD_F16:
        hipLaunchKernelGGL(gather_elementwise<UD_F16>, grid, block, 0, s, a);
        break;
    case UD_F16_TO_F32:
        hipLaunchKernelGGL(gather_elementwise<UD_F16_TO_F32>, grid, block, 0, s, a);
        break;
    default:
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

} // namespace ud
