// One lane per output element: lane g = i*D + j copies element j of row idx[i].
// This is the thread layout of the unmodified indexing kernel that Section 4.5
// (Figure 4) of PyTorch-Direct starts from: rows straddle wavefronts and memory
// lines.  It is kept as the comparison point for the tuning table and as the
// fallback that works for any pointer alignment.
//
// With SHIFT the kernel applies the paper's own remedy (Section 4.5, Figure 5):
// every row's lanes are rotated by s = ((i - r) * D) mod 64, so that lane g
// reads the element whose position within a 64-element (one wavefront) span of
// memory equals the lane's position in its wavefront; lanes pushed over the row
// end wrap around by the row length, and the output index is rotated
// identically, so the result is unchanged.  On a 64-lane wavefront the aligned
// span is 256 bytes (two lines) for 4-byte and 128 bytes for 2-byte elements.
#include "ud_gather_kernel.hpp"

namespace ud {

template <int DT, bool SHIFT>
__global__ __launch_bounds__(kBlockThreads) void gather_elementwise(GatherArgs a)
{
    const int64_t total = a.M * a.D;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlockThreads;
    for (int64_t g = static_cast<int64_t>(blockIdx.x) * kBlockThreads + threadIdx.x; g < total; g += stride) {
        const int64_t i = g / a.D;
        int64_t j = g - i * a.D;
        const int64_t r = load_id(a.idx, a.itype, i);
        if (r < 0 || r >= a.N) {
            if (j == 0)
                atomicMin(a.err, static_cast<unsigned long long>(i));
            continue;
        }
        constexpr int IN_ESZ = (DT == UD_F32) ? 4 : 2;
        const char *row = row_source(a, r, a.D * IN_ESZ);
        int64_t o = g;
        if constexpr (SHIFT) {
            // element number of the row start relative to a 64-element boundary of memory, minus the
            // same for the lane: rotate so that both agree
            const int64_t first = static_cast<int64_t>(reinterpret_cast<uintptr_t>(row) / IN_ESZ);
            int64_t s = (i * a.D - first) % 64;
            if (s < 0)
                s += 64;
            j = (j + s) % a.D;
            o = i * a.D + j;
        }
        if constexpr (DT == UD_F32)
            static_cast<uint32_t *>(a.out)[o] = reinterpret_cast<const uint32_t *>(row)[j];
        else if constexpr (DT == UD_F16)
            static_cast<uint16_t *>(a.out)[o] = reinterpret_cast<const uint16_t *>(row)[j];
        else
            static_cast<uint32_t *>(a.out)[o] = widen_half(reinterpret_cast<const uint16_t *>(row)[j]);
    }
}

__global__ __launch_bounds__(kBlockThreads) void fill_slots(const int64_t *rows, int64_t n, int32_t *slot)
{
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlockThreads;
    for (int64_t k = static_cast<int64_t>(blockIdx.x) * kBlockThreads + threadIdx.x; k < n; k += stride)
        slot[rows[k]] = static_cast<int32_t>(k);
}

hipError_t launch_fill_slots(const int64_t *rows, int64_t n, int32_t *slot, hipStream_t s)
{
    int64_t blocks = (n + kBlockThreads - 1) / kBlockThreads;
    if (blocks > 65536)
        blocks = 65536;
    if (blocks < 1)
        return hipSuccess;
    hipLaunchKernelGGL(fill_slots, dim3(static_cast<unsigned>(blocks)), dim3(kBlockThreads), 0, s, rows, n, slot);
    return hipGetLastError();
}

// *result = old value of *slot, and *slot = "no bad ID", in one atomic step.  `result` is pinned host
// memory the GPU can write.
__global__ void fetch_and_reset(unsigned long long *slot, unsigned long long *result)
{
    *result = atomicExch(slot, kNoBadIndex);
}

hipError_t launch_fetch_and_reset(unsigned long long *slot, unsigned long long *result, hipStream_t s)
{
    hipLaunchKernelGGL(fetch_and_reset, dim3(1), dim3(1), 0, s, slot, result);
    return hipGetLastError();
}

__global__ void init_slots(unsigned long long *words, int n)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k < n)
        words[k] = kNoBadIndex;
}

hipError_t launch_init_slots(unsigned long long *words, int n, hipStream_t s)
{
    if (n < 1)
        return hipSuccess;
    hipLaunchKernelGGL(init_slots, dim3((n + 63) / 64), dim3(64), 0, s, words, n);
    return hipGetLastError();
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
    const bool shift = p.flags & UD_TUNE_CIRCULAR_SHIFT;
    switch (dtype) {
    case UD_F32:
        if (shift)
            hipLaunchKernelGGL((gather_elementwise<UD_F32, true>), grid, block, 0, s, a);
        else
            hipLaunchKernelGGL((gather_elementwise<UD_F32, false>), grid, block, 0, s, a);
        break;
    case UD_F16:
        if (shift)
            hipLaunchKernelGGL((gather_elementwise<UD_F16, true>), grid, block, 0, s, a);
        else
            hipLaunchKernelGGL((gather_elementwise<UD_F16, false>), grid, block, 0, s, a);
        break;
    case UD_F16_TO_F32:
        if (shift)
            hipLaunchKernelGGL((gather_elementwise<UD_F16_TO_F32, true>), grid, block, 0, s, a);
        else
            hipLaunchKernelGGL((gather_elementwise<UD_F16_TO_F32, false>), grid, block, 0, s, a);
        break;
    default:
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

} // namespace ud
