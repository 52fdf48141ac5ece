// Write direction: table[idx[i], :] = src[i, :], rows written by GPU wavefronts
// straight into the (host-mapped or HBM) table.  PyTorch-Direct, Section 3: a
// GPU that can dereference host memory generates write requests on the host
// link just as it generates reads.
//
// Mirror image of the chunked gather: a destination row is cut into the
// 16-byte chunks of memory it overlaps, aligned on the DESTINATION (table)
// address, so that every full chunk is one aligned dwordx4 store and a
// wavefront store instruction covers consecutive whole lines of the table.
// Unlike a load, a store must not spill over the row's ends: of the partial head
// and tail chunks only the row's own elements are loaded (element by element,
// in the same load phase as the full chunks, so that nothing waits on them
// alone) and stored.  The source rows (dense, in HBM) generally have another
// alignment and are read with loads that are only element-aligned.
#include "ud_gather_kernel.hpp"

namespace ud {

// 16 bytes from a source address that is only element-aligned
template <int ESZ>
__device__ __forceinline__ u32x4 ld_src_chunk(const char *p)
{
    if constexpr (ESZ == 4)
        return *(const UD_GLOBAL u32x4_a4 *)p;
    else
        return *(const UD_GLOBAL u32x4_a2 *)p;
}

// Elements [lo, hi) of the 16 bytes at p (the others read as zero and are never stored).
template <int ESZ>
__device__ __forceinline__ u32x4 ld_src_partial(const char *p, int lo, int hi)
{
    uint32_t w[4] = {0, 0, 0, 0};
    if constexpr (ESZ == 4) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (q >= lo && q < hi)
                w[q] = ((const UD_GLOBAL uint32_t *)p)[q];
    } else {
#pragma unroll
        for (int q = 0; q < 8; ++q)
            if (q >= lo && q < hi)
                w[q >> 1] |= static_cast<uint32_t>(((const UD_GLOBAL uint16_t *)p)[q]) << ((q & 1) * 16);
    }
    return u32x4{w[0], w[1], w[2], w[3]};
}

// ESZ: element bytes (4 or 2).  U rows in flight per lane group, P chunks per
// lane per row, lg = log2(lanes per row).  a.table is the destination, a.out
// the dense source (reusing GatherArgs: `out` is read, `table` written).
template <int ESZ, int U, int P>
__global__ __launch_bounds__(kBlockThreads) void scatter_chunked(GatherArgs a, int lg)
{
    constexpr int EPC = 16 / ESZ;
    const int lane = threadIdx.x & 63;
    const int lpr = 1 << lg;
    const int grp = lane >> lg;
    const int l = lane & (lpr - 1);
    const int rpw = 64 >> lg;
    const int64_t rows_per_iter = static_cast<int64_t>(rpw) * U;
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t nwaves = static_cast<int64_t>(gridDim.x) * kWavesPerBlock;
    const int64_t row_bytes = a.D * ESZ;
    const int64_t span = static_cast<int64_t>(P) * lpr;
    const int64_t nch_bound = (row_bytes + 15 + 15) >> 4;
    char *table = const_cast<char *>(a.table);
    const char *src = static_cast<const char *>(a.out);

    for (int64_t rb = wave * rows_per_iter; rb < a.M; rb += nwaves * rows_per_iter) {
        int64_t i[U];
        char *base[U];   // 16-byte aligned address at or below the destination row's first byte
        int head[U];
        int64_t nch[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            i[u] = rb + static_cast<int64_t>(u) * rpw + grp;
            nch[u] = 0;
            base[u] = table;
            head[u] = 0;
            if (i[u] < a.M) {
                const int64_t r = load_id(a.idx, a.itype, i[u]);
                if (r < 0 || r >= a.N) {
                    if (l == 0)
                        atomicMin(a.err, static_cast<unsigned long long>(i[u]));
                } else {
                    char *dst = table + r * a.pitch_bytes;
                    head[u] = static_cast<int>(reinterpret_cast<uintptr_t>(dst) & 15u);
                    base[u] = dst - head[u];
                    nch[u] = (head[u] + row_bytes + 15) >> 4;
                }
            }
        }
        for (int64_t cb = 0; cb < nch_bound; cb += span) {
            u32x4 v[U][P];
            int lo[U][P], hi[U][P];      // elements of the chunk that belong to the row; lo >= hi: no chunk
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    const int64_t c = cb + static_cast<int64_t>(p) * lpr + l;
                    const int64_t e0 = c * EPC - head[u] / ESZ;   // first element of the chunk, relative to the row
                    const int64_t left = a.D - e0;
                    lo[u][p] = e0 < 0 ? static_cast<int>(-e0) : 0;
                    hi[u][p] = c < nch[u] ? (left < EPC ? static_cast<int>(left) : EPC) : 0;
                    v[u][p] = u32x4{0, 0, 0, 0};
                    const char *s16 = src + (i[u] * a.D + e0) * ESZ;
                    if (lo[u][p] == 0 && hi[u][p] == EPC)
                        v[u][p] = ld_src_chunk<ESZ>(s16);
                    else if (lo[u][p] < hi[u][p])
                        v[u][p] = ld_src_partial<ESZ>(s16, lo[u][p], hi[u][p]);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    if (lo[u][p] >= hi[u][p])
                        continue;
                    const int64_t c = cb + static_cast<int64_t>(p) * lpr + l;
                    char *d16 = base[u] + c * 16;
                    if (lo[u][p] == 0 && hi[u][p] == EPC) {
                        *(UD_GLOBAL u32x4 *)d16 = v[u][p];
                        continue;
                    }
                    // head or tail chunk: only the elements that belong to the row
                    const uint32_t w[4] = {v[u][p].x, v[u][p].y, v[u][p].z, v[u][p].w};
                    if constexpr (ESZ == 4) {
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            if (q >= lo[u][p] && q < hi[u][p])
                                ((UD_GLOBAL uint32_t *)d16)[q] = w[q];
                    } else {
#pragma unroll
                        for (int q = 0; q < 8; ++q)
                            if (q >= lo[u][p] && q < hi[u][p])
                                ((UD_GLOBAL uint16_t *)d16)[q] = static_cast<uint16_t>(w[q >> 1] >> ((q & 1) * 16));
                    }
                }
            }
        }
    }
}

template <int ESZ>
static hipError_t launch_scatter_esz(const GatherArgs &a, const Plan &p, int lg, dim3 grid, hipStream_t s)
{
    const int key = p.rows_in_flight * 10 + p.chunks_per_lane;
    switch (key) {
#define UD_CASE(U_, P_)                                                                                          \
    case U_ * 10 + P_:                                                                                           \
        hipLaunchKernelGGL((scatter_chunked<ESZ, U_, P_>), grid, dim3(kBlockThreads), 0, s, a, lg);              \
        return hipGetLastError();
        UD_CASE(1, 1)
        UD_CASE(2, 1)
        UD_CASE(4, 1)
        UD_CASE(1, 2)
        UD_CASE(2, 2)
        UD_CASE(1, 3)
        UD_CASE(1, 4)
#undef UD_CASE
    default:
        return hipErrorInvalidValue;
    }
}

hipError_t launch_scatter(const GatherArgs &a, int elem_bytes, const Plan &p, hipStream_t s)
{
    int lg = 0;
    while ((1 << lg) < p.lanes_per_row)
        ++lg;
    if ((1 << lg) != p.lanes_per_row || lg > 6)
        return hipErrorInvalidValue;
    const int64_t rows_per_wave = static_cast<int64_t>(64 >> lg) * p.rows_in_flight;
    const int64_t waves = (a.M + rows_per_wave - 1) / rows_per_wave;
    int64_t blocks = (waves + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > p.max_blocks)
        blocks = p.max_blocks;
    if (blocks < 1)
        return hipSuccess;
    const dim3 grid(static_cast<unsigned>(blocks));
    return elem_bytes == 4 ? launch_scatter_esz<4>(a, p, lg, grid, s) : launch_scatter_esz<2>(a, p, lg, grid, s);
}

} // namespace ud
