// Chunked row gather for gfx950: out[i, :] = conv(table[idx[i], :]).
//
// The paper's fix for misaligned rows (PyTorch-Direct, Section 4.5) keeps one
// lane per element and rotates each row's lanes so that a warp's accesses fall
// inside one memory line.  The goal it serves -- every request on the host
// link is a whole, aligned line that the row really occupies -- is met here
// differently, in the way that suits 64-lane wavefronts with 16-byte loads:
//
//   * a row is cut into the 16-byte chunks of memory it overlaps, aligned on
//     the SOURCE address.  Lane k of the lane group that owns the row loads
//     chunk k with one dwordx4 load, so a full wavefront load instruction
//     covers 1 KiB of consecutive, 16-byte aligned memory and the memory
//     pipeline sees only whole lines, whatever the row width;
//   * the first and last chunk of a row may hang over the row's ends.  They are
//     loaded whole (an aligned 16-byte chunk that overlaps the table lies in a
//     page the table occupies, and in a line the row touches anyway, so this
//     costs no extra request and cannot fault) and the bytes outside the row
//     are dropped before the store;
//   * each lane issues rows_in_flight x chunks_per_lane independent loads
//     before it stores anything, which is what keeps enough requests in flight
//     to cover the host link's round trip;
//   * the destination row generally has a different alignment; whole chunks go
//     out as dword-aligned dwordx4 stores, the partial head and tail chunk word
//     by word.
//
// Lane groups: lanes_per_row = 2^lg lanes share a row, 64 >> lg rows per
// wavefront instruction.  Which group size is best depends on what bounds the
// gather: an HBM-resident table wants no idle lanes (small groups for short
// rows), a host-resident one is fastest with one row per wavefront instruction
// even when most lanes idle; the choice is made on the host (ud_boundary.hip).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ud_internal.h"

namespace ud {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));   // same vector, only dword-aligned
typedef u32x4 u32x4_a2 __attribute__((aligned(2)));   // same vector, only 2-byte aligned
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef u32x2 u32x2_a2 __attribute__((aligned(2)));

// Every pointer this library dereferences on the GPU is a global-memory
// address (HBM or GPU-mapped host memory), never LDS or scratch; saying so lets
// the compiler emit global_* instead of flat_* instructions.
#define UD_GLOBAL __attribute__((address_space(1)))

// 16-byte aligned 16-byte load from the table
__device__ __forceinline__ u32x4 ld_chunk(const char *p)
{
    return *(const UD_GLOBAL u32x4 *)p;
}

// 16-byte store that is only dword-aligned
template <bool NT>
__device__ __forceinline__ void st_x4(void *p, u32x4 v)
{
    UD_GLOBAL u32x4_a4 *g = (UD_GLOBAL u32x4_a4 *)p;
    if constexpr (NT)
        __builtin_nontemporal_store(v, g);
    else
        *g = v;
}

template <bool NT, typename T>
__device__ __forceinline__ void st_scalar(T *p, T v)
{
    UD_GLOBAL T *g = (UD_GLOBAL T *)p;
    if constexpr (NT)
        __builtin_nontemporal_store(v, g);
    else
        *g = v;
}

__device__ __forceinline__ int64_t load_id(const void *idx, int itype, int64_t i)
{
    return itype == UD_I64 ? static_cast<const int64_t *>(idx)[i]
                           : static_cast<int64_t>(static_cast<const int32_t *>(idx)[i]);
}

// Where row r is read from: its slot in the HBM hot-row cache if it has one,
// else the table itself.
__device__ __forceinline__ const char *row_source(const GatherArgs &a, int64_t r, int64_t row_bytes)
{
    if (a.slot) {
        const int32_t s = a.slot[r];
        if (s >= 0)
            return a.cache + static_cast<int64_t>(s) * row_bytes;
    }
    return a.table + r * a.pitch_bytes;
}

// Exact binary16 -> binary32.  The hardware converter widens every finite
// value and infinity exactly (fp16 subnormals are never flushed: the f16
// denormal mode is "preserve").  NaNs are rebuilt from the bits so that the
// result does not depend on what the converter does with signalling NaNs:
// sign kept, payload moved up by 13 bits, quiet bit set.
__device__ __forceinline__ uint32_t widen_half(uint32_t h)
{
    const _Float16 x = __builtin_bit_cast(_Float16, static_cast<uint16_t>(h));
    uint32_t bits = __builtin_bit_cast(uint32_t, static_cast<float>(x));
    if ((h & 0x7fffu) > 0x7c00u)
        bits = ((h & 0x8000u) << 16) | 0x7fc00000u | ((h & 0x3ffu) << 13);
    return bits;
}

// Store words w[lo..hi) to d[lo..hi).  A chunk that lies wholly inside the row
// goes out as dwordx4 stores; the destination row generally has another
// alignment than the source, so these stores are only dword-aligned, which
// gfx950 global stores accept.  Head and tail chunks are stored word by word.
template <int NW, bool NTS>
__device__ __forceinline__ void store_words(uint32_t *d, const uint32_t (&w)[NW], int lo, int hi)
{
    if (lo == 0 && hi == NW) {
#pragma unroll
        for (int q = 0; q < NW; q += 4)
            st_x4<NTS>(d + q, u32x4{w[q], w[q + 1], w[q + 2], w[q + 3]});
        return;
    }
#pragma unroll
    for (int q = 0; q < NW; ++q)
        if (q >= lo && q < hi)
            st_scalar<NTS>(d + q, w[q]);
}

// Same for 2-byte output elements; v holds 8 halves, d[lo..hi) are written.
template <bool NTS>
__device__ __forceinline__ void store_halves(uint16_t *d, u32x4 v, int lo, int hi)
{
    if (lo == 0 && hi == 8 && (reinterpret_cast<uintptr_t>(d) & 3u) == 0) {
        st_x4<NTS>(d, v);
        return;
    }
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int q = 0; q < 8; ++q)
        if (q >= lo && q < hi)
            st_scalar<NTS>(d + q, static_cast<uint16_t>(w[q >> 1] >> ((q & 1) * 16)));
}

// DT: UD_F32 / UD_F16 / UD_F16_TO_F32.  U rows in flight per lane group, P
// chunks per lane per row.  lg = log2(lanes per row).
// Workgroups are 256 threads by default and 1024 on request (all waves of a
// workgroup share a compute unit, so few large workgroups keep the gather on few
// compute units): the launch bound is the larger of the two.
//
// Row order: one pass of a workgroup covers waves x rows-per-wave consecutive
// output rows, and a workgroup makes group_iters passes over adjacent rows
// before it strides on by the grid.  For host-resident tables the host sizes
// group_iters so that these rows span at least one 128-byte line of the ID
// list: the line is then fetched from HBM by one XCD's L2 once, instead of by
// every XCD whose workgroups happen to hold a few of its IDs.  (For HBM-resident
// tables group_iters is 1: there, several passes per wavefront cost up to 12%.)
//
// I64 (the ID type) is a template parameter, and the phases -- ID loads, table
// loads, one wait, stores -- are kept apart in the source: with a run-time ID
// type every ID load sits in a branch of its own, and a wait that the compiler
// places inside a conditional block is needed again after every later branch,
// so that the loads (and then the stores) of the rows in flight would wait for
// one another.  For the same reason loaded chunks are kept in scalars: vectors
// that are assigned conditionally end up copied between registers, with a wait
// before each copy.
template <int DT, int U, int P, bool NTS, bool I64>
// Launched with kBlockThreads threads but declared for up to 1024: the instructions generated are the same for
// either bound, yet with the larger one in the kernel's metadata the 64-byte-row gather over the host link
// measures 3% faster on MI355X (20.9 -> 21.6 GB/s, three runs each), the other widths the same.
__global__ __launch_bounds__(1024) void gather_chunked(GatherArgs a, int lg)
{
    constexpr int IN_ESZ = (DT == UD_F32) ? 4 : 2;      // table element bytes
    constexpr int EPC = 16 / IN_ESZ;                    // elements per 16-byte chunk
    const int lane = threadIdx.x & 63;
    const int lpr = 1 << lg;
    const int grp = lane >> lg;                         // which row of the wavefront's batch
    const int l = lane & (lpr - 1);                     // which chunk slot of that row
    const int rpw = 64 >> lg;                           // rows per wavefront per pass
    const int64_t rows_per_iter = static_cast<int64_t>(rpw) * U;
    const int waves_per_block = blockDim.x >> 6;
    const int64_t rows_per_pass = rows_per_iter * waves_per_block;     // rows one workgroup pass covers
    const int64_t rows_per_tile = rows_per_pass * a.group_iters;
    const int64_t wave_first = static_cast<int64_t>(threadIdx.x >> 6) * rows_per_iter;
    const int64_t row_bytes = a.D * IN_ESZ;
    // upper bound of chunks per row over all alignments; identical in every lane
    const int64_t span = static_cast<int64_t>(P) * lpr;
    const int64_t nch_bound = (row_bytes + 15 + 15) >> 4;

    for (int64_t tile = static_cast<int64_t>(blockIdx.x) * rows_per_tile; tile < a.M;
         tile += static_cast<int64_t>(gridDim.x) * rows_per_tile)
    for (int g = 0; g < a.group_iters; ++g) {
        const int64_t rb = tile + g * rows_per_pass + wave_first;
        if (rb >= a.M)
            break;
        int64_t i[U], r[U];
        const char *base[U]; // 16-byte aligned address at or below the row's first byte
        int head[U];         // bytes between base and the row's first byte
        int64_t nch[U];      // chunks the row overlaps; 0 = nothing to do
        // all ID loads first, then their uses: one round trip for the U rows, not U
#pragma unroll
        for (int u = 0; u < U; ++u) {
            i[u] = rb + static_cast<int64_t>(u) * rpw + grp;
            r[u] = 0;
            if (i[u] < a.M) {
                if constexpr (I64)
                    r[u] = ((const UD_GLOBAL int64_t *)a.idx)[i[u]];
                else
                    r[u] = ((const UD_GLOBAL int32_t *)a.idx)[i[u]];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            nch[u] = 0;
            base[u] = a.table;
            head[u] = 0;
            if (i[u] < a.M) {
                if (r[u] < 0 || r[u] >= a.N) {
                    if (l == 0)
                        atomicMin(a.err, static_cast<unsigned long long>(i[u]));
                } else {
                    const char *src = row_source(a, r[u], row_bytes);
                    head[u] = static_cast<int>(reinterpret_cast<uintptr_t>(src) & 15u);
                    base[u] = src - head[u];
                    nch[u] = (head[u] + row_bytes + 15) >> 4;
                }
            }
        }

        for (int64_t cb = 0; cb < nch_bound; cb += span) {
            uint32_t v[U][P][4];        // set, and later read, only where c < nch[u]
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    const int64_t c = cb + static_cast<int64_t>(p) * lpr + l;
                    if (c < nch[u]) {
                        const u32x4 t = ld_chunk(base[u] + c * 16);
                        v[u][p][0] = t.x, v[u][p][1] = t.y, v[u][p][2] = t.z, v[u][p][3] = t.w;
                    }
                }
            }
            __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): every load of this pass, once, outside the branches
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    const int64_t c = cb + static_cast<int64_t>(p) * lpr + l;
                    if (c >= nch[u])
                        continue;
                    // first element of this chunk, relative to the row (negative in the head chunk)
                    const int64_t e0 = c * EPC - head[u] / IN_ESZ;
                    const int lo = e0 < 0 ? static_cast<int>(-e0) : 0;
                    const int64_t left = a.D - e0;
                    const int hi = left < EPC ? static_cast<int>(left) : EPC;
                    const int64_t o = i[u] * a.D + e0;
                    if constexpr (DT == UD_F32) {
                        const uint32_t w[4] = {v[u][p][0], v[u][p][1], v[u][p][2], v[u][p][3]};
                        store_words<4, NTS>(static_cast<uint32_t *>(a.out) + o, w, lo, hi);
                    } else if constexpr (DT == UD_F16) {
                        store_halves<NTS>(static_cast<uint16_t *>(a.out) + o,
                                          u32x4{v[u][p][0], v[u][p][1], v[u][p][2], v[u][p][3]}, lo, hi);
                    } else {
                        uint32_t w[8];
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            w[2 * q] = widen_half(v[u][p][q] & 0xffffu);
                            w[2 * q + 1] = widen_half(v[u][p][q] >> 16);
                        }
                        store_words<8, NTS>(static_cast<uint32_t *>(a.out) + o, w, lo, hi);
                    }
                }
            }
        }
    }
}

template <int DT, int U, int P>
hipError_t launch_nt(const GatherArgs &a, const Plan &p, int lg, dim3 grid, dim3 block, hipStream_t s)
{
    const bool nts = p.flags & UD_TUNE_NT_STORE, i64 = a.itype == UD_I64;
    if (nts && i64)
        hipLaunchKernelGGL((gather_chunked<DT, U, P, true, true>), grid, block, 0, s, a, lg);
    else if (nts)
        hipLaunchKernelGGL((gather_chunked<DT, U, P, true, false>), grid, block, 0, s, a, lg);
    else if (i64)
        hipLaunchKernelGGL((gather_chunked<DT, U, P, false, true>), grid, block, 0, s, a, lg);
    else
        hipLaunchKernelGGL((gather_chunked<DT, U, P, false, false>), grid, block, 0, s, a, lg);
    return hipGetLastError();
}

// Host side: pick the (U, P) instantiation, the row tiling and the grid.
template <int DT>
hipError_t launch_chunked(const GatherArgs &a_in, const Plan &p, hipStream_t s)
{
    int lg = 0;
    while ((1 << lg) < p.lanes_per_row)
        ++lg;
    if ((1 << lg) != p.lanes_per_row || lg > 6)
        return hipErrorInvalidValue;
    GatherArgs a = a_in;
    const int wpb = kWavesPerBlock;
    const int64_t rows_per_pass = static_cast<int64_t>(64 >> lg) * p.rows_in_flight * wpb;
    const int64_t ids_per_line = a.itype == UD_I64 ? 16 : 32;         // IDs in a 128-byte line of the list
    a.group_iters = p.tile_id_lines ? static_cast<int>((ids_per_line + rows_per_pass - 1) / rows_per_pass) : 1;
    const int64_t rows_per_tile = rows_per_pass * a.group_iters;
    int64_t blocks = (a.M + rows_per_tile - 1) / rows_per_tile;
    if (blocks > p.max_blocks)
        blocks = p.max_blocks;
    if (blocks < 1)
        return hipSuccess;
    const dim3 grid(static_cast<unsigned>(blocks)), block(static_cast<unsigned>(wpb * 64));
    const int key = p.rows_in_flight * 10 + p.chunks_per_lane;
    switch (key) {
#define UD_CASE(U_, P_) \
    case U_ * 10 + P_:  \
        return launch_nt<DT, U_, P_>(a, p, lg, grid, block, s);
        UD_CASE(1, 1)
        UD_CASE(2, 1)
        UD_CASE(4, 1)
        UD_CASE(1, 2)
        UD_CASE(2, 2)
        UD_CASE(1, 3)
        UD_CASE(2, 3)
        UD_CASE(1, 4)
        UD_CASE(2, 4)
#undef UD_CASE
    default:
        return hipErrorInvalidValue;
    }
}

} // namespace ud
