// Shared by the two kernels that treat a dense [M, D] buffer as one stream of aligned 16-byte chunks
// (the destination-aligned gather and the source-aligned scatter): where a wavefront tile of chunks
// begins in (row, column) terms, and which row a chunk of the tile starts in.
#pragma once

#include "ud_gather_kernel.hpp"

namespace ud {

// What the host works out once per launch.
struct FlatArgs {
    char *obase;        // 16-byte boundary at or below element 0 of the dense buffer: chunk c is obase + 16 c
    int64_t nchunks;    // chunks that overlap the buffer
    int64_t ntiles;
    int64_t pre;        // vrows * D - shift: chunk-grid element x is element x + pre counted from row -vrows
    int64_t vrows;      // virtual rows before row 0 that hold the `shift` elements preceding element 0
    double rcp_d;       // 1 / D
    float rcp_d_f;
};

// ID number k (>= 0) counted from `base`, which need not be a valid address itself.  The ID type is a
// template parameter: a run-time choice would put every load in a branch of its own, and the loads of a
// tile would then wait for one another.
template <bool I64>
__device__ __forceinline__ int64_t load_id_at(const char *base, uint32_t k)
{
    if constexpr (I64)
        return ((const UD_GLOBAL int64_t *)base)[k];
    else
        return static_cast<int64_t>(((const UD_GLOBAL int32_t *)base)[k]);
}

// The chunk grid of a dense buffer of M x D elements of `esz` bytes at `dense`, P x 64 chunks per tile.
inline FlatArgs make_flat_args(const void *dense, int64_t M, int64_t D, int esz, int P)
{
    FlatArgs f{};
    const int64_t epc = 16 / esz;
    const uintptr_t addr = reinterpret_cast<uintptr_t>(dense);
    const int64_t shift = static_cast<int64_t>(addr & 15u) / esz;
    f.obase = reinterpret_cast<char *>(addr - static_cast<uintptr_t>(shift) * esz);
    f.vrows = (shift + D - 1) / D;
    f.pre = f.vrows * D - shift;
    f.nchunks = (shift + M * D + epc - 1) / epc;
    const int64_t tile = 64 * P;
    f.ntiles = (f.nchunks + tile - 1) / tile;
    f.rcp_d = 1.0 / static_cast<double>(D);
    f.rcp_d_f = 1.0f / static_cast<float>(D);
    return f;
}

// Row i0 and column j0 of chunk-grid element x0 (the first of a tile; the same in every lane).  Counting
// from the vrows virtual rows keeps the dividend non-negative; one double-precision multiply stands in
// for the 64-bit division (the quotient is off by one at most, M x D being below 2^48).
__device__ __forceinline__ void tile_origin(const FlatArgs &f, int64_t D, int64_t x0, int64_t *i0, uint32_t *j0)
{
    const int64_t y0 = x0 + f.pre;
    int64_t q0 = static_cast<int64_t>(static_cast<double>(y0) * f.rcp_d);
    int64_t rem = y0 - q0 * D;
    if (rem < 0) {
        --q0;
        rem += D;
    } else if (rem >= D) {
        ++q0;
        rem -= D;
    }
    *i0 = q0 - f.vrows;
    *j0 = static_cast<uint32_t>(rem);
}

// How many rows after the tile's first row an element lies that is y columns past that row's start
// (y < D + TILE_ELEMS <= D + 2048).
template <uint32_t TILE_ELEMS>
__device__ __forceinline__ uint32_t rows_ahead(uint32_t y, uint32_t D, float rcp_d_f)
{
    if (D >= TILE_ELEMS)
        return y >= D ? 1u : 0u;
    // y < 2 * TILE_ELEMS <= 4096: the float quotient is off by one at most
    uint32_t di = static_cast<uint32_t>(static_cast<float>(y) * rcp_d_f);
    if (di * D > y)
        --di;
    else if (y - di * D >= D)
        ++di;
    return di;
}

} // namespace ud
