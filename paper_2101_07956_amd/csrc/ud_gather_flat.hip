// Destination-aligned row gather for tables that live in HBM.
//
// When the table is read over the host link, what matters is the shape of the
// read requests, and the chunked kernel aligns its 16-byte chunks on the source
// rows (ud_gather_kernel.hpp).  When the table is in HBM the gather is a copy
// bound by HBM bandwidth, and the side that is sensitive to alignment is the
// write: a store instruction whose lanes are only dword-aligned straddles
// 16-byte segments, and output lines that two wavefronts each write in part
// leave the L2 as partial lines.  Widths that are no multiple of 16 bytes
// (602 floats = 2408 bytes) pay for both.
//
// Here the dense output [M, D] is taken as one stream of 16-byte chunks,
// aligned on the output address.  A wavefront owns 64 x P consecutive chunks
// (P KiB of output), so every store is an aligned dwordx4 and every output
// line is written whole by one wavefront, whatever D is.  Lane l finds the row
// and column its chunk starts at, and
//   * if the chunk lies inside one row (all but one chunk per row end at
//     most), loads its 16 bytes of output from that row with one load that is
//     only element-aligned on the source -- reads tolerate that: the lines are
//     fetched whole from HBM either way;
//   * else (the chunk lies across a row end) loads its elements one by one from
//     the two rows, in the same load phase, so that such chunks cost no extra
//     round trip; elements outside the output, or of rows with a bad ID, are
//     left out of the store.
// At HBM rates the instruction stream matters: everything that is the same for
// a whole wavefront tile (its first row and column, base addresses, bounds) is
// computed once in scalar registers, per-chunk work is 32-bit, and the row of a
// tile's first element comes from one double-precision multiply instead of a
// 64-bit division.  Results are bit-identical to the chunked kernel's.
#include "ud_flat.hpp"

namespace ud {

// Columns and row offsets inside a tile are handled in 32 bits, the row address as a 32 x 32-bit
// product: D plus one tile of elements, the row pitch and the row count must fit.  The element
// count M x D must be small enough (2^48) for the double-precision quotient to be off by one at most.
bool flat_supports(int64_t N, int64_t D, int64_t pitch_bytes, int64_t M)
{
    if (D < 1 || D > (int64_t{1} << 31) - 8192 || N > (int64_t{1} << 32) || pitch_bytes >= (int64_t{1} << 32))
        return false;
    int64_t total;
    return !__builtin_mul_overflow(M, D, &total) && total < (int64_t{1} << 48);
}

template <bool NT>
__device__ __forceinline__ void st_x4_aligned(char *p, u32x4 v)
{
    UD_GLOBAL u32x4 *g = (UD_GLOBAL u32x4 *)p;
    if constexpr (NT)
        __builtin_nontemporal_store(v, g);
    else
        *g = v;
}

// One output element (as its 16- or 32-bit pattern) from source element j of the row at `row`.
template <int DT>
__device__ __forceinline__ uint32_t load_element(const char *row, uint32_t j)
{
    if constexpr (DT == UD_F32)
        return ((const UD_GLOBAL uint32_t *)row)[j];
    else if constexpr (DT == UD_F16)
        return ((const UD_GLOBAL uint16_t *)row)[j];
    else
        return widen_half(((const UD_GLOBAL uint16_t *)row)[j]);
}

// A chunk that lies across a row end, put together from two loads: A = the last 16 output bytes' worth of
// row i, B = the first of row i+1 (NDW dwords each); the chunk is the `k` last elements of A followed by
// the first elements of B.  E16: elements are 16-bit (else 32-bit).  1 <= k < elements per load.
template <int NDW, bool E16>
__device__ __forceinline__ void splice(const uint32_t (&A)[NDW], const uint32_t (&B)[NDW], int k, uint32_t (&out)[NDW])
{
    constexpr int EPL = E16 ? 2 * NDW : NDW;            // elements per load
    const int e = EPL - k;                              // first element taken, counted in A ++ B
    const int ds = E16 ? e >> 1 : e;                    // ... in whole dwords
    uint32_t X[2 * NDW + 1];
#pragma unroll
    for (int m = 0; m < NDW; ++m) {
        X[m] = A[m];
        X[NDW + m] = B[m];
    }
    X[2 * NDW] = 0;
    uint32_t Y[NDW + 1];
#pragma unroll
    for (int m = 0; m <= NDW; ++m) {
        Y[m] = X[m];
#pragma unroll
        for (int sft = 1; sft < NDW; ++sft)
            if (ds == sft)
                Y[m] = X[m + sft];
    }
#pragma unroll
    for (int m = 0; m < NDW; ++m) {
        out[m] = Y[m];
        if constexpr (E16)
            if (e & 1)
                out[m] = (Y[m] >> 16) | (Y[m + 1] << 16);
    }
}

// Address of row r (0 <= r < N <= 2^32, pitch < 2^32: one 32 x 32 -> 64-bit multiply-add).
__device__ __forceinline__ const char *row_address(const GatherArgs &a, int64_t r, uint32_t row_bytes)
{
    const uint32_t r32 = static_cast<uint32_t>(r);
    if (a.slot) {
        const int32_t s = a.slot[r32];
        if (s >= 0)
            return a.cache + static_cast<uint64_t>(static_cast<uint32_t>(s)) * row_bytes;
    }
    return a.table + static_cast<uint64_t>(r32) * static_cast<uint32_t>(a.pitch_bytes);
}

// A chunk's elements, walked one by one across as many row ends as it meets: the general form, used
// only for rows shorter than a chunk (D < EPC), where a chunk can hold pieces of three or more rows.
template <int DT, int EPC, bool NTS>
__device__ __forceinline__ void walk_chunk(const GatherArgs &a, int64_t iq, uint32_t jq, uint32_t D, uint32_t row_bytes,
                                           char *dst)
{
    constexpr int OUT_ESZ = 16 / EPC;
    const char *row = nullptr;
#pragma unroll
    for (int q = 0; q < EPC; ++q) {
        if (q == 0 || jq == 0) {
            row = nullptr;
            if (iq >= 0 && iq < a.M) {
                const int64_t rq = load_id(a.idx, a.itype, iq);
                if (rq >= 0 && rq < a.N)
                    row = row_address(a, rq, row_bytes);
                else if (jq == 0)
                    atomicMin(a.err, static_cast<unsigned long long>(iq));
            }
        }
        if (row) {
            const uint32_t w = load_element<DT>(row, jq);
            if constexpr (OUT_ESZ == 4)
                st_scalar<NTS>(reinterpret_cast<uint32_t *>(dst) + q, w);
            else
                st_scalar<NTS>(reinterpret_cast<uint16_t *>(dst) + q, static_cast<uint16_t>(w));
        }
        if (++jq == D) {
            jq = 0;
            ++iq;
        }
    }
}

template <int DT, int P, bool NTS, bool I64>
__global__ __launch_bounds__(kBlockThreads) void gather_flat(GatherArgs a, FlatArgs f)
{
    constexpr int IN_ESZ = (DT == UD_F32) ? 4 : 2;      // table element bytes
    constexpr int OUT_ESZ = (DT == UD_F16) ? 2 : 4;     // output element bytes
    constexpr int EPC = 16 / OUT_ESZ;                   // output elements per 16-byte chunk
    constexpr uint32_t TILE = 64 * P;                   // chunks per wavefront tile
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t D = static_cast<uint32_t>(a.D);
    const uint32_t row_bytes = D * IN_ESZ;
    const int64_t wave =
        __builtin_amdgcn_readfirstlane(static_cast<int>(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6)));
    const int64_t nwaves = static_cast<int64_t>(gridDim.x) * kWavesPerBlock;

    for (int64_t t = wave; t < f.ntiles; t += nwaves) {
        // ---- per tile, the same in every lane: row i0 and column j0 of the tile's first element ----
        int64_t i0;
        uint32_t j0;
        tile_origin(f, a.D, t * (TILE * EPC), &i0, &j0);
        const int64_t left = f.nchunks - t * TILE;                   // chunks from this tile's first to the last
        const uint32_t nch_t = left < TILE ? static_cast<uint32_t>(left) : TILE;
        char *const ob = f.obase + t * (TILE * 16);

        if (D < static_cast<uint32_t>(EPC)) {                        // rows shorter than a chunk: the general walk
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const uint32_t cl = p * 64 + lane;
                if (cl >= nch_t)
                    continue;
                const uint32_t y = j0 + cl * EPC;
                const uint32_t di = y / D;
                walk_chunk<DT, EPC, NTS>(a, i0 + di, y - di * D, D, row_bytes, ob + cl * 16);
            }
            continue;
        }

        // Rows i0 + di that exist are those with lo_di <= di <= hi_di (32-bit, tile-uniform).
        uint32_t lo_di = i0 < 0 ? static_cast<uint32_t>(-i0) : 0u;
        const int64_t last = a.M - 1 - i0;
        uint32_t hi_di = last > 0x7fffffff ? 0x7fffffffu : static_cast<uint32_t>(last);
        if (last < 0) {
            lo_di = 1;
            hi_di = 0;
        }
        // ID of row i0 + di is at idp[di] (idp itself may lie before the list when i0 < 0)
        const char *const idp = static_cast<const char *>(a.idx) + i0 * (I64 ? 8 : 4);

        // From here on a chunk lies in row i alone or in rows i and i+1: its first `split` elements
        // are columns j.. of row i, the others columns 0.. of row i+1.
        constexpr int NDW = (DT == UD_F16_TO_F32) ? 2 : 4;           // dwords loaded per chunk
        uint32_t j[P], di[P];
        int split[P];           // EPC: the whole chunk is in row i
        int64_t ida[P], idb[P]; // IDs of rows i and i+1 as loaded
        bool va[P], vb[P];      // row i / row i+1 is a row of the output (and the chunk exists)
        // first all ID loads of the tile, then their uses: one round trip, not one per chunk
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const uint32_t cl = p * 64 + lane;
            const uint32_t y = j0 + cl * EPC;
            di[p] = rows_ahead<TILE * EPC>(y, D, f.rcp_d_f);
            j[p] = y - di[p] * D;
            split[p] = (D - j[p] < static_cast<uint32_t>(EPC)) ? static_cast<int>(D - j[p]) : EPC;
            ida[p] = idb[p] = 0;
            va[p] = cl < nch_t && di[p] >= lo_di && di[p] <= hi_di;
            vb[p] = split[p] < EPC && cl < nch_t && di[p] + 1 >= lo_di && di[p] + 1 <= hi_di;
            if (va[p])
                ida[p] = load_id_at<I64>(idp, di[p]);
            if (vb[p])
                idb[p] = load_id_at<I64>(idp, di[p] + 1);
        }
        const char *ra[P];      // source of row i / row i+1; null: not part of the output, or a bad ID
        const char *rb[P];
#pragma unroll
        for (int p = 0; p < P; ++p) {
            ra[p] = rb[p] = nullptr;
            if (va[p]) {
                if (static_cast<uint64_t>(ida[p]) < static_cast<uint64_t>(a.N))
                    ra[p] = row_address(a, ida[p], row_bytes);
                else if (j[p] == 0)
                    atomicMin(a.err, static_cast<unsigned long long>(i0 + di[p]));
            }
            if (vb[p]) {
                if (static_cast<uint64_t>(idb[p]) < static_cast<uint64_t>(a.N))
                    rb[p] = row_address(a, idb[p], row_bytes);
                else
                    atomicMin(a.err, static_cast<unsigned long long>(i0 + di[p] + 1));   // column 0 of row i+1 is here
            }
        }

        // Loads.  A chunk inside row i: its own bytes.  A chunk across a row end: the last chunk's worth of
        // row i and the first of row i+1 (both inside their rows since D >= EPC), spliced after the loads
        // have come back, so that such chunks add no round trip of their own.
        uint32_t va_[P][NDW], vb_[P][NDW];
#pragma unroll
        for (int p = 0; p < P; ++p) {
#pragma unroll
            for (int m = 0; m < NDW; ++m)
                va_[p][m] = vb_[p][m] = 0;
            if (ra[p]) {
                const uint32_t col = split[p] == EPC ? j[p] : D - EPC;
                const char *src = ra[p] + col * IN_ESZ;
                if constexpr (DT == UD_F32) {
                    const u32x4 v = *(const UD_GLOBAL u32x4_a4 *)src;
                    va_[p][0] = v.x, va_[p][1] = v.y, va_[p][2] = v.z, va_[p][3] = v.w;
                } else if constexpr (DT == UD_F16) {
                    const u32x4 v = *(const UD_GLOBAL u32x4_a2 *)src;
                    va_[p][0] = v.x, va_[p][1] = v.y, va_[p][2] = v.z, va_[p][3] = v.w;
                } else {
                    const u32x2 v = *(const UD_GLOBAL u32x2_a2 *)src;
                    va_[p][0] = v.x, va_[p][1] = v.y;
                }
            }
            if (rb[p]) {
                if constexpr (DT == UD_F32) {
                    const u32x4 v = *(const UD_GLOBAL u32x4_a4 *)rb[p];
                    vb_[p][0] = v.x, vb_[p][1] = v.y, vb_[p][2] = v.z, vb_[p][3] = v.w;
                } else if constexpr (DT == UD_F16) {
                    const u32x4 v = *(const UD_GLOBAL u32x4_a2 *)rb[p];
                    vb_[p][0] = v.x, vb_[p][1] = v.y, vb_[p][2] = v.z, vb_[p][3] = v.w;
                } else {
                    const u32x2 v = *(const UD_GLOBAL u32x2_a2 *)rb[p];
                    vb_[p][0] = v.x, vb_[p][1] = v.y;
                }
            }
        }

        // Wait for the loads here, once and in straight-line code.  Left to the compiler, the wait lands
        // inside the first conditional block that uses a loaded value, is then needed again after
        // every later branch, and there it also waits for the stores issued in between.
        // (vmcnt = 0; expcnt and lgkmcnt fields left at their maxima.)
        __builtin_amdgcn_s_waitcnt(0x0F70);

        // All register work first (splicing, widening), then the full stores back to back, then the
        // rare partial ones.
        u32x4 v[P];
        bool full[P], part[P];
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const uint32_t cl = p * 64 + lane;
            uint32_t c[NDW];
#pragma unroll
            for (int m = 0; m < NDW; ++m)
                c[m] = va_[p][m];
            if (split[p] < EPC)
                splice<NDW, IN_ESZ == 2>(va_[p], vb_[p], split[p], c);
            if constexpr (DT == UD_F16_TO_F32)
                v[p] = u32x4{widen_half(c[0] & 0xffffu), widen_half(c[0] >> 16), widen_half(c[1] & 0xffffu), widen_half(c[1] >> 16)};
            else
                v[p] = u32x4{c[0], c[1], c[2], c[3]};
            const bool have_a = ra[p] != nullptr, have_b = split[p] == EPC || rb[p] != nullptr;
            full[p] = cl < nch_t && have_a && have_b;
            part[p] = cl < nch_t && !full[p] && (have_a || rb[p] != nullptr);
        }
#pragma unroll
        for (int p = 0; p < P; ++p)
            if (full[p])
                st_x4_aligned<NTS>(ob + (p * 64 + lane) * 16, v[p]);
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if (!part[p])
                continue;
            // one of the two rows is outside the output or has a bad ID: store the other row's elements only
            char *dst = ob + (p * 64 + lane) * 16;
            const uint32_t w4[4] = {v[p].x, v[p].y, v[p].z, v[p].w};
#pragma unroll
            for (int q = 0; q < EPC; ++q) {
                if (!(q < split[p] ? ra[p] != nullptr : rb[p] != nullptr))
                    continue;
                if constexpr (OUT_ESZ == 4)
                    st_scalar<NTS>(reinterpret_cast<uint32_t *>(dst) + q, w4[q & 3]);
                else
                    st_scalar<NTS>(reinterpret_cast<uint16_t *>(dst) + q, static_cast<uint16_t>(w4[q >> 1] >> ((q & 1) * 16)));
            }
        }
    }
}

template <int DT, int P, bool I64>
static hipError_t launch_flat_i(const GatherArgs &a, const FlatArgs &f, const Plan &p, dim3 grid, hipStream_t s)
{
    if (p.flags & UD_TUNE_NT_STORE)
        hipLaunchKernelGGL((gather_flat<DT, P, true, I64>), grid, dim3(kBlockThreads), 0, s, a, f);
    else
        hipLaunchKernelGGL((gather_flat<DT, P, false, I64>), grid, dim3(kBlockThreads), 0, s, a, f);
    return hipGetLastError();
}

template <int DT, int P>
static hipError_t launch_flat_p(const GatherArgs &a, const FlatArgs &f, const Plan &p, dim3 grid, hipStream_t s)
{
    return a.itype == UD_I64 ? launch_flat_i<DT, P, true>(a, f, p, grid, s) : launch_flat_i<DT, P, false>(a, f, p, grid, s);
}

template <int DT>
static hipError_t launch_flat_dt(const GatherArgs &a, const Plan &p, hipStream_t s)
{
    constexpr int OUT_ESZ = (DT == UD_F16) ? 2 : 4;
    const int P = p.chunks_per_lane;
    if (P != 1 && P != 2 && P != 4)
        return hipErrorInvalidValue;
    const FlatArgs f = make_flat_args(a.out, a.M, a.D, OUT_ESZ, P);
    int64_t blocks = (f.ntiles + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > p.max_blocks)
        blocks = p.max_blocks;
    if (blocks > (1 << 24))
        blocks = 1 << 24;                  // the kernel numbers its wavefronts in 32 bits; it strides beyond
    if (blocks < 1)
        return hipSuccess;
    const dim3 grid(static_cast<unsigned>(blocks));
    switch (P) {
    case 1: return launch_flat_p<DT, 1>(a, f, p, grid, s);
    case 2: return launch_flat_p<DT, 2>(a, f, p, grid, s);
    default: return launch_flat_p<DT, 4>(a, f, p, grid, s);
    }
}

hipError_t launch_flat(const GatherArgs &a, int dtype, const Plan &p, hipStream_t s)
{
    if (!flat_supports(a.N, a.D, a.pitch_bytes, a.M))
        return hipErrorInvalidValue;
    switch (dtype) {
    case UD_F32: return launch_flat_dt<UD_F32>(a, p, s);
    case UD_F16: return launch_flat_dt<UD_F16>(a, p, s);
    case UD_F16_TO_F32: return launch_flat_dt<UD_F16_TO_F32>(a, p, s);
    default: return hipErrorInvalidValue;
    }
}

} // namespace ud
