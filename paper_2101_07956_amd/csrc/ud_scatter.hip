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
// and tail chunks only the row's own elements are stored (masked, unrolled
// element stores of the chunk that was loaded whole).  The source rows (dense,
// in HBM) generally have another alignment and are read with loads that are
// only element-aligned.
#include "ud_flat.hpp"

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

// ESZ: element bytes (4 or 2).  U rows in flight per lane group, P chunks per
// lane per row, lg = log2(lanes per row).  a.table is the destination, a.out
// the dense source (reusing GatherArgs: `out` is read, `table` written).
// I64: the ID type, fixed at compile time so that the ID loads of the U rows are
// plain loads issued together (a run-time choice puts each in a branch, and
// they then wait for one another).  The phases -- IDs, source loads, one wait,
// full stores, partial stores -- are kept apart for the same reason: a wait
// placed inside a conditional block by the compiler has to be repeated after
// every later branch, where it also waits for the stores issued so far.
template <int ESZ, int U, int P, bool I64>
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
        int64_t i[U], r[U];
        char *base[U];   // 16-byte aligned address at or below the destination row's first byte
        int head[U];
        int64_t nch[U];
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
            base[u] = table;
            head[u] = 0;
            if (i[u] < a.M) {
                if (r[u] < 0 || r[u] >= a.N) {
                    if (l == 0)
                        atomicMin(a.err, static_cast<unsigned long long>(i[u]));
                } else {
                    char *dst = table + r[u] * a.pitch_bytes;
                    head[u] = static_cast<int>(reinterpret_cast<uintptr_t>(dst) & 15u);
                    base[u] = dst - head[u];
                    nch[u] = (head[u] + row_bytes + 15) >> 4;
                }
            }
        }
        for (int64_t cb = 0; cb < nch_bound; cb += span) {
            uint32_t w[U][P][4];         // scalars, not vectors: conditionally assigned vectors end up copied around
            int lo[U][P], hi[U][P];      // elements of the chunk that belong to the row; lo >= hi: no chunk
            bool edge[U][P];             // the chunk hangs over an end of the whole source: copied element by element
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    const int64_t c = cb + static_cast<int64_t>(p) * lpr + l;
                    const int64_t e0 = c * EPC - head[u] / ESZ;   // first element of the chunk, relative to the row
                    const int64_t left = a.D - e0;
                    lo[u][p] = e0 < 0 ? static_cast<int>(-e0) : 0;
                    hi[u][p] = c < nch[u] ? (left < EPC ? static_cast<int>(left) : EPC) : 0;
                    // A head or tail chunk is loaded whole like any other: what it reads beyond the row are
                    // elements of the neighbouring source rows.  Only where those 16 bytes would begin before
                    // the first or end after the last source element (the first and last rows of a launch;
                    // with rows shorter than a chunk, their neighbours too) is the chunk copied element by
                    // element instead.
                    const int64_t s0 = i[u] * a.D + e0;           // first source element the whole-chunk load reads
                    edge[u][p] = s0 < 0 || s0 + EPC > a.M * a.D;
                    w[u][p][0] = w[u][p][1] = w[u][p][2] = w[u][p][3] = 0;
                    if (lo[u][p] < hi[u][p] && !edge[u][p]) {
                        const u32x4 t = ld_src_chunk<ESZ>(src + (i[u] * a.D + e0) * ESZ);
                        w[u][p][0] = t.x, w[u][p][1] = t.y, w[u][p][2] = t.z, w[u][p][3] = t.w;
                    }
                }
            }
            __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): all source loads, once, outside the branches
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    const int64_t c = cb + static_cast<int64_t>(p) * lpr + l;
                    if (lo[u][p] == 0 && hi[u][p] == EPC)
                        *(UD_GLOBAL u32x4 *)(base[u] + c * 16) = u32x4{w[u][p][0], w[u][p][1], w[u][p][2], w[u][p][3]};
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    if (lo[u][p] >= hi[u][p] || (lo[u][p] == 0 && hi[u][p] == EPC))
                        continue;
                    // head or tail chunk: only the elements that belong to the row
                    const int64_t c = cb + static_cast<int64_t>(p) * lpr + l;
                    char *d16 = base[u] + c * 16;
                    if (edge[u][p]) {
                        const int64_t e0 = c * EPC - head[u] / ESZ;
                        const char *s16 = src + (i[u] * a.D + e0) * ESZ;
                        for (int q = lo[u][p]; q < hi[u][p]; ++q) {
                            if constexpr (ESZ == 4)
                                ((UD_GLOBAL uint32_t *)d16)[q] = ((const UD_GLOBAL uint32_t *)s16)[q];
                            else
                                ((UD_GLOBAL uint16_t *)d16)[q] = ((const UD_GLOBAL uint16_t *)s16)[q];
                        }
                        continue;
                    }
                    if constexpr (ESZ == 4) {
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            if (q >= lo[u][p] && q < hi[u][p])
                                ((UD_GLOBAL uint32_t *)d16)[q] = w[u][p][q];
                    } else {
#pragma unroll
                        for (int q = 0; q < 8; ++q)
                            if (q >= lo[u][p] && q < hi[u][p])
                                ((UD_GLOBAL uint16_t *)d16)[q] = static_cast<uint16_t>(w[u][p][q >> 1] >> ((q & 1) * 16));
                    }
                }
            }
        }
    }
}

template <int ESZ, int U, int P>
static hipError_t launch_scatter_up(const GatherArgs &a, int lg, dim3 grid, hipStream_t s)
{
    if (a.itype == UD_I64)
        hipLaunchKernelGGL((scatter_chunked<ESZ, U, P, true>), grid, dim3(kBlockThreads), 0, s, a, lg);
    else
        hipLaunchKernelGGL((scatter_chunked<ESZ, U, P, false>), grid, dim3(kBlockThreads), 0, s, a, lg);
    return hipGetLastError();
}

template <int ESZ>
static hipError_t launch_scatter_esz(const GatherArgs &a, const Plan &p, int lg, dim3 grid, hipStream_t s)
{
    const int key = p.rows_in_flight * 10 + p.chunks_per_lane;
    switch (key) {
#define UD_CASE(U_, P_) \
    case U_ * 10 + P_:  \
        return launch_scatter_up<ESZ, U_, P_>(a, lg, grid, s);
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

// ---------------------------------------------------------------------------------------------------------------
// Source-aligned scatter, for tables in HBM.  There the scatter is a copy bound by HBM bandwidth, and the
// row-per-lane-group kernel above leaves lanes idle wherever a row's chunk count is no power of two (25 of
// 32 lanes busy at 400-byte rows, 151 of 192 chunk slots at 2408 bytes).  Here the dense SOURCE [M, D] is
// taken as one stream of aligned 16-byte chunks: every lane of every wavefront moves one chunk per pass with
// an aligned load, finds the row and column the chunk starts at, and stores it into the table row with a
// store that is only element-aligned.  A chunk that lies across a source row end goes out as element
// stores into the two destination rows.  (For tables behind the host link the kernel above stays the
// choice: there the shape of the write requests matters, and it writes whole aligned chunks.)
// ---------------------------------------------------------------------------------------------------------------
template <int ESZ, int P, bool I64, bool NTS>
__global__ __launch_bounds__(kBlockThreads) void scatter_flat(GatherArgs a, FlatArgs f)
{
    constexpr int EPC = 16 / ESZ;
    constexpr uint32_t TILE = 64 * P;
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t D = static_cast<uint32_t>(a.D);
    char *const table = const_cast<char *>(a.table);
    const uint32_t pitch = static_cast<uint32_t>(a.pitch_bytes);
    const int64_t wave =
        __builtin_amdgcn_readfirstlane(static_cast<int>(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6)));
    const int64_t nwaves = static_cast<int64_t>(gridDim.x) * kWavesPerBlock;

    for (int64_t t = wave; t < f.ntiles; t += nwaves) {
        int64_t i0;
        uint32_t j0;
        tile_origin(f, a.D, t * (TILE * EPC), &i0, &j0);
        const int64_t left = f.nchunks - t * TILE;
        const uint32_t nch_t = left < TILE ? static_cast<uint32_t>(left) : TILE;
        const char *const sb = f.obase + t * (TILE * 16);            // this tile's first source chunk

        if (D < static_cast<uint32_t>(EPC)) {
            // rows shorter than a chunk: element by element, a chunk may hold pieces of several rows
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const uint32_t cl = p * 64 + lane;
                if (cl >= nch_t)
                    continue;
                const uint32_t y = j0 + cl * EPC;
                const uint32_t di = y / D;
                int64_t iq = i0 + di;
                uint32_t jq = y - di * D;
                char *row = nullptr;
                for (int q = 0; q < EPC; ++q) {
                    if (q == 0 || jq == 0) {
                        row = nullptr;
                        if (iq >= 0 && iq < a.M) {
                            const int64_t rq = load_id(a.idx, a.itype, iq);
                            if (rq >= 0 && rq < a.N)
                                row = table + rq * a.pitch_bytes;
                            else if (jq == 0)
                                atomicMin(a.err, static_cast<unsigned long long>(iq));
                        }
                    }
                    if (row) {
                        if constexpr (ESZ == 4)
                            ((UD_GLOBAL uint32_t *)row)[jq] = ((const UD_GLOBAL uint32_t *)(sb + cl * 16))[q];
                        else
                            ((UD_GLOBAL uint16_t *)row)[jq] = ((const UD_GLOBAL uint16_t *)(sb + cl * 16))[q];
                    }
                    if (++jq == D) {
                        jq = 0;
                        ++iq;
                    }
                }
            }
            continue;
        }

        uint32_t lo_di = i0 < 0 ? static_cast<uint32_t>(-i0) : 0u;
        const int64_t last = a.M - 1 - i0;
        uint32_t hi_di = last > 0x7fffffff ? 0x7fffffffu : static_cast<uint32_t>(last);
        if (last < 0) {
            lo_di = 1;
            hi_di = 0;
        }
        const char *const idp = static_cast<const char *>(a.idx) + i0 * (I64 ? 8 : 4);

        uint32_t j[P], di[P];
        int split[P];
        int64_t ida[P], idb[P];
        bool va[P], vb[P];
        uint32_t w[P][4];           // the source chunk (read only where the chunk exists)
        // all loads first: the IDs of the rows involved and the source chunks themselves, which do not depend on them
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
            if (cl < nch_t) {
                // aligned, and it overlaps the source: the bytes of it that lie outside are in a page the source occupies
                const u32x4 v = ld_chunk(sb + cl * 16);
                w[p][0] = v.x, w[p][1] = v.y, w[p][2] = v.z, w[p][3] = v.w;
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0), once, in straight-line code
        char *ra[P];
        char *rb[P];
#pragma unroll
        for (int p = 0; p < P; ++p) {
            ra[p] = rb[p] = nullptr;
            if (va[p]) {
                if (static_cast<uint64_t>(ida[p]) < static_cast<uint64_t>(a.N))
                    ra[p] = table + static_cast<uint64_t>(static_cast<uint32_t>(ida[p])) * pitch;
                else if (j[p] == 0)
                    atomicMin(a.err, static_cast<unsigned long long>(i0 + di[p]));
            }
            if (vb[p]) {
                if (static_cast<uint64_t>(idb[p]) < static_cast<uint64_t>(a.N))
                    rb[p] = table + static_cast<uint64_t>(static_cast<uint32_t>(idb[p])) * pitch;
                else
                    atomicMin(a.err, static_cast<unsigned long long>(i0 + di[p] + 1));
            }
        }
        // whole chunks, back to back
#pragma unroll
        for (int p = 0; p < P; ++p)
            if (split[p] == EPC && ra[p]) {
                char *d = ra[p] + j[p] * ESZ;
                const u32x4 v = u32x4{w[p][0], w[p][1], w[p][2], w[p][3]};
                if constexpr (ESZ == 4) {
                    if constexpr (NTS)
                        __builtin_nontemporal_store(v, (UD_GLOBAL u32x4_a4 *)d);
                    else
                        *(UD_GLOBAL u32x4_a4 *)d = v;
                } else {
                    if constexpr (NTS)
                        __builtin_nontemporal_store(v, (UD_GLOBAL u32x4_a2 *)d);
                    else
                        *(UD_GLOBAL u32x4_a2 *)d = v;
                }
            }
        // chunks across a source row end: their elements go to two table rows
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if (split[p] == EPC || (!ra[p] && !rb[p]))
                continue;
#pragma unroll
            for (int q = 0; q < EPC; ++q) {
                char *row = q < split[p] ? ra[p] : rb[p];
                const uint32_t col = q < split[p] ? j[p] + q : static_cast<uint32_t>(q - split[p]);
                if (!row)
                    continue;
                if constexpr (ESZ == 4)
                    ((UD_GLOBAL uint32_t *)row)[col] = w[p][q];
                else
                    ((UD_GLOBAL uint16_t *)row)[col] = static_cast<uint16_t>(w[p][q >> 1] >> ((q & 1) * 16));
            }
        }
    }
}

template <int ESZ, int P>
static hipError_t launch_scatter_flat_p(const GatherArgs &a, const FlatArgs &f, bool nts, dim3 grid, hipStream_t s)
{
    const bool i64 = a.itype == UD_I64;
    if (i64 && nts)
        hipLaunchKernelGGL((scatter_flat<ESZ, P, true, true>), grid, dim3(kBlockThreads), 0, s, a, f);
    else if (i64)
        hipLaunchKernelGGL((scatter_flat<ESZ, P, true, false>), grid, dim3(kBlockThreads), 0, s, a, f);
    else if (nts)
        hipLaunchKernelGGL((scatter_flat<ESZ, P, false, true>), grid, dim3(kBlockThreads), 0, s, a, f);
    else
        hipLaunchKernelGGL((scatter_flat<ESZ, P, false, false>), grid, dim3(kBlockThreads), 0, s, a, f);
    return hipGetLastError();
}

hipError_t launch_scatter_flat(const GatherArgs &a, int elem_bytes, const Plan &p, hipStream_t s)
{
    const int P = p.chunks_per_lane;
    if ((P != 1 && P != 2 && P != 4) || !flat_supports(a.N, a.D, a.pitch_bytes, a.M))
        return hipErrorInvalidValue;
    const FlatArgs f = make_flat_args(a.out, a.M, a.D, elem_bytes, P);      // a.out is the dense source
    int64_t blocks = (f.ntiles + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > p.max_blocks)
        blocks = p.max_blocks;
    if (blocks > (1 << 24))
        blocks = 1 << 24;
    if (blocks < 1)
        return hipSuccess;
    const dim3 grid(static_cast<unsigned>(blocks));
    const bool nts = p.flags & UD_TUNE_NT_STORE;
    if (elem_bytes == 4) {
        switch (P) {
        case 1: return launch_scatter_flat_p<4, 1>(a, f, nts, grid, s);
        case 2: return launch_scatter_flat_p<4, 2>(a, f, nts, grid, s);
        default: return launch_scatter_flat_p<4, 4>(a, f, nts, grid, s);
        }
    }
    switch (P) {
    case 1: return launch_scatter_flat_p<2, 1>(a, f, nts, grid, s);
    case 2: return launch_scatter_flat_p<2, 2>(a, f, nts, grid, s);
    default: return launch_scatter_flat_p<2, 4>(a, f, nts, grid, s);
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
