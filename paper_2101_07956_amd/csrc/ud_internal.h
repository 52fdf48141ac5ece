// Internal interface between the C-ABI boundary and the gfx950 kernel launchers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ud.h"

namespace ud {

// Sentinel held by a device error slot while no bad ID has been seen.
constexpr unsigned long long kNoBadIndex = 0x7fffffffffffffffull;

struct GatherArgs {
    const char *table;       // device pointer to row 0
    int64_t N, D;
    int64_t pitch_bytes;     // distance between table rows in bytes (>= D * element size)
    const void *idx;         // device pointer, M entries
    int itype;               // UD_I64 / UD_I32
    int64_t M;
    void *out;               // device pointer, M x D output elements
    unsigned long long *err; // device error slot of the launch stream (atomic min of bad positions)
    // hot-row cache (both null when unused): slot[r] >= 0 means row r is read
    // from cache + slot[r] * row_bytes (HBM) instead of table + r * row_bytes
    const int32_t *slot;
    const char *cache;
    int group_iters;         // consecutive row batches one workgroup serves before it strides on (>= 1)
};

// Resolved kernel parameters (every field concrete, see ud_tuning).
struct Plan {
    int lanes_per_row;   // power of two, 1..64
    int chunks_per_lane; // 1..4
    int rows_in_flight;  // 1, 2, 4
    int max_blocks;      // > 0
    unsigned flags;      // UD_TUNE_*
    bool tile_id_lines;  // chunked kernel: a workgroup serves runs of rows that share a line of the ID list
};

// Wavefronts per workgroup used by every kernel here.
constexpr int kWavesPerBlock = 4;
constexpr int kBlockThreads = 64 * kWavesPerBlock;

// Enqueue the chunked (row-per-lane-group, source-aligned) gather.  Returns
// hipErrorInvalidValue if (dtype, plan) has no instantiation.
hipError_t launch_chunked_f32(const GatherArgs &a, const Plan &p, hipStream_t s);
hipError_t launch_chunked_f16(const GatherArgs &a, const Plan &p, hipStream_t s);
hipError_t launch_chunked_f16_to_f32(const GatherArgs &a, const Plan &p, hipStream_t s);

// Enqueue the destination-aligned gather (the output seen as one stream of
// 16-byte chunks).  Uses p.chunks_per_lane (1, 2 or 4), p.max_blocks and the
// UD_TUNE_NT_STORE bit.  Returns hipErrorInvalidValue if there is no instantiation
// or the shape is outside what its 32-bit arithmetic covers (see flat_supports).
hipError_t launch_flat(const GatherArgs &a, int dtype, const Plan &p, hipStream_t s);
bool flat_supports(int64_t N, int64_t D, int64_t pitch_bytes, int64_t M);

// slot[rows[k]] = k for k < n (building a hot-row cache's map).
hipError_t launch_fill_slots(const int64_t *rows, int64_t n, int32_t *slot, hipStream_t s);

// Enqueue the chunked scatter table[idx[i], :] = src[i, :]; a.out is the dense
// source, a.table the destination.  elem_bytes is 4 or 2.
hipError_t launch_scatter(const GatherArgs &a, int elem_bytes, const Plan &p, hipStream_t s);

// Enqueue the source-aligned scatter (the dense source seen as one stream of 16-byte chunks): p.chunks_per_lane
// (1, 2 or 4) and p.max_blocks.  hipErrorInvalidValue outside what flat_supports covers.
hipError_t launch_scatter_flat(const GatherArgs &a, int elem_bytes, const Plan &p, hipStream_t s);

// Enqueue the one-lane-per-element gather.
hipError_t launch_elementwise(const GatherArgs &a, int dtype, const Plan &p, hipStream_t s);

// *result = the slot's value, and the slot is cleared, in one atomic step, in stream order.
hipError_t launch_fetch_and_reset(unsigned long long *slot, unsigned long long *result, hipStream_t s);
// words[k] = kNoBadIndex for k < n (a fill kernel: no memset node, so callers may capture it).
hipError_t launch_init_slots(unsigned long long *words, int n, hipStream_t s);

} // namespace ud
