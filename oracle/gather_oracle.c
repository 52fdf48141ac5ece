/*
 * CPU oracle for the feature-row gather  out[i,:] = table[idx[i],:].
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It is built by the host C compiler alone,
 * includes no HIP header and shares no code, table or helper with the GPU
 * path.  Only tests, the smoke check and the benchmark's cpu_baseline leg may
 * load it; the product path never does.
 *
 * What it follows (PyTorch-Direct, arXiv 2101.07956):
 *   - Section 2.2: the features form a 2-D array whose row index is the node ID
 *     and whose columns are that node's features.
 *   - Listings 1 and 2 (Section 4.1): a minibatch tensor is
 *     features[neighbor_id], one output row per entry of the ID list.
 *   - Section 4.5: whatever access order the GPU uses, output ordering is kept,
 *     i.e. output row i always corresponds to entry i of the ID list.
 * The method reaches this definition exactly, so the oracle is the definition
 * written out: one element at a time, 64-bit index arithmetic, a single
 * thread, no blocking and no row-wise memcpy.
 *
 * Readings where the paper is silent: the ID list may be int64 or int32;
 * negative or >= N entries are rejected (never wrapped) and nothing is written
 * when any entry is bad; duplicates are allowed; M == 0 is a valid no-op.
 * The half -> single widening is an addition of this library (the paper never
 * states a precision): the exact IEEE-754 binary16 -> binary32 conversion with
 * signalling NaNs quieted (convertFormat semantics).
 *
 * Every function here is pinned by tests that do not go through this file:
 * brute force on tiny shapes, numpy.take, closed-form tag tables, the
 * hardware F16C converter, textbook binary16 values and the request counts
 * printed with Figures 4 and 5.  Nothing is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_F16 = 1, ORACLE_F16_TO_F32 = 2 };
enum { ORACLE_I64 = 0, ORACLE_I32 = 1 };
enum { ORACLE_OK = 0, ORACLE_ERR_INVALID_ARG = 1, ORACLE_ERR_INDEX = 4 };

/*
 * Exact binary16 -> binary32 widening, by value.
 * A binary16 pattern s|eeeee|ffffffffff denotes
 *     e == 0        : (-1)^s * f * 2^-24              (zero and subnormals)
 *     1 <= e <= 30  : (-1)^s * (1024 + f) * 2^(e-25)  (normals)
 *     e == 31, f==0 : (-1)^s * infinity
 *     e == 31, f!=0 : NaN
 * Every finite binary16 value is representable in binary32, so computing the
 * value in double and narrowing to float is exact.  NaN keeps its sign and its
 * 10 payload bits (moved to the top of the 23-bit fraction) and comes out
 * quiet: fraction bit 22 is set.
 */
uint32_t oracle_f16_bits_to_f32_bits(uint16_t h)
{
    const uint32_t s = (uint32_t)(h >> 15) & 1u;
    const uint32_t e = (uint32_t)(h >> 10) & 0x1fu;
    const uint32_t f = (uint32_t)h & 0x3ffu;
    uint32_t bits;

    if (e == 31u) {
        if (f == 0u)
            bits = 0x7f800000u;                       /* infinity */
        else
            bits = 0x7f800000u | 0x00400000u | (f << 13); /* quiet NaN, payload kept */
        return bits | (s << 31);
    }

    double v;
    if (e == 0u)
        v = ldexp((double)f, -24);
    else
        v = ldexp((double)(1024u + f), (int)e - 25);
    float fl = (float)v;                               /* exact */
    memcpy(&bits, &fl, sizeof bits);
    return bits | (s << 31);                           /* sign last, so -0 survives */
}

static int64_t read_index(const void *idx, int itype, int64_t i)
{
    if (itype == ORACLE_I64)
        return ((const int64_t *)idx)[i];
    return (int64_t)((const int32_t *)idx)[i];
}

/*
 * out[i*D + j] = conv(table[idx[i]*D + j])   for 0 <= i < M, 0 <= j < D.
 *
 * dtype ORACLE_F32        : table and out hold 32-bit patterns, conv = identity
 * dtype ORACLE_F16        : table and out hold 16-bit patterns, conv = identity
 * dtype ORACLE_F16_TO_F32 : table holds 16-bit, out 32-bit, conv = widening
 * Bit patterns are copied as integers, so NaN payloads and -0 pass unchanged.
 *
 * All M entries of idx are checked before anything is written.  If entry i is
 * the first one outside [0, N), *bad_pos = i, ORACLE_ERR_INDEX is returned and
 * out is untouched.  Otherwise *bad_pos = -1.
 */
int oracle_gather_pitched(const void *table, int64_t N, int64_t D, int64_t pitch, int dtype,
                          const void *idx, int itype, int64_t M,
                          void *out, int64_t *bad_pos);

int oracle_gather(const void *table, int64_t N, int64_t D, int dtype,
                  const void *idx, int itype, int64_t M,
                  void *out, int64_t *bad_pos)
{
    return oracle_gather_pitched(table, N, D, D, dtype, idx, itype, M, out, bad_pos);
}

/*
 * The same gather from a table whose rows are `pitch` elements apart
 * (pitch >= D; elements D..pitch-1 of every row are padding and never read):
 *     out[i*D + j] = conv(table[idx[i]*pitch + j]).
 * The output stays dense.  pitch == D is the paper's plain 2-D array.
 */
int oracle_gather_pitched(const void *table, int64_t N, int64_t D, int64_t pitch, int dtype,
                          const void *idx, int itype, int64_t M,
                          void *out, int64_t *bad_pos)
{
    if (bad_pos)
        *bad_pos = -1;
    if (N < 1 || D < 1 || M < 0 || pitch < D)
        return ORACLE_ERR_INVALID_ARG;
    if (dtype != ORACLE_F32 && dtype != ORACLE_F16 && dtype != ORACLE_F16_TO_F32)
        return ORACLE_ERR_INVALID_ARG;
    if (itype != ORACLE_I64 && itype != ORACLE_I32)
        return ORACLE_ERR_INVALID_ARG;
    if (M == 0)
        return ORACLE_OK;
    if (!table || !idx || !out)
        return ORACLE_ERR_INVALID_ARG;

    for (int64_t i = 0; i < M; ++i) {
        const int64_t r = read_index(idx, itype, i);
        if (r < 0 || r >= N) {
            if (bad_pos)
                *bad_pos = i;
            return ORACLE_ERR_INDEX;
        }
    }

    for (int64_t i = 0; i < M; ++i) {
        const int64_t r = read_index(idx, itype, i);
        for (int64_t j = 0; j < D; ++j) {
            const int64_t src = r * pitch + j;
            const int64_t dst = i * D + j;
            if (dtype == ORACLE_F32)
                ((uint32_t *)out)[dst] = ((const uint32_t *)table)[src];
            else if (dtype == ORACLE_F16)
                ((uint16_t *)out)[dst] = ((const uint16_t *)table)[src];
            else
                ((uint32_t *)out)[dst] =
                    oracle_f16_bits_to_f32_bits(((const uint16_t *)table)[src]);
        }
    }
    return ORACLE_OK;
}

/*
 * Access-count model of Section 4.5 (Figures 4 and 5).
 *
 * The stock indexing kernel gives one thread to each output element: thread
 * g = i*D + j serves element j of output row i, threads are grouped into warps
 * of W consecutive threads, and every distinct memory line of line_bytes that
 * one warp touches costs one request on the link.  With a per-row circular
 * shift s_i the thread reads (and writes) element (j + s_i) mod D instead.
 * The count returned is the number of distinct (warp, line) pairs over the
 * output rows [row_lo, row_hi).
 *
 * rows[i] is the table row read for output row i, shift[i] its circular shift
 * (NULL = no shift, the unmodified kernel), elem_bytes the element size.
 * Returns -1 on invalid arguments.
 */
int64_t oracle_count_requests(const int64_t *rows, const int64_t *shift,
                              int64_t M, int64_t D, int64_t elem_bytes,
                              int64_t W, int64_t line_bytes,
                              int64_t row_lo, int64_t row_hi)
{
    if (!rows || M < 0 || D < 1 || elem_bytes < 1 || W < 1 || line_bytes < 1)
        return -1;
    if (row_lo < 0 || row_hi > M || row_lo > row_hi)
        return -1;
    const int64_t n = (row_hi - row_lo) * D;
    if (n == 0)
        return 0;
    int64_t *warp = (int64_t *)malloc((size_t)n * sizeof *warp);
    int64_t *line = (int64_t *)malloc((size_t)n * sizeof *line);
    if (!warp || !line) {
        free(warp);
        free(line);
        return -1;
    }
    int64_t t = 0;
    for (int64_t i = row_lo; i < row_hi; ++i) {
        const int64_t s = shift ? shift[i] : 0;
        for (int64_t j = 0; j < D; ++j, ++t) {
            const int64_t g = i * D + j;
            const int64_t k = (((j + s) % D) + D) % D;
            warp[t] = g / W;
            line[t] = ((rows[i] * D + k) * elem_bytes) / line_bytes;
        }
    }
    int64_t distinct = 0;
    for (int64_t a = 0; a < n; ++a) {
        int seen = 0;
        for (int64_t b = 0; b < a && !seen; ++b)
            seen = (warp[b] == warp[a] && line[b] == line[a]);
        distinct += !seen;
    }
    free(warp);
    free(line);
    return distinct;
}

/*
 * The shift of Section 4.5: the offset that makes thread g = i*D + j read an
 * element whose position within its memory line equals the thread's position
 * within its warp, when one warp spans exactly one line (W * elem_bytes ==
 * line_bytes).  Element addresses are r*D + k, thread numbers i*D + j, so
 * k = j + (i - r)*D modulo the number of elements per line.
 */
int64_t oracle_circular_shift(int64_t i, int64_t r, int64_t D, int64_t elems_per_line)
{
    if (elems_per_line < 1)
        return -1;
    int64_t s = ((i - r) * D) % elems_per_line;
    if (s < 0)
        s += elems_per_line;
    return s;
}

/*
 * Write direction: table[idx[i]*D + j] = src[i*D + j]  for 0 <= i < M, 0 <= j < D,
 * applied in the order i = 0, 1, ..., so with duplicate IDs the last occurrence
 * wins.  The paper states (Section 3) that GPU threads can issue both read and
 * write requests to host memory; this is the gather's mirror image, needed
 * e.g. to update rows of a host-resident table.  Bit patterns are copied; dtype
 * is ORACLE_F32 (4-byte elements) or ORACLE_F16 (2-byte elements).
 * All IDs are checked before anything is written; on a bad ID *bad_pos is its
 * first position, ORACLE_ERR_INDEX is returned and the table is untouched.
 */
int oracle_scatter_pitched(void *table, int64_t N, int64_t D, int64_t pitch, int dtype,
                           const void *idx, int itype, int64_t M,
                           const void *src, int64_t *bad_pos);

int oracle_scatter(void *table, int64_t N, int64_t D, int dtype,
                   const void *idx, int itype, int64_t M,
                   const void *src, int64_t *bad_pos)
{
    return oracle_scatter_pitched(table, N, D, D, dtype, idx, itype, M, src, bad_pos);
}

/* The same with table rows `pitch` elements apart (pitch >= D): table[idx[i]*pitch + j] = src[i*D + j];
 * the padding elements D..pitch-1 of every row are never written. */
int oracle_scatter_pitched(void *table, int64_t N, int64_t D, int64_t pitch, int dtype,
                           const void *idx, int itype, int64_t M,
                           const void *src, int64_t *bad_pos)
{
    if (bad_pos)
        *bad_pos = -1;
    if (N < 1 || D < 1 || M < 0 || pitch < D)
        return ORACLE_ERR_INVALID_ARG;
    if (dtype != ORACLE_F32 && dtype != ORACLE_F16)
        return ORACLE_ERR_INVALID_ARG;
    if (itype != ORACLE_I64 && itype != ORACLE_I32)
        return ORACLE_ERR_INVALID_ARG;
    if (M == 0)
        return ORACLE_OK;
    if (!table || !idx || !src)
        return ORACLE_ERR_INVALID_ARG;

    for (int64_t i = 0; i < M; ++i) {
        const int64_t r = read_index(idx, itype, i);
        if (r < 0 || r >= N) {
            if (bad_pos)
                *bad_pos = i;
            return ORACLE_ERR_INDEX;
        }
    }
    for (int64_t i = 0; i < M; ++i) {
        const int64_t r = read_index(idx, itype, i);
        for (int64_t j = 0; j < D; ++j) {
            if (dtype == ORACLE_F32)
                ((uint32_t *)table)[r * pitch + j] = ((const uint32_t *)src)[i * D + j];
            else
                ((uint16_t *)table)[r * pitch + j] = ((const uint16_t *)src)[i * D + j];
        }
    }
    return ORACLE_OK;
}
