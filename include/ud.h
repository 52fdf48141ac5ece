/*
 * ud.h -- C ABI of the GPU-centric feature-row gather for AMD MI355X (gfx950).
 *
 * The operation is the one PyTorch-Direct (arXiv 2101.07956) builds its case
 * on: a 2-D feature array whose row index is the node ID (Section 2.2) stays in
 * host memory that the GPU can dereference directly (Section 3, Figure 2b;
 * Section 4.1), and a minibatch tensor features[neighbor_id] (Listings 1-2) is
 * produced by GPU threads reading the selected rows over the host link and
 * writing them, in ID-list order (Section 4.5), to a dense tensor in GPU
 * memory.  No CPU gather, no staging buffer, no DMA call.
 *
 * Conventions for every call
 *   - returns a ud_status; UD_OK is 0.  Output arguments are written only on UD_OK
 *     unless stated otherwise.
 *   - "device pointer" = an address the GPU can dereference (HBM, or pinned host
 *     memory mapped into the GPU's address space); "host pointer" = an address
 *     the CPU can dereference.
 *   - tables and outputs are contiguous row-major, row stride = D elements.
 *   - the library is bound to the HIP device that is current in the calling
 *     thread; it never changes the current device.
 *   - not thread-safe per table handle; distinct handles and distinct streams
 *     may be used from distinct threads.
 */
#ifndef UD_H
#define UD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    UD_OK = 0,
    UD_ERR_INVALID_ARG = 1,        /* null pointer, non-positive size, unknown enum, misaligned pointer */
    UD_ERR_UNSUPPORTED = 2,        /* valid request the library has no code path for */
    UD_ERR_OOM = 3,                /* host pinning or device allocation failed */
    UD_ERR_INDEX_OUT_OF_RANGE = 4, /* an ID outside [0, N) was met by a gather */
    UD_ERR_HIP = 5                 /* any other HIP runtime failure; see ud_last_hip_error */
} ud_status;

/* element type of the table, and of the output */
typedef enum {
    UD_F32 = 0,        /* 4-byte elements in, 4-byte elements out (bit copy) */
    UD_F16 = 1,        /* 2-byte elements in, 2-byte elements out (bit copy) */
    UD_F16_TO_F32 = 2  /* IEEE binary16 in, binary32 out: exact widening, subnormals kept,
                          NaN keeps sign and payload and is returned quiet */
} ud_dtype;

/* element type of the ID list */
typedef enum { UD_I64 = 0, UD_I32 = 1 } ud_itype;

/* flags for ud_alloc_table */
enum {
    UD_TABLE_COHERENT = 0,     /* fine-grained (host-coherent) pinned memory: the default */
    UD_TABLE_NONCOHERENT = 1,  /* coarse-grained pinned memory: GPU caches may keep lines, so CPU
                                  writes made while a kernel runs may not be seen by it */
    UD_TABLE_PAD_ROWS = 2      /* row pitch rounded up to a multiple of 128 bytes, so that every row starts on
                                  a memory line of its own.  The GPU fetches host memory in whole 128-byte
                                  lines; rows of a dense table whose size is no multiple of 128 share their
                                  first and last line with their neighbours and fetch up to 127 bytes more
                                  than they hold (2408-byte rows: 5% more).  Read the pitch with ud_table_pitch */
};

typedef struct ud_table ud_table; /* opaque handle, owned by the library */

/*
 * Feature table in pinned, GPU-mapped host memory (the paper's "unified
 * tensor" storage, Section 4.1: physically in host memory, directly
 * accessible by the GPU, ordinary memory to the CPU).
 * N rows of D elements; elem is UD_F32 (4-byte) or UD_F16 (2-byte).  The memory
 * is uninitialised; the caller fills it through ud_table_host_ptr.  It belongs
 * to the library until ud_free_table.
 * Errors: UD_ERR_INVALID_ARG (N < 1, D < 1, bad elem/flags, t == NULL, size
 * overflow), UD_ERR_OOM (the host could not pin that much).
 */
ud_status ud_alloc_table(int64_t N, int64_t D, ud_dtype elem, unsigned flags, ud_table **t);

/*
 * Device-resident variant: a new table in HBM holding rows [row0, row0 + n) of
 * src (Section 2.2 notes that a table small enough may simply live in GPU
 * memory).  The copy is complete when the call returns.  The result has no
 * host pointer.  src must be a host table.
 * Errors: UD_ERR_INVALID_ARG (bad range, src NULL or already device-resident),
 * UD_ERR_OOM (HBM exhausted).
 */
ud_status ud_table_to_device(const ud_table *src, int64_t row0, int64_t n, ud_table **t);

/* Host address of row 0 (NULL is stored for a device-resident table). */
ud_status ud_table_host_ptr(const ud_table *t, void **p);
/* Device pointer of row 0: what ud_gather takes as `table`. */
ud_status ud_table_device_ptr(const ud_table *t, const void **p);
/* Shape and element type as given at allocation. */
ud_status ud_table_shape(const ud_table *t, int64_t *N, int64_t *D, ud_dtype *elem);
/* Elements between the starts of consecutive rows: D, or more for UD_TABLE_PAD_ROWS.
 * Element (r, c) of the table is at index r * pitch + c from the row-0 pointer. */
ud_status ud_table_pitch(const ud_table *t, int64_t *pitch);
/* Releases the handle and its memory.  NULL is a no-op.  No gather that reads
 * the table may still be in flight. */
ud_status ud_free_table(ud_table *t);

/*
 * out[i, j] = conv(table[idx[i], j])   for 0 <= i < M, 0 <= j < D
 * (features[neighbor_id] of Listings 1-2, result in GPU memory, row order =
 * ID-list order as Section 4.5 requires).
 *
 *   table  device pointer to N x D elements (host-mapped or HBM), aligned to its
 *          element size; read only.
 *   dtype  UD_F32, UD_F16 or UD_F16_TO_F32 (conv = identity on bits, or widening).
 *   idx    device pointer to M IDs of type itype, normally in HBM (the paper's
 *          index is a GPU tensor, Table 1); any GPU-readable memory works, so a
 *          small ID list may stay in pinned host memory and be read over the link
 *          like the rows, which saves its copy.  Duplicates allowed.  Never read
 *          by the CPU.
 *   out    device pointer (HBM) to M x D output elements (4-byte for UD_F32 and
 *          UD_F16_TO_F32, 2-byte for UD_F16), aligned to its element size; must
 *          not overlap table.
 *   stream a hipStream_t passed as void* (NULL = the default stream).
 *
 * Asynchronous: arguments are validated on the host, kernels are enqueued on
 * stream, and the call returns.  M == 0 is UD_OK and enqueues nothing.
 * An ID < 0 or >= N is never dereferenced: its output row is left unwritten and
 * the smallest such position is recorded for ud_gather_status; other rows of
 * the same call are still gathered.  Negative IDs are not wrapped.
 * Errors (synchronous): UD_ERR_INVALID_ARG (N < 1, D < 1, M < 0, unknown enum,
 * NULL or misaligned pointer with M > 0, sizes whose byte counts overflow
 * int64), UD_ERR_HIP (launch failure).
 * The library allocates nothing per call; the first call on a device allocates
 * a 512-byte table of ID-error slots in HBM (one slot per stream, see
 * ud_gather_status) that lives until the process ends.  That first call copies
 * the table's initial contents synchronously, so it must not happen under
 * stream capture: run one gather eagerly before capturing gathers in a HIP graph.
 * For tuning runs the environment variable UD_GATHER_TUNING =
 * "lanes,chunks,rows,max_blocks,flags" (see ud_tuning; 0 = automatic) makes this
 * call use those kernel parameters; it is read once per process.
 */
ud_status ud_gather(const void *table, int64_t N, int64_t D, ud_dtype dtype,
                    const void *idx, ud_itype itype, int64_t M,
                    void *out, void *stream);

/*
 * ud_gather for callers that must not allocate: code running under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same asynchrony, same results and the same
 * ID-error reporting through ud_gather_status as ud_gather -- but the ID-error slots its kernels write
 * to lie in a static device array of the library (64 slots of 8 bytes per GPU, held until the process
 * ends) instead of the table ud_gather allocates on its first call.  This call never calls hipMalloc,
 * hipFree or any allocating library routine, on its first call on a device either (that call only asks
 * the runtime for the array's address on that device).
 * The limit of the fixed array: 63 streams per device may have work of this call outstanding (launched
 * and not yet followed by ud_gather_status on that stream); a call on a further stream is refused with
 * UD_ERR_UNSUPPORTED (ud_last_hip_error tells why) and enqueues nothing.  The
 * array is shared by all calls on a GPU and keeps its contents between calls: a stream's slot holds
 * the smallest bad position seen since ud_gather_status last read (and thereby cleared) it.  Calls on
 * one stream are ordered by the stream; calls that overlap on one GPU on different streams use
 * different slots and do not disturb one another.  ud_gather_status itself pins a few host words on
 * its first use on a device.
 */
ud_status ud_gather_noalloc(const void *table, int64_t N, int64_t D, ud_dtype dtype,
                            const void *idx, ud_itype itype, int64_t M,
                            void *out, void *stream);

/*
 * ud_gather from a table whose rows are `pitch` elements apart (pitch >= D; the
 * elements D .. pitch-1 of each row are padding and are never read): out[i, j] =
 * conv(table[idx[i] * pitch + j]).  The output stays dense (row stride D).  This
 * is the form to use with UD_TABLE_PAD_ROWS tables.  Everything else as ud_gather;
 * extra error: UD_ERR_INVALID_ARG for pitch < D.
 */
ud_status ud_gather_pitched(const void *table, int64_t N, int64_t D, int64_t pitch, ud_dtype dtype,
                            const void *idx, ud_itype itype, int64_t M,
                            void *out, void *stream);

/*
 * Hot-row cache (hybrid placement).  The paper's placement discussion (Section
 * 4.3) notes that data which is reused is better held in GPU memory than
 * re-read over the host link; node IDs of power-law graphs are heavily skewed,
 * so a small set of rows takes a large share of every minibatch.  A cache holds
 * HBM copies of chosen rows of a host table plus a row -> slot map (one int32
 * per table row, in HBM); ud_gather_cached reads a row from HBM when it is
 * cached and over the host link otherwise, in one kernel.  Results are
 * identical to ud_gather on the same table.
 *
 *   table     a host table (ud_alloc_table, dense or padded); must outlive the cache and must
 *             not be written while the cache exists (cached copies would go stale)
 *   hot_rows  host pointer to n_hot row IDs in [0, N); duplicates are tolerated
 *   n_hot     1 .. min(N, 2^31 - 1)
 * The call returns when the cache is filled.  HBM used: n_hot rows + 4 N bytes.
 * Errors: UD_ERR_INVALID_ARG (NULL, device-resident table, bad n_hot or row ID),
 * UD_ERR_OOM (HBM exhausted).
 */
typedef struct ud_cache ud_cache;
ud_status ud_cache_create(const ud_table *table, const int64_t *hot_rows, int64_t n_hot, ud_cache **c);
/* Releases the cache's HBM.  NULL is a no-op.  No gather that uses it may be in flight. */
ud_status ud_cache_free(ud_cache *c);
/* ud_gather on the cache's table (N, D and storage type are the table's): dtype must be
 * UD_F32 for an fp32 table, UD_F16 or UD_F16_TO_F32 for an fp16 table.  Same
 * asynchrony, ID-error behaviour and status reporting as ud_gather. */
ud_status ud_gather_cached(const ud_cache *c, ud_dtype dtype, const void *idx, ud_itype itype, int64_t M,
                           void *out, void *stream);

/*
 * Kernel tuning for ud_gather_tuned.  A zero in one of the first four fields means "choose
 * automatically"; `flags` is taken literally (0 = none of the options; the automatic choice of flags
 * for a table is what ud_gather_plan returns).
 *   lanes_per_row    power of two in [1, 64]: lanes of a wavefront that share one row
 *   chunks_per_lane  1..4: 16-byte chunks of one row each lane keeps in flight
 *                    (with UD_TUNE_DEST_ALIGNED: 1, 2 or 4 output chunks per lane)
 *   rows_in_flight   1, 2 or 4: rows each lane group loads before storing any
 *                    (rows_in_flight x chunks_per_lane <= 8; 4 x 2 is not built)
 *   max_blocks       cap on workgroups (grid-stride beyond it).  A gather that should run beside another
 *                    stream's kernels needs a small grid: with 256 or more workgroups nothing else is
 *                    scheduled until it ends, with 64..128 it overlaps (rows of 1 KiB or more then still
 *                    reach the full link rate; shorter rows want rows_in_flight > 1 as well)
 *   flags            UD_TUNE_* bits
 */
typedef struct {
    int32_t lanes_per_row;
    int32_t chunks_per_lane;
    int32_t rows_in_flight;
    int32_t max_blocks;
    uint32_t flags;
} ud_tuning;

enum {
    UD_TUNE_NT_STORE = 2u,      /* non-temporal (streaming) stores to out */
    UD_TUNE_ELEMENTWISE = 4u,   /* one lane per element, rows straddling wavefronts: the layout of
                                   the unmodified indexing kernel of Section 4.5 / Figure 4, kept as
                                   the comparison point and as the fallback for odd alignments */
    UD_TUNE_CIRCULAR_SHIFT = 32u, /* with UD_TUNE_ELEMENTWISE: rotate each row's lanes as in Section 4.5 / Figure 5 of
                                   the paper (its alignment fix), for comparison */
    UD_TUNE_SHARE_GPU = 128u,   /* launch shape for a gather that runs beside another stream's kernels: a grid of
                                   64 workgroups for rows of 1 KiB or more, 128 below (unless max_blocks is given),
                                   and enough rows in flight per lane group to keep about 1 KiB per wavefront on
                                   the link; 94-100% of the stand-alone rate */
    UD_TUNE_DEST_ALIGNED = 256u, /* the kernel that cuts the OUTPUT, taken as one dense stream, into aligned 16-byte
                                   chunks (every store an aligned dwordx4, every output line written whole by one
                                   wavefront) and reads the table with element-aligned loads.  The automatic
                                   choice for tables in HBM, where the gather is bound by HBM bandwidth; tables
                                   read over the host link use the source-aligned kernel (flag clear).  Uses
                                   chunks_per_lane and max_blocks; lanes_per_row and rows_in_flight are ignored.
                                   Not combinable with ELEMENTWISE or SHARE_GPU */
    UD_TUNE_FLAT_SOURCE = 512u  /* ud_scatter_tuned only: the scatter kernel that cuts the dense SOURCE into aligned
                                   16-byte chunks, one per lane (no idle lanes whatever the width), and writes the table
                                   rows with element-aligned stores.  The automatic choice for tables in HBM; tables
                                   behind the host link take the kernel that writes whole aligned chunks of the table
                                   (flag clear).  Uses chunks_per_lane (1, 2 or 4; automatic: 2 for rows up to 256
                                   bytes, else 1) and max_blocks; may be combined with UD_TUNE_NT_STORE (streaming
                                   stores to the table, which the automatic choice uses) */
};

/* ud_gather with explicit kernel parameters (for the tuning loop and for tests that
 * exercise every kernel instantiation).  tuning == NULL behaves like ud_gather.
 * Extra error: UD_ERR_INVALID_ARG for a field outside the ranges above,
 * UD_ERR_UNSUPPORTED for a combination with no instantiation. */
ud_status ud_gather_tuned(const void *table, int64_t N, int64_t D, ud_dtype dtype,
                          const void *idx, ud_itype itype, int64_t M,
                          void *out, void *stream, const ud_tuning *tuning);

/*
 * Write direction: table[idx[i], j] = src[i, j]  for 0 <= i < M, 0 <= j < D.
 * The paper notes (Section 3) that a GPU which dereferences host memory issues
 * write requests on the host link as well as reads; this is the gather's
 * mirror image, e.g. for updating rows of a host-resident table from the GPU.
 *
 *   table  device pointer to N x D elements (host-mapped or HBM), written
 *   dtype  UD_F32 or UD_F16 (bit copy; UD_F16_TO_F32 is an invalid argument)
 *   idx    device pointer (HBM) to M row IDs.  IDs should be distinct: if an ID
 *          occurs more than once, each element of that row receives the value
 *          from one of its source rows, which one is unspecified
 *   src    device pointer (HBM) to M x D dense source elements; must not
 *          overlap table
 * Asynchronous on stream like ud_gather; the CPU may read the rows of a host
 * table after the stream has been synchronised (ud_gather_status does).
 * Rows whose ID is out of range are skipped and reported through
 * ud_gather_status exactly as for ud_gather.  Errors as ud_gather.
 */
ud_status ud_scatter(void *table, int64_t N, int64_t D, ud_dtype dtype,
                     const void *idx, ud_itype itype, int64_t M,
                     const void *src, void *stream);
/* ud_scatter into a table whose rows are `pitch` elements apart (UD_TABLE_PAD_ROWS); the padding is never written. */
ud_status ud_scatter_pitched(void *table, int64_t N, int64_t D, int64_t pitch, ud_dtype dtype,
                             const void *idx, ud_itype itype, int64_t M,
                             const void *src, void *stream);
/* ud_scatter with explicit kernel parameters (tuning->flags: 0, UD_TUNE_FLAT_SOURCE, or that with UD_TUNE_NT_STORE). */
ud_status ud_scatter_tuned(void *table, int64_t N, int64_t D, ud_dtype dtype,
                           const void *idx, ud_itype itype, int64_t M,
                           const void *src, void *stream, const ud_tuning *tuning);

/* The parameters ud_gather would pick for this shape and table alignment (no launch). */
ud_status ud_gather_plan(const void *table, int64_t D, ud_dtype dtype, ud_tuning *plan);

/*
 * Waits for stream, then reports the ID errors of the gathers and scatters that were enqueued on
 * THAT stream (on the current device) since the previous ud_gather_status call for it: UD_OK and
 * *bad_pos = -1 if none, else UD_ERR_INDEX_OUT_OF_RANGE and *bad_pos = the smallest offending
 * position i (position in idx, not the ID).  bad_pos is written in both cases and may be NULL.
 * The stream's record is read and cleared in one step, in stream order (a one-thread kernel on
 * `stream`), so errors of work on other streams are neither reported nor lost, and nothing runs on
 * the default stream.  A device keeps 63 per-stream records.  When all are taken, a stream that
 * launches for the first time takes over the record of a stream that has launched nothing since its
 * own last ud_gather_status call; if there is none, it shares one common record with all other
 * streams in that position.  A stream handle that is destroyed and handed out again by the runtime
 * inherits its predecessor's record.  A stream is driven by one thread at a time; different threads
 * may drive different streams concurrently.  Gathers replayed from a HIP graph report to the record
 * of the stream they were captured on: synchronise the replay, then query that stream.
 * Not to be called while `stream` is being captured.
 */
ud_status ud_gather_status(void *stream, int64_t *bad_pos);

/* Static, human-readable name of a status code. */
const char *ud_status_str(ud_status s);
/* HIP's message for the most recent UD_ERR_HIP / UD_ERR_OOM in this thread ("" if none). */
const char *ud_last_hip_error(void);
/* Identifies the sources this library was built from: the hex digest the build script computed over
 * them ("unknown" for a build made some other way).  Static string. */
const char *ud_build_id(void);

#ifdef __cplusplus
}
#endif
#endif /* UD_H */
