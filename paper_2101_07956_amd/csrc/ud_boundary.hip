// C-ABI boundary of the row-gather library: table allocation in pinned,
// GPU-mapped host memory (the storage of the paper's "unified tensor",
// PyTorch-Direct Section 4.1), the device-resident variant, argument checks,
// kernel selection and the asynchronous ID-error record.  Host code only; the
// kernels live in ud_gather_*.hip.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "ud.h"
#include "ud_internal.h"

struct ud_table {
    void *host;      // CPU address of row 0, nullptr when device-resident
    void *dev;       // GPU address of row 0
    int64_t N, D;
    int64_t pitch;   // elements between rows, >= D
    ud_dtype elem;
    bool device_resident;
};

struct ud_cache {
    const void *table; // GPU address of the host table's row 0
    int64_t N, D;
    int64_t pitch;     // the host table's row pitch in elements
    ud_dtype elem;
    void *rows;        // HBM copy of the hot rows, slot-major
    int32_t *slot;     // HBM, N entries: slot of each table row in `rows`, or -1
    int64_t n_hot;
};

namespace {

thread_local char g_hip_msg[256] = "";

ud_status hip_fail(hipError_t e, const char *what)
{
    std::snprintf(g_hip_msg, sizeof g_hip_msg, "%s: %s", what, hipGetErrorString(e));
    (void)hipGetLastError(); // do not leave the error for an unrelated later call
    return e == hipErrorOutOfMemory ? UD_ERR_OOM : UD_ERR_HIP;
}

int elem_bytes(ud_dtype t) { return t == UD_F32 ? 4 : 2; }
int out_elem_bytes(ud_dtype t) { return t == UD_F16 ? 2 : 4; }

bool mul3_overflows(int64_t a, int64_t b, int64_t c, int64_t *r)
{
    int64_t ab;
    return __builtin_mul_overflow(a, b, &ab) || __builtin_mul_overflow(ab, c, r);
}

// ID-error records.  Every device has a small table of error slots in HBM, one
// per stream that has launched a gather or scatter (the kernels take the slot's
// address and atomic-min the position of a bad ID into it).  The table is
// allocated once, on the first launch on that device, and nothing is allocated
// per call.  A stream keeps its slot until the table is full and another stream
// needs one: then a slot whose owner has launched nothing since its last
// ud_gather_status call (so all its work is complete and its record is clear) is
// handed on.  If there is none, the last slot is shared by the streams that
// found no slot of their own.
constexpr int kMaxDevices = 64;
constexpr int kErrSlots = 64;

struct SlotTable {
    unsigned long long *words = nullptr;     // device memory, kErrSlots words
    hipStream_t owner[kErrSlots] = {};
    std::atomic<bool> busy[kErrSlots] = {};  // launched on since the owner's last status call
    int used = 0;
};

// Bumped whenever a slot changes hands, so that per-thread shortcuts to a slot notice.
std::atomic<unsigned long long> g_slot_generation{0};

constexpr int kSlotTables = 2;                // slot tables a stream can hold a slot in

struct DeviceState {
    SlotTable heap;                          // hipMalloc'd at the first launch
    SlotTable fixed;                         // this device's copy of `scratch` (ud_gather_noalloc)
    unsigned long long *result_host = nullptr;   // pinned: where ud_gather_status receives a slot's value
    unsigned long long *result_dev = nullptr;    // the same words as the GPU addresses them
};

std::mutex g_err_mutex;
DeviceState g_dev[kMaxDevices];

// Error slots for ud_gather_noalloc: device memory that exists without any allocation call.  Every
// GPU the library runs on holds its own copy of this array (512 bytes) until the process ends.  In
// host code the name is only a stand-in for the symbol: the address the kernels use is asked for
// once per device with hipGetSymbolAddress and kept in DeviceState::fixed.words.  The array comes
// up holding "no bad ID" in every slot; afterwards it keeps what the last calls left, and each slot is
// cleared when ud_gather_status reads it.
#define UD_REP4(x) x, x, x, x
#define UD_REP16(x) UD_REP4(x), UD_REP4(x), UD_REP4(x), UD_REP4(x)
#define UD_REP64(x) UD_REP16(x), UD_REP16(x), UD_REP16(x), UD_REP16(x)
static_assert(kErrSlots == 64, "the initialiser below names 64 slots");
static __device__ __align__(256) unsigned long long scratch[kErrSlots] = {UD_REP64(0x7fffffffffffffffull)};
static_assert(ud::kNoBadIndex == 0x7fffffffffffffffull, "scratch is initialised with the no-bad-ID sentinel");

// Index of `stream`'s slot in t, claiming one if `claim`; -1 if it has none.
int find_slot(SlotTable &t, hipStream_t stream, bool claim, bool share_last)
{
    for (int k = 0; k < t.used; ++k)
        if (t.owner[k] == stream)
            return k;
    if (!claim)
        return (share_last && t.used == kErrSlots - 1) ? kErrSlots - 1 : -1;
    if (t.used < kErrSlots - 1) {
        t.owner[t.used] = stream;
        return t.used++;
    }
    for (int k = 0; k < t.used; ++k)
        if (!t.busy[k].load()) {                               // idle since its owner's last status call
            // The old owner's thread may be about to launch again through its per-thread shortcut, which marks
            // the slot busy first and compares the generation afterwards.  Bumping the generation first and
            // taking the slot only if it is still idle means exactly one side gets it: a shortcut that marked
            // it busy before this exchange keeps the slot, one that comes later sees the new generation.
            g_slot_generation.fetch_add(1);
            bool idle = false;
            if (t.busy[k].compare_exchange_strong(idle, true)) {
                t.owner[k] = stream;
                return k;
            }
        }
    return share_last ? kErrSlots - 1 : -1;
}

ud_status current_device(int *dev)
{
    const hipError_t e = hipGetDevice(dev);
    if (e != hipSuccess)
        return hip_fail(e, "hipGetDevice");
    if (*dev < 0 || *dev >= kMaxDevices)
        return UD_ERR_UNSUPPORTED;
    return UD_OK;
}

// The error slot the kernels of a launch on `stream` report to.  `fixed`: take it from the static
// device array instead of the allocated table; this path allocates nothing and fails, rather than
// share a slot, when every slot belongs to another stream.
ud_status error_slot(hipStream_t stream, bool fixed, unsigned long long **w)
{
    // the common case: the same thread launching on the same stream again
    thread_local int last_dev[2] = {-1, -1};
    thread_local hipStream_t last_stream[2] = {nullptr, nullptr};
    thread_local unsigned long long *last_slot[2] = {nullptr, nullptr};
    thread_local std::atomic<bool> *last_busy[2] = {nullptr, nullptr};
    thread_local unsigned long long last_generation[2] = {0, 0};
    int dev = 0;
    const ud_status st = current_device(&dev);
    if (st != UD_OK)
        return st;
    const int f = fixed ? 1 : 0;
    if (last_slot[f] && dev == last_dev[f] && stream == last_stream[f]) {
        // busy first, generation second (see find_slot): if the slot went to another stream in between,
        // the generation has moved and the slow path finds this stream a slot of its own
        last_busy[f]->store(true);
        if (last_generation[f] == g_slot_generation.load()) {
            *w = last_slot[f];
            return UD_OK;
        }
    }
    std::lock_guard<std::mutex> lock(g_err_mutex);
    SlotTable &t = fixed ? g_dev[dev].fixed : g_dev[dev].heap;
    if (!t.words && fixed) {
        // once per device, with that device current: where this GPU keeps its copy of the array
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return hip_fail(e != hipSuccess ? e : hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch)");
        t.words = static_cast<unsigned long long *>(p);
    } else if (!t.words) {
        unsigned long long *p = nullptr;
        hipError_t e = hipMalloc(reinterpret_cast<void **>(&p), kErrSlots * sizeof *p);
        if (e != hipSuccess)
            return hip_fail(e, "hipMalloc(error slots)");
        unsigned long long init[kErrSlots];
        for (unsigned long long &x : init)
            x = ud::kNoBadIndex;
        e = hipMemcpy(p, init, sizeof init, hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            (void)hipFree(p);
            return hip_fail(e, "hipMemcpy(error slots)");
        }
        t.words = p;
    }
    const int k = find_slot(t, stream, true, !fixed);
    if (k < 0) {
        std::snprintf(g_hip_msg, sizeof g_hip_msg,
                      "ud_gather_noalloc: all %d static error slots of this device belong to other streams", kErrSlots - 1);
        return UD_ERR_UNSUPPORTED;
    }
    *w = t.words + k;
    t.busy[k].store(true, std::memory_order_release);
    if (k < kErrSlots - 1) {                 // the shared slot is not worth remembering
        last_dev[f] = dev;
        last_stream[f] = stream;
        last_slot[f] = *w;
        last_busy[f] = &t.busy[k];
        last_generation[f] = g_slot_generation.load(std::memory_order_acquire);
    }
    return UD_OK;
}

// Where a table lives decides the launch shape (the host link and HBM bound different kernels).
// Tables made by this library are known exactly: their address ranges are kept here from
// allocation to ud_free_table.
struct Range {
    uintptr_t lo, hi;
    bool hbm;
};
std::mutex g_range_mutex;
std::vector<Range> g_ranges;

void remember_range(const void *p, size_t bytes, bool hbm)
{
    std::lock_guard<std::mutex> lock(g_range_mutex);
    const uintptr_t lo = reinterpret_cast<uintptr_t>(p);
    g_ranges.push_back(Range{lo, lo + bytes, hbm});
}

void forget_range(const void *p)
{
    std::lock_guard<std::mutex> lock(g_range_mutex);
    const uintptr_t lo = reinterpret_cast<uintptr_t>(p);
    for (size_t k = 0; k < g_ranges.size(); ++k)
        if (g_ranges[k].lo == lo) {
            g_ranges[k] = g_ranges.back();
            g_ranges.pop_back();
            return;
        }
}

// A pointer inside no table of this library is asked of the runtime, and the answer kept in a
// small per-thread cache (callers alternate between a few tables: a host table and its HBM
// slice, say).  The cache is keyed on the address, so memory that is freed and allocated again as
// the other kind can be misjudged until it leaves the cache; like an unknown pointer, which is
// taken for host memory, that only costs launch-shape tuning, never correctness.
bool table_is_in_hbm(const void *table)
{
    const uintptr_t a = reinterpret_cast<uintptr_t>(table);
    {
        std::lock_guard<std::mutex> lock(g_range_mutex);
        for (const Range &r : g_ranges)
            if (a >= r.lo && a < r.hi)
                return r.hbm;
    }
    constexpr int kRecent = 8;
    thread_local uintptr_t ptr[kRecent] = {};
    thread_local bool kind[kRecent] = {};
    thread_local int next = 0;
    for (int k = 0; k < kRecent; ++k)
        if (a && ptr[k] == a)
            return kind[k];
    hipPointerAttribute_t attr{};
    bool in_hbm = false;
    if (hipPointerGetAttributes(&attr, table) == hipSuccess)
        in_hbm = attr.type == hipMemoryTypeDevice;
    else
        (void)hipGetLastError();
    ptr[next] = a;
    kind[next] = in_hbm;
    next = (next + 1) % kRecent;
    return in_hbm;
}

int next_pow2(int64_t x)
{
    int p = 1;
    while (p < x && p < 64)
        p <<= 1;
    return p;
}

// Largest number of 16-byte chunks any row can overlap, given the base address
// and the row pitch: the row start offsets modulo 16 cycle with period <= 16.
int64_t max_chunks_per_row(uintptr_t base, int64_t row_bytes, int64_t pitch_bytes)
{
    int64_t worst_head = 0;
    for (int k = 0; k < 16; ++k) {
        const int64_t head = static_cast<int64_t>((base + static_cast<uintptr_t>(k) * static_cast<uintptr_t>(pitch_bytes)) & 15u);
        if (head > worst_head)
            worst_head = head;
    }
    return (worst_head + row_bytes + 15) >> 4;
}

constexpr int kDefaultMaxBlocks = 1 << 22;

// Launch shape by row width and table residence, from sweeps on MI355X:
//  * host table (link-bound): the source-aligned chunked kernel, one row per
//    wavefront instruction (64 lanes per row) for every row longer than 64
//    bytes, a single row in flight per lane group.  Whole-wave loads of one row
//    reach 99-100% of the pinned-memcpy rate for 256..1024-byte rows; packing
//    several short rows into one instruction costs 3-5%.  From 1 KiB rows up a
//    fixed grid of 128 workgroups striding over the rows, two rows in flight per
//    wavefront, is 1-3% faster than one wavefront per row.
//  * HBM table (bandwidth-bound): the destination-aligned kernel with streaming
//    stores, kFlatChunks chunks per lane, for rows longer than 64 bytes (equal to
//    the chunked kernel on widths that are multiples of 128 bytes, 3% faster at
//    400-byte and 12% at 2408-byte rows); 64-byte rows and shorter stay with the
//    chunked kernel (no idle lanes, two rows in flight, streaming stores).
constexpr int kFlatChunks = 2;
constexpr int kScatterFlatChunks = 1;

// The source-aligned chunked kernel's shape (also the scatter's, which mirrors it).
ud::Plan chunked_plan(const void *table, int64_t D, int64_t pitch, ud_dtype dtype, bool hbm)
{
    const int64_t row_bytes = D * elem_bytes(dtype);
    const int64_t nch = max_chunks_per_row(reinterpret_cast<uintptr_t>(table), row_bytes, pitch * elem_bytes(dtype));
    ud::Plan p{};
    p.flags = hbm ? UD_TUNE_NT_STORE : 0u;
    p.max_blocks = kDefaultMaxBlocks;
    p.tile_id_lines = !hbm;
    if (nch <= 64) {
        p.lanes_per_row = (!hbm && row_bytes > 64) ? 64 : next_pow2(nch);
        p.chunks_per_lane = 1;
        p.rows_in_flight = hbm ? 2 : 1;
    } else {
        p.lanes_per_row = 64;
        const int64_t passes = (nch + 63) / 64;
        p.chunks_per_lane = passes > 4 ? 4 : static_cast<int>(passes);
        p.rows_in_flight = (hbm && p.chunks_per_lane <= 2) ? 2 : 1;
    }
    if (!hbm && row_bytes >= 1024) {
        // few wavefronts, two rows in flight each: 0.3-0.7% faster than 512 workgroups with one row each, and
        // a grid of 128 workgroups leaves room for another stream's kernels to run beside the gather
        p.max_blocks = 128;
        if (p.chunks_per_lane * 2 <= 8)
            p.rows_in_flight = 2;
    }
    return p;
}

// What ud_gather does by itself.
ud::Plan auto_plan(const void *table, int64_t D, int64_t pitch, ud_dtype dtype)
{
    const bool hbm = table_is_in_hbm(table);
    if (hbm && D * elem_bytes(dtype) > 64) {
        ud::Plan p{};
        p.flags = UD_TUNE_NT_STORE | UD_TUNE_DEST_ALIGNED;
        p.max_blocks = kDefaultMaxBlocks;
        p.lanes_per_row = 64;              // not used by the destination-aligned kernel
        p.chunks_per_lane = kFlatChunks;
        p.rows_in_flight = 1;
        return p;
    }
    return chunked_plan(table, D, pitch, dtype, hbm);
}

bool is_pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

// UD_GATHER_TUNING="lanes,chunks,rows,max_blocks,flags" (any field may be 0 = automatic) makes
// ud_gather behave like ud_gather_tuned with those parameters: an A/B switch for tuning runs that
// needs no change in the caller.  Read once per process; malformed values are ignored.
const ud_tuning *env_tuning()
{
    static const ud_tuning *cached = []() -> const ud_tuning * {
        const char *v = std::getenv("UD_GATHER_TUNING");
        if (!v || !*v)
            return nullptr;
        static ud_tuning t{};
        int lanes = 0, chunks = 0, rows = 0, blocks = 0;
        unsigned flags = 0;
        if (std::sscanf(v, "%d,%d,%d,%d,%u", &lanes, &chunks, &rows, &blocks, &flags) != 5)
            return nullptr;
        t.lanes_per_row = lanes;
        t.chunks_per_lane = chunks;
        t.rows_in_flight = rows;
        t.max_blocks = blocks;
        t.flags = flags;
        return &t;
    }();
    return cached;
}

} // namespace

extern "C" {

ud_status ud_alloc_table(int64_t N, int64_t D, ud_dtype elem, unsigned flags, ud_table **t)
{
    if (!t || N < 1 || D < 1 || (elem != UD_F32 && elem != UD_F16) || (flags & ~3u))
        return UD_ERR_INVALID_ARG;
    int64_t pitch = D;
    if (flags & UD_TABLE_PAD_ROWS) {
        // rows start on 128-byte lines: no row shares a line with its neighbours
        const int64_t per_line = 128 / elem_bytes(elem);
        if (D > INT64_MAX - per_line)
            return UD_ERR_INVALID_ARG;
        pitch = (D + per_line - 1) / per_line * per_line;
    }
    int64_t bytes;
    if (mul3_overflows(N, pitch, elem_bytes(elem), &bytes))
        return UD_ERR_INVALID_ARG;
    const unsigned hip_flags =
        hipHostMallocMapped | ((flags & UD_TABLE_NONCOHERENT) ? hipHostMallocNonCoherent : hipHostMallocCoherent);
    void *host = nullptr;
    hipError_t e = hipHostMalloc(&host, static_cast<size_t>(bytes), hip_flags);
    if (e != hipSuccess)
        return hip_fail(e, "hipHostMalloc");
    void *dev = nullptr;
    e = hipHostGetDevicePointer(&dev, host, 0);
    if (e != hipSuccess) {
        (void)hipHostFree(host);
        return hip_fail(e, "hipHostGetDevicePointer");
    }
    ud_table *h = new (std::nothrow) ud_table{host, dev, N, D, pitch, elem, false};
    if (!h) {
        (void)hipHostFree(host);
        return UD_ERR_OOM;
    }
    remember_range(dev, static_cast<size_t>(bytes), false);
    *t = h;
    return UD_OK;
}

ud_status ud_table_to_device(const ud_table *src, int64_t row0, int64_t n, ud_table **t)
{
    if (!src || !t || src->device_resident || row0 < 0 || n < 1 || row0 > src->N - n)
        return UD_ERR_INVALID_ARG;
    const int64_t row_bytes = src->pitch * elem_bytes(src->elem);   // the copy keeps the pitch
    const size_t bytes = static_cast<size_t>(n) * static_cast<size_t>(row_bytes);
    void *dev = nullptr;
    hipError_t e = hipMalloc(&dev, bytes);
    if (e != hipSuccess)
        return hip_fail(e, "hipMalloc(table)");
    e = hipMemcpy(dev, static_cast<const char *>(src->host) + row0 * row_bytes, bytes, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        (void)hipFree(dev);
        return hip_fail(e, "hipMemcpy(table)");
    }
    ud_table *h = new (std::nothrow) ud_table{nullptr, dev, n, src->D, src->pitch, src->elem, true};
    if (!h) {
        (void)hipFree(dev);
        return UD_ERR_OOM;
    }
    remember_range(dev, bytes, true);
    *t = h;
    return UD_OK;
}

ud_status ud_table_host_ptr(const ud_table *t, void **p)
{
    if (!t || !p)
        return UD_ERR_INVALID_ARG;
    *p = t->host;
    return UD_OK;
}

ud_status ud_table_device_ptr(const ud_table *t, const void **p)
{
    if (!t || !p)
        return UD_ERR_INVALID_ARG;
    *p = t->dev;
    return UD_OK;
}

ud_status ud_table_shape(const ud_table *t, int64_t *N, int64_t *D, ud_dtype *elem)
{
    if (!t)
        return UD_ERR_INVALID_ARG;
    if (N)
        *N = t->N;
    if (D)
        *D = t->D;
    if (elem)
        *elem = t->elem;
    return UD_OK;
}

ud_status ud_table_pitch(const ud_table *t, int64_t *pitch)
{
    if (!t || !pitch)
        return UD_ERR_INVALID_ARG;
    *pitch = t->pitch;
    return UD_OK;
}

ud_status ud_free_table(ud_table *t)
{
    if (!t)
        return UD_OK;
    forget_range(t->dev);
    const hipError_t e = t->device_resident ? hipFree(t->dev) : hipHostFree(t->host);
    delete t;
    return e == hipSuccess ? UD_OK : hip_fail(e, "free");
}

ud_status ud_gather_plan(const void *table, int64_t D, ud_dtype dtype, ud_tuning *plan)
{
    if (!plan || D < 1 || (dtype != UD_F32 && dtype != UD_F16 && dtype != UD_F16_TO_F32))
        return UD_ERR_INVALID_ARG;
    int64_t row_bytes;
    if (__builtin_mul_overflow(D, static_cast<int64_t>(elem_bytes(dtype)), &row_bytes) || row_bytes > INT64_MAX - 64)
        return UD_ERR_INVALID_ARG;
    const ud::Plan p = auto_plan(table, D, D, dtype);
    plan->lanes_per_row = p.lanes_per_row;
    plan->chunks_per_lane = p.chunks_per_lane;
    plan->rows_in_flight = p.rows_in_flight;
    plan->max_blocks = p.max_blocks;
    plan->flags = p.flags;
    return UD_OK;
}

static ud_status gather_impl(const void *table, int64_t N, int64_t D, int64_t pitch, ud_dtype dtype,
                             const void *idx, ud_itype itype, int64_t M,
                             void *out, void *stream, const ud_tuning *tuning,
                             const int32_t *slot, const char *cache, bool fixed_slots = false)
{
    if (N < 1 || D < 1 || M < 0 || pitch < D)
        return UD_ERR_INVALID_ARG;
    if (dtype != UD_F32 && dtype != UD_F16 && dtype != UD_F16_TO_F32)
        return UD_ERR_INVALID_ARG;
    if (itype != UD_I64 && itype != UD_I32)
        return UD_ERR_INVALID_ARG;
    int64_t table_bytes, out_bytes;
    if (mul3_overflows(N, pitch, elem_bytes(dtype), &table_bytes) || mul3_overflows(M, D, out_elem_bytes(dtype), &out_bytes))
        return UD_ERR_INVALID_ARG;
    if (table_bytes > INT64_MAX - 64)
        return UD_ERR_INVALID_ARG;

    ud::Plan plan = auto_plan(table, D, pitch, dtype);
    if (tuning) {
        if (tuning->flags & ~(UD_TUNE_NT_STORE | UD_TUNE_ELEMENTWISE | UD_TUNE_CIRCULAR_SHIFT |
                              UD_TUNE_SHARE_GPU | UD_TUNE_DEST_ALIGNED))
            return UD_ERR_INVALID_ARG;
        if ((tuning->flags & UD_TUNE_CIRCULAR_SHIFT) && !(tuning->flags & UD_TUNE_ELEMENTWISE))
            return UD_ERR_INVALID_ARG;
        if ((tuning->flags & UD_TUNE_DEST_ALIGNED) &&
            (tuning->flags & (UD_TUNE_ELEMENTWISE | UD_TUNE_SHARE_GPU)))
            return UD_ERR_INVALID_ARG;
        if (tuning->lanes_per_row < 0 || tuning->lanes_per_row > 64 ||
            (tuning->lanes_per_row && !is_pow2(tuning->lanes_per_row)))
            return UD_ERR_INVALID_ARG;
        if (tuning->chunks_per_lane < 0 || tuning->chunks_per_lane > 4)
            return UD_ERR_INVALID_ARG;
        const int u = tuning->rows_in_flight;
        if (u != 0 && u != 1 && u != 2 && u != 4)
            return UD_ERR_INVALID_ARG;
        if (tuning->max_blocks < 0)
            return UD_ERR_INVALID_ARG;
        if ((plan.flags & UD_TUNE_DEST_ALIGNED) && !(tuning->flags & UD_TUNE_DEST_ALIGNED)) {
            // the automatic plan chose the destination-aligned kernel, the caller another one: start
            // from the chunked kernel's defaults for this width
            plan = chunked_plan(table, D, pitch, dtype, true);
        } else if (!(plan.flags & UD_TUNE_DEST_ALIGNED) && (tuning->flags & UD_TUNE_DEST_ALIGNED)) {
            plan.chunks_per_lane = kFlatChunks;
            plan.rows_in_flight = 1;
            plan.max_blocks = kDefaultMaxBlocks;
        }
        plan.flags = tuning->flags;
        if (tuning->lanes_per_row)
            plan.lanes_per_row = tuning->lanes_per_row;
        if (tuning->chunks_per_lane)
            plan.chunks_per_lane = tuning->chunks_per_lane;
        if (tuning->rows_in_flight)
            plan.rows_in_flight = tuning->rows_in_flight;
        else if (tuning->chunks_per_lane && plan.rows_in_flight * plan.chunks_per_lane > 8)
            plan.rows_in_flight = 1;
        if (tuning->max_blocks)
            plan.max_blocks = tuning->max_blocks;
        if (tuning->flags & UD_TUNE_SHARE_GPU) {
            // few wavefronts, each with about 1 KiB on the link: 64 workgroups x 4 wavefronts cover the
            // link's round trip for rows of 1 KiB and more (measured: 99-100% of the stand-alone rate),
            // 128 workgroups are needed below that (94-98%); either leaves the compute units free
            // for the other stream's kernels, 256 or more do not
            const int64_t rb = D * elem_bytes(dtype);
            if (!tuning->max_blocks)
                plan.max_blocks = rb >= 1024 ? 64 : 128;
            if (!tuning->rows_in_flight && !tuning->chunks_per_lane && plan.chunks_per_lane == 1) {
                const int64_t per_pass = rb * (64 / plan.lanes_per_row);     // bytes one wavefront instruction fetches
                plan.rows_in_flight = per_pass >= 1024 ? 1 : per_pass >= 512 ? 2 : 4;
            }
        }
        if (plan.flags & UD_TUNE_DEST_ALIGNED) {
            if (!ud::flat_supports(N, D, pitch * elem_bytes(dtype), M) || plan.chunks_per_lane == 3)
                return UD_ERR_UNSUPPORTED;
        } else if (plan.rows_in_flight * plan.chunks_per_lane > 8 || (plan.rows_in_flight == 4 && plan.chunks_per_lane == 2)) {
            return UD_ERR_UNSUPPORTED;
        }
    }

    // the automatic choice falls back to the source-aligned kernel for shapes the other does not cover
    if ((plan.flags & UD_TUNE_DEST_ALIGNED) && !ud::flat_supports(N, D, pitch * elem_bytes(dtype), M))
        plan = chunked_plan(table, D, pitch, dtype, true);

    if (M == 0)
        return UD_OK;
    if (!table || !idx || !out)
        return UD_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(table) % elem_bytes(dtype) || reinterpret_cast<uintptr_t>(out) % out_elem_bytes(dtype) ||
        reinterpret_cast<uintptr_t>(idx) % (itype == UD_I64 ? 8 : 4))
        return UD_ERR_INVALID_ARG;

    ud::GatherArgs a{};
    a.table = static_cast<const char *>(table);
    a.N = N;
    a.D = D;
    a.pitch_bytes = pitch * elem_bytes(dtype);
    a.idx = idx;
    a.itype = itype;
    a.M = M;
    a.out = out;
    a.slot = slot;
    a.cache = cache;
    a.group_iters = 1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const ud_status es = error_slot(s, fixed_slots, &a.err);
    if (es != UD_OK)
        return es;

    hipError_t e;
    if (plan.flags & UD_TUNE_ELEMENTWISE)
        e = ud::launch_elementwise(a, dtype, plan, s);
    else if (plan.flags & UD_TUNE_DEST_ALIGNED)
        e = ud::launch_flat(a, dtype, plan, s);
    else if (dtype == UD_F32)
        e = ud::launch_chunked_f32(a, plan, s);
    else if (dtype == UD_F16)
        e = ud::launch_chunked_f16(a, plan, s);
    else
        e = ud::launch_chunked_f16_to_f32(a, plan, s);
    if (e == hipErrorInvalidValue)
        return UD_ERR_UNSUPPORTED;
    if (e != hipSuccess)
        return hip_fail(e, "kernel launch");
    return UD_OK;
}

ud_status ud_gather_tuned(const void *table, int64_t N, int64_t D, ud_dtype dtype,
                          const void *idx, ud_itype itype, int64_t M,
                          void *out, void *stream, const ud_tuning *tuning)
{
    return gather_impl(table, N, D, D, dtype, idx, itype, M, out, stream, tuning, nullptr, nullptr);
}

ud_status ud_gather_pitched(const void *table, int64_t N, int64_t D, int64_t pitch, ud_dtype dtype,
                            const void *idx, ud_itype itype, int64_t M,
                            void *out, void *stream)
{
    return gather_impl(table, N, D, pitch, dtype, idx, itype, M, out, stream, nullptr, nullptr, nullptr);
}

ud_status ud_gather(const void *table, int64_t N, int64_t D, ud_dtype dtype,
                    const void *idx, ud_itype itype, int64_t M,
                    void *out, void *stream)
{
    return gather_impl(table, N, D, D, dtype, idx, itype, M, out, stream, env_tuning(), nullptr, nullptr);
}

ud_status ud_gather_noalloc(const void *table, int64_t N, int64_t D, ud_dtype dtype,
                            const void *idx, ud_itype itype, int64_t M,
                            void *out, void *stream)
{
    return gather_impl(table, N, D, D, dtype, idx, itype, M, out, stream, nullptr, nullptr, nullptr, true);
}

static ud_status scatter_impl(void *table, int64_t N, int64_t D, int64_t pitch, ud_dtype dtype,
                              const void *idx, ud_itype itype, int64_t M,
                              const void *src, void *stream, const ud_tuning *tuning)
{
    if (N < 1 || D < 1 || M < 0 || pitch < D)
        return UD_ERR_INVALID_ARG;
    if (dtype != UD_F32 && dtype != UD_F16)
        return UD_ERR_INVALID_ARG;
    if (itype != UD_I64 && itype != UD_I32)
        return UD_ERR_INVALID_ARG;
    int64_t table_bytes, src_bytes;
    if (mul3_overflows(N, pitch, elem_bytes(dtype), &table_bytes) || mul3_overflows(M, D, elem_bytes(dtype), &src_bytes))
        return UD_ERR_INVALID_ARG;
    if (table_bytes > INT64_MAX - 64)
        return UD_ERR_INVALID_ARG;
    // Launch shape: the row-per-lane-group kernel (aligned whole-chunk writes) for tables behind the host link;
    // the source-aligned kernel (no idle lanes) for tables in HBM, where it is 10-25% faster on widths whose
    // chunk count is no power of two and equal elsewhere.
    const bool hbm = table_is_in_hbm(table);
    ud::Plan plan = chunked_plan(table, D, pitch, dtype, hbm);
    plan.flags = 0;
    plan.rows_in_flight = 1;           // measured: one row in flight is 0-6% faster than two for the write direction
    if (!hbm && D * elem_bytes(dtype) >= 1024)
        plan.max_blocks = 512;         // the write direction's own optimum for long rows behind the host link
    const bool flat_ok = ud::flat_supports(N, D, pitch * elem_bytes(dtype), M);
    if (hbm && flat_ok && !tuning) {
        // streaming stores: +8% at 400- and 2408-byte rows, nothing on longer multiples of 128 bytes; rows up to
        // 256 bytes gain 4-14% from streaming stores together with two chunks per lane, longer rows lose 5% to
        // the second chunk
        plan.flags = UD_TUNE_FLAT_SOURCE | UD_TUNE_NT_STORE;
        plan.chunks_per_lane = D * elem_bytes(dtype) <= 256 ? 2 : kScatterFlatChunks;
        plan.max_blocks = kDefaultMaxBlocks;
    }
    if (tuning) {
        if (tuning->flags & ~(UD_TUNE_FLAT_SOURCE | UD_TUNE_NT_STORE))
            return UD_ERR_INVALID_ARG;
        if ((tuning->flags & UD_TUNE_NT_STORE) && !(tuning->flags & UD_TUNE_FLAT_SOURCE))
            return UD_ERR_INVALID_ARG;
        if (tuning->lanes_per_row < 0 || tuning->lanes_per_row > 64 ||
            (tuning->lanes_per_row && !is_pow2(tuning->lanes_per_row)))
            return UD_ERR_INVALID_ARG;
        if (tuning->chunks_per_lane < 0 || tuning->chunks_per_lane > 4 || tuning->rows_in_flight < 0 ||
            tuning->max_blocks < 0)
            return UD_ERR_INVALID_ARG;
        plan.flags = tuning->flags;
        if (tuning->flags & UD_TUNE_FLAT_SOURCE) {
            plan.chunks_per_lane = tuning->chunks_per_lane ? tuning->chunks_per_lane : kScatterFlatChunks;
            plan.max_blocks = kDefaultMaxBlocks;
            if (!flat_ok || plan.chunks_per_lane == 3)
                return UD_ERR_UNSUPPORTED;
        } else {
            if (tuning->lanes_per_row)
                plan.lanes_per_row = tuning->lanes_per_row;
            if (tuning->chunks_per_lane)
                plan.chunks_per_lane = tuning->chunks_per_lane;
            if (tuning->rows_in_flight)
                plan.rows_in_flight = tuning->rows_in_flight;
            else if (tuning->chunks_per_lane)
                plan.rows_in_flight = 1;
        }
        if (tuning->max_blocks)
            plan.max_blocks = tuning->max_blocks;
    }
    if (M == 0)
        return UD_OK;
    if (!table || !idx || !src)
        return UD_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(table) % elem_bytes(dtype) || reinterpret_cast<uintptr_t>(src) % elem_bytes(dtype) ||
        reinterpret_cast<uintptr_t>(idx) % (itype == UD_I64 ? 8 : 4))
        return UD_ERR_INVALID_ARG;
    ud::GatherArgs a{};
    a.table = static_cast<const char *>(table);
    a.N = N;
    a.D = D;
    a.idx = idx;
    a.itype = itype;
    a.M = M;
    a.out = const_cast<void *>(src);
    a.pitch_bytes = pitch * elem_bytes(dtype);
    a.group_iters = 1;
    const ud_status es = error_slot(static_cast<hipStream_t>(stream), false, &a.err);
    if (es != UD_OK)
        return es;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const hipError_t e = (plan.flags & UD_TUNE_FLAT_SOURCE) ? ud::launch_scatter_flat(a, elem_bytes(dtype), plan, s)
                                                            : ud::launch_scatter(a, elem_bytes(dtype), plan, s);
    if (e == hipErrorInvalidValue)
        return UD_ERR_UNSUPPORTED;
    if (e != hipSuccess)
        return hip_fail(e, "kernel launch");
    return UD_OK;
}

ud_status ud_scatter_tuned(void *table, int64_t N, int64_t D, ud_dtype dtype,
                           const void *idx, ud_itype itype, int64_t M,
                           const void *src, void *stream, const ud_tuning *tuning)
{
    return scatter_impl(table, N, D, D, dtype, idx, itype, M, src, stream, tuning);
}

ud_status ud_scatter(void *table, int64_t N, int64_t D, ud_dtype dtype,
                     const void *idx, ud_itype itype, int64_t M,
                     const void *src, void *stream)
{
    return scatter_impl(table, N, D, D, dtype, idx, itype, M, src, stream, nullptr);
}

ud_status ud_scatter_pitched(void *table, int64_t N, int64_t D, int64_t pitch, ud_dtype dtype,
                             const void *idx, ud_itype itype, int64_t M,
                             const void *src, void *stream)
{
    return scatter_impl(table, N, D, pitch, dtype, idx, itype, M, src, stream, nullptr);
}

ud_status ud_cache_create(const ud_table *table, const int64_t *hot_rows, int64_t n_hot, ud_cache **c)
{
    if (!table || !c || table->device_resident || n_hot < 1 || n_hot > table->N || n_hot > INT32_MAX || !hot_rows)
        return UD_ERR_INVALID_ARG;
    for (int64_t k = 0; k < n_hot; ++k)
        if (hot_rows[k] < 0 || hot_rows[k] >= table->N)
            return UD_ERR_INVALID_ARG;
    const int64_t row_bytes = table->D * elem_bytes(table->elem);
    ud_cache *h = new (std::nothrow) ud_cache{};
    if (!h)
        return UD_ERR_OOM;
    h->table = table->dev;
    h->N = table->N;
    h->D = table->D;
    h->pitch = table->pitch;
    h->elem = table->elem;
    h->n_hot = n_hot;
    int64_t *ids_dev = nullptr;
    ud_status st = UD_OK;
    hipError_t e = hipMalloc(&h->rows, static_cast<size_t>(n_hot) * static_cast<size_t>(row_bytes));
    if (e == hipSuccess)
        e = hipMalloc(reinterpret_cast<void **>(&h->slot), static_cast<size_t>(table->N) * sizeof(int32_t));
    if (e == hipSuccess)
        e = hipMalloc(reinterpret_cast<void **>(&ids_dev), static_cast<size_t>(n_hot) * sizeof(int64_t));
    if (e == hipSuccess)
        e = hipMemcpy(ids_dev, hot_rows, static_cast<size_t>(n_hot) * sizeof(int64_t), hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = hipMemset(h->slot, 0xff, static_cast<size_t>(table->N) * sizeof(int32_t)); // every row: slot -1
    if (e != hipSuccess)
        st = hip_fail(e, "ud_cache_create");
    // the cache is filled by the library's own zero-copy gather, then the map is scattered
    if (st == UD_OK)
        st = gather_impl(table->dev, table->N, table->D, table->pitch, table->elem, ids_dev, UD_I64, n_hot, h->rows, nullptr,
                         nullptr, nullptr, nullptr);
    if (st == UD_OK) {
        e = ud::launch_fill_slots(ids_dev, n_hot, h->slot, nullptr);
        if (e == hipSuccess)
            e = hipStreamSynchronize(nullptr);
        if (e != hipSuccess)
            st = hip_fail(e, "ud_cache_create(slot map)");
    }
    if (ids_dev)
        (void)hipFree(ids_dev);
    if (st != UD_OK) {
        (void)ud_cache_free(h);
        return st;
    }
    *c = h;
    return UD_OK;
}

ud_status ud_cache_free(ud_cache *c)
{
    if (!c)
        return UD_OK;
    hipError_t e1 = c->rows ? hipFree(c->rows) : hipSuccess;
    hipError_t e2 = c->slot ? hipFree(c->slot) : hipSuccess;
    delete c;
    if (e1 != hipSuccess)
        return hip_fail(e1, "hipFree(cache rows)");
    if (e2 != hipSuccess)
        return hip_fail(e2, "hipFree(cache map)");
    return UD_OK;
}

ud_status ud_gather_cached(const ud_cache *c, ud_dtype dtype, const void *idx, ud_itype itype, int64_t M,
                           void *out, void *stream)
{
    if (!c)
        return UD_ERR_INVALID_ARG;
    // the table's storage type must match the gather's input type
    if ((dtype == UD_F32) != (c->elem == UD_F32))
        return UD_ERR_INVALID_ARG;
    return gather_impl(c->table, c->N, c->D, c->pitch, dtype, idx, itype, M, out, stream, nullptr, c->slot,
                       static_cast<const char *>(c->rows));
}

ud_status ud_gather_status(void *stream, int64_t *bad_pos)
{
    if (bad_pos)
        *bad_pos = -1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int dev = 0;
    ud_status st = current_device(&dev);
    if (st != UD_OK)
        return st;
    // the stream may hold a slot in the allocated table, in the static one (ud_gather_noalloc), or in both
    unsigned long long *slot[2] = {nullptr, nullptr}, *res_host[2] = {nullptr, nullptr}, *res_dev[2] = {nullptr, nullptr};
    std::atomic<bool> *busy[2] = {nullptr, nullptr};
    {
        std::lock_guard<std::mutex> lock(g_err_mutex);
        DeviceState &d = g_dev[dev];
        SlotTable *tables[2] = {&d.heap, &d.fixed};
        for (int f = 0; f < kSlotTables; ++f) {
            const int k = tables[f]->words ? find_slot(*tables[f], s, false, f == 0) : -1;
            if (k < 0)
                continue;
            if (!d.result_host) {
                // one pinned word per slot of either table, so that status calls on different streams do not share one
                void *h = nullptr, *g = nullptr;
                hipError_t e = hipHostMalloc(&h, 2 * kErrSlots * sizeof(unsigned long long), hipHostMallocMapped | hipHostMallocCoherent);
                if (e == hipSuccess) {
                    e = hipHostGetDevicePointer(&g, h, 0);
                    if (e != hipSuccess)
                        (void)hipHostFree(h);
                }
                if (e != hipSuccess)
                    return hip_fail(e, "hipHostMalloc(status words)");
                d.result_host = static_cast<unsigned long long *>(h);
                d.result_dev = static_cast<unsigned long long *>(g);
            }
            slot[f] = tables[f]->words + k;
            if (k < kErrSlots - 1)
                busy[f] = &tables[f]->busy[k];
            res_host[f] = d.result_host + f * kErrSlots + k;
            res_dev[f] = d.result_dev + f * kErrSlots + k;
        }
    }
    hipError_t e;
    for (int f = 0; f < kSlotTables; ++f) {
        if (!slot[f])
            continue;
        // read and clear in one atomic step, ordered after this stream's gathers and before its next ones;
        // other streams' slots are not touched
        *res_host[f] = ud::kNoBadIndex;
        e = ud::launch_fetch_and_reset(slot[f], res_dev[f], s);
        if (e != hipSuccess)
            return hip_fail(e, "status kernel launch");
    }
    e = hipStreamSynchronize(s);
    if (e != hipSuccess)
        return hip_fail(e, "hipStreamSynchronize");
    // everything this stream launched is complete and its records are clear: until its next launch its
    // slots may be handed to another stream (a stream is driven by one thread at a time)
    for (int f = 0; f < kSlotTables; ++f)
        if (busy[f])
            busy[f]->store(false, std::memory_order_release);
    unsigned long long v = ud::kNoBadIndex;
    for (int f = 0; f < kSlotTables; ++f)
        if (slot[f]) {
            const unsigned long long x = *static_cast<volatile unsigned long long *>(res_host[f]);
            if (x < v)
                v = x;
        }
    if (v == ud::kNoBadIndex)
        return UD_OK;                       // nothing bad, or nothing was ever launched on this stream
    if (bad_pos)
        *bad_pos = static_cast<int64_t>(v);
    return UD_ERR_INDEX_OUT_OF_RANGE;
}

const char *ud_status_str(ud_status s)
{
    switch (s) {
    case UD_OK: return "UD_OK";
    case UD_ERR_INVALID_ARG: return "UD_ERR_INVALID_ARG";
    case UD_ERR_UNSUPPORTED: return "UD_ERR_UNSUPPORTED";
    case UD_ERR_OOM: return "UD_ERR_OOM";
    case UD_ERR_INDEX_OUT_OF_RANGE: return "UD_ERR_INDEX_OUT_OF_RANGE";
    case UD_ERR_HIP: return "UD_ERR_HIP";
    }
    return "UD_ERR_UNKNOWN";
}

const char *ud_last_hip_error(void) { return g_hip_msg; }

#ifndef UD_BUILD_ID
#define UD_BUILD_ID "unknown"
#endif
const char *ud_build_id(void) { return UD_BUILD_ID; }

} // extern "C"
