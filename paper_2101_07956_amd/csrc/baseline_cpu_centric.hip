// Host baselines for the benchmark -- not part of the gather library.
//
//  * udb_cpu_centric_*: the data path PyTorch-Direct argues against (Section 3,
//    Figure 2a): CPU threads read the selected rows and write them back to back
//    into a temporary pinned buffer, a copy call sets up the DMA, and the GPU's
//    DMA engine pulls the buffer into GPU memory.  Both the plain form (gather
//    everything, then one copy) and a double-buffered form (gather slice k+1
//    while slice k is in flight) are timed, so the baseline is not a straw man.
//  * udb_h2d_peak / udb_d2d_peak: the copy rates used as rooflines -- the best
//    pinned-host -> device hipMemcpy rate (the host link's practical peak) and a
//    device -> device copy rate.
//
//  * udb_plain_copy: a plain streaming copy kernel of known size, the reference
//    against which hardware byte counters are scaled when profiling.
//
// Shares nothing with the gather kernels.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>

namespace {

using clk = std::chrono::steady_clock;
double seconds_since(clk::time_point t0) { return std::chrono::duration<double>(clk::now() - t0).count(); }

struct Ctx {
    char *staging[2];
    size_t staging_bytes; // each
    hipStream_t stream;
    hipEvent_t done[2];
};

// rows [lo, hi) of the ID list -> dst, row by row, split over `threads` threads
void cpu_gather_rows(const char *table, int64_t row_bytes, const int64_t *idx, int64_t lo, int64_t hi, char *dst,
                     int threads)
{
    const int64_t n = hi - lo;
    if (threads < 1)
        threads = 1;
    if (threads > n)
        threads = static_cast<int>(n > 0 ? n : 1);
    auto work = [&](int t) {
        const int64_t a = lo + n * t / threads, b = lo + n * (t + 1) / threads;
        for (int64_t i = a; i < b; ++i)
            std::memcpy(dst + (i - lo) * row_bytes, table + idx[i] * row_bytes, static_cast<size_t>(row_bytes));
    };
    if (threads == 1) {
        work(0);
        return;
    }
    std::vector<std::thread> pool;
    pool.reserve(threads - 1);
    for (int t = 1; t < threads; ++t)
        pool.emplace_back(work, t);
    work(0);
    for (auto &th : pool)
        th.join();
}

// dst[k] = src[k] for n 16-byte words, grid-stride
__global__ __launch_bounds__(256) void plain_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n)
{
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    for (size_t k = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; k < n; k += stride)
        dst[k] = src[k];
}

} // namespace

extern "C" {

// Enqueue a copy of `bytes` bytes (a multiple of 16; both pointers 16-byte
// aligned device pointers) on `stream`: reads `bytes`, writes `bytes`.
int udb_plain_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (bytes % 16 || !dst || !src)
        return 1;
    const size_t n = bytes / 16;
    if (n == 0)
        return 0;
    const unsigned blocks = static_cast<unsigned>(std::min<size_t>((n + 255) / 256, 256 * 32));
    hipLaunchKernelGGL(plain_copy_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), n);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

// Best and median rate (GB/s, 1e9 bytes) of `reps` synchronous pinned-host ->
// device copies of `bytes` bytes.  Allocates and frees its own buffers.
int udb_h2d_peak(size_t bytes, int reps, double *best_gbps, double *median_gbps)
{
    void *h = nullptr, *d = nullptr;
    if (hipHostMalloc(&h, bytes, hipHostMallocDefault) != hipSuccess)
        return 1;
    if (hipMalloc(&d, bytes) != hipSuccess) {
        (void)hipHostFree(h);
        return 1;
    }
    std::memset(h, 1, bytes);
    (void)hipMemcpy(d, h, bytes, hipMemcpyHostToDevice); // warm-up
    std::vector<double> rates;
    for (int r = 0; r < reps; ++r) {
        (void)hipDeviceSynchronize();
        const auto t0 = clk::now();
        if (hipMemcpy(d, h, bytes, hipMemcpyHostToDevice) != hipSuccess)
            break;
        (void)hipDeviceSynchronize();
        rates.push_back(static_cast<double>(bytes) / seconds_since(t0) / 1e9);
    }
    (void)hipFree(d);
    (void)hipHostFree(h);
    if (rates.empty())
        return 2;
    std::sort(rates.begin(), rates.end());
    *best_gbps = rates.back();
    *median_gbps = rates[rates.size() / 2];
    return 0;
}

// Same in the other direction: device -> pinned host.
int udb_d2h_peak(size_t bytes, int reps, double *best_gbps, double *median_gbps)
{
    void *h = nullptr, *d = nullptr;
    if (hipHostMalloc(&h, bytes, hipHostMallocDefault) != hipSuccess)
        return 1;
    if (hipMalloc(&d, bytes) != hipSuccess) {
        (void)hipHostFree(h);
        return 1;
    }
    (void)hipMemset(d, 1, bytes);
    (void)hipMemcpy(h, d, bytes, hipMemcpyDeviceToHost); // warm-up
    std::vector<double> rates;
    for (int r = 0; r < reps; ++r) {
        (void)hipDeviceSynchronize();
        const auto t0 = clk::now();
        if (hipMemcpy(h, d, bytes, hipMemcpyDeviceToHost) != hipSuccess)
            break;
        (void)hipDeviceSynchronize();
        rates.push_back(static_cast<double>(bytes) / seconds_since(t0) / 1e9);
    }
    (void)hipFree(d);
    (void)hipHostFree(h);
    if (rates.empty())
        return 2;
    std::sort(rates.begin(), rates.end());
    *best_gbps = rates.back();
    *median_gbps = rates[rates.size() / 2];
    return 0;
}

// Same for device -> device copies; the rate counts bytes copied once (the
// HBM traffic is twice that: one read and one write).
int udb_d2d_peak(size_t bytes, int reps, double *best_gbps, double *median_gbps)
{
    void *a = nullptr, *b = nullptr;
    if (hipMalloc(&a, bytes) != hipSuccess)
        return 1;
    if (hipMalloc(&b, bytes) != hipSuccess) {
        (void)hipFree(a);
        return 1;
    }
    (void)hipMemset(a, 1, bytes);
    (void)hipMemcpy(b, a, bytes, hipMemcpyDeviceToDevice);
    std::vector<double> rates;
    for (int r = 0; r < reps; ++r) {
        (void)hipDeviceSynchronize();
        const auto t0 = clk::now();
        if (hipMemcpy(b, a, bytes, hipMemcpyDeviceToDevice) != hipSuccess)
            break;
        (void)hipDeviceSynchronize();
        rates.push_back(static_cast<double>(bytes) / seconds_since(t0) / 1e9);
    }
    (void)hipFree(a);
    (void)hipFree(b);
    if (rates.empty())
        return 2;
    std::sort(rates.begin(), rates.end());
    *best_gbps = rates.back();
    *median_gbps = rates[rates.size() / 2];
    return 0;
}

// Two pinned staging buffers of staging_bytes each, one stream.
int udb_cpu_centric_create(size_t staging_bytes, void **ctx)
{
    Ctx *c = new Ctx{};
    c->staging_bytes = staging_bytes;
    for (int k = 0; k < 2; ++k)
        if (hipHostMalloc(reinterpret_cast<void **>(&c->staging[k]), staging_bytes, hipHostMallocDefault) != hipSuccess)
            return 1;
    if (hipStreamCreate(&c->stream) != hipSuccess)
        return 1;
    for (int k = 0; k < 2; ++k)
        if (hipEventCreateWithFlags(&c->done[k], hipEventDisableTiming) != hipSuccess)
            return 1;
    for (int k = 0; k < 2; ++k)
        std::memset(c->staging[k], 0, staging_bytes); // touch the pages once
    *ctx = c;
    return 0;
}

void udb_cpu_centric_destroy(void *ctx)
{
    Ctx *c = static_cast<Ctx *>(ctx);
    if (!c)
        return;
    for (int k = 0; k < 2; ++k) {
        (void)hipHostFree(c->staging[k]);
        (void)hipEventDestroy(c->done[k]);
    }
    (void)hipStreamDestroy(c->stream);
    delete c;
}

// One minibatch through the CPU-centric path.
//   table_host  CPU address of the table, row_bytes its row pitch
//   idx_host    M int64 IDs in CPU memory (validated by the caller)
//   out_dev     device pointer, M * row_bytes bytes
//   slices      1 = gather everything, then one copy; k > 1 = double-buffered
//               pipeline over k slices of rows
// Reports wall seconds: whole call, and (slices == 1 only) the gather and the
// copy phase separately.  Returns 0, or 1 if a slice does not fit the staging
// buffer, or 2 on a HIP error.
int udb_cpu_centric_gather(void *ctx, const void *table_host, int64_t row_bytes, const int64_t *idx_host, int64_t M,
                           void *out_dev, int threads, int slices, double *t_total, double *t_gather, double *t_copy)
{
    Ctx *c = static_cast<Ctx *>(ctx);
    if (slices < 1)
        slices = 1;
    const int64_t per = (M + slices - 1) / slices;
    if (static_cast<size_t>(per) * static_cast<size_t>(row_bytes) > c->staging_bytes)
        return 1;
    const char *table = static_cast<const char *>(table_host);
    char *out = static_cast<char *>(out_dev);
    *t_gather = *t_copy = 0.0;
    const auto t0 = clk::now();
    for (int k = 0; k < slices; ++k) {
        const int64_t lo = per * k, hi = std::min<int64_t>(M, per * (k + 1));
        if (lo >= hi)
            break;
        const int b = k & 1;
        if (k >= 2 && hipEventSynchronize(c->done[b]) != hipSuccess) // buffer b is free again
            return 2;
        const auto tg = clk::now();
        cpu_gather_rows(table, row_bytes, idx_host, lo, hi, c->staging[b], threads);
        *t_gather += seconds_since(tg);
        const auto tc = clk::now();
        if (hipMemcpyAsync(out + lo * row_bytes, c->staging[b], static_cast<size_t>(hi - lo) * row_bytes,
                           hipMemcpyHostToDevice, c->stream) != hipSuccess)
            return 2;
        if (hipEventRecord(c->done[b], c->stream) != hipSuccess)
            return 2;
        if (slices == 1) {
            if (hipStreamSynchronize(c->stream) != hipSuccess)
                return 2;
            *t_copy = seconds_since(tc);
        }
    }
    if (hipStreamSynchronize(c->stream) != hipSuccess)
        return 2;
    *t_total = seconds_since(t0);
    return 0;
}

} // extern "C"
