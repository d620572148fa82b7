// Measurement aid: a streaming read / copy / write kernel launched with the same
// shape as the fused kernel (persistent grid of `budget` workgroups of 1024
// threads, one per compute unit, 16-byte accesses, several in flight per
// thread); the workgroup size and the number of accesses in flight per thread
// can be varied, to show what the per-compute-unit ceiling does and does not
// depend on. It measures what a CU budget can move to and from HBM, the ceiling
// the fused kernel is compared with, and serves as the copy of known size that
// hardware byte counters are scaled against.
#include <atomic>

#include "tw_device.h"
#include "tw_internal.h"

namespace tw {

static constexpr int kProbeThreads = 1024;
static constexpr unsigned kProbePadBytes = 96 * 1024;  // one workgroup per compute unit

// kInFlight 16-byte accesses per thread are issued before the first is used;
// the workgroup has blockDim.x threads (a multiple of 64, at most 1024).
template <int MODE, int kInFlight>
__global__ __launch_bounds__(kProbeThreads) void probe_kernel(const u32x4 *src, u32x4 *dst, long long n_vec)
{
    const long long stride = static_cast<long long>(gridDim.x) * blockDim.x;
    long long i = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    const u32x4 pattern = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};

    for (; i + (kInFlight - 1) * stride < n_vec; i += kInFlight * stride) {
        if constexpr (MODE == TW_PROBE_WRITE) {
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) __builtin_nontemporal_store(pattern, dst + i + u * stride);
        } else {
            u32x4 v[kInFlight];
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                if constexpr (MODE == TW_PROBE_COPY) __builtin_nontemporal_store(v[u], dst + i + u * stride);
                else acc ^= v[u];
            }
        }
    }
    for (; i < n_vec; i += stride) {
        if constexpr (MODE == TW_PROBE_WRITE) {
            __builtin_nontemporal_store(pattern, dst + i);
        } else {
            const u32x4 v = __builtin_nontemporal_load(src + i);
            if constexpr (MODE == TW_PROBE_COPY) __builtin_nontemporal_store(v, dst + i);
            else acc ^= v;
        }
    }
    if constexpr (MODE == TW_PROBE_READ) {
        // fold the workgroup's lanes so that every load feeds the one word written
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            acc.x ^= __shfl_xor(acc.x, off, 64);
            acc.y ^= __shfl_xor(acc.y, off, 64);
            acc.z ^= __shfl_xor(acc.z, off, 64);
            acc.w ^= __shfl_xor(acc.w, off, 64);
        }
        if ((threadIdx.x & 63) == 0) dst[blockIdx.x * (kProbeThreads / 64) + (threadIdx.x >> 6)] = acc;  // 16 slots per workgroup
    }
}

// The fused kernel's traffic shape without its arithmetic: per 16 KiB "row" a
// workgroup reads NR streams and writes n_write streams at the same offset.
// Loads and stores carry the fused kernel's cache policies. What this reaches is
// the ceiling for any kernel with that mix of loads and stores at the given
// budget. NR is a template parameter so that exactly NR
// loads are issued per row (a run-time count would issue dead ones).
template <int NR>
__global__ __launch_bounds__(kProbeThreads) void probe_mixed_kernel(const char *src, char *dst,
                                                                    unsigned stream_bytes, int n_write)
{
    const unsigned row_bytes = blockDim.x * 16u;  // 16 KiB with the fused kernel's 1024 threads
    const unsigned rows = stream_bytes / row_bytes;
    u32x4 acc = {1u, 2u, 3u, 4u};
    for (unsigned row = blockIdx.x; row < rows; row += gridDim.x) {
        const unsigned off = row * row_bytes + threadIdx.x * 16u;
        u32x4 v[NR > 0 ? NR : 1];
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<char *>(src) + static_cast<size_t>(r) * stream_bytes, 0,
                static_cast<int>(stream_bytes), 0x00020000);
            v[r] = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, kStreamPolicy);
        }
        for (int wst = 0; wst < n_write; ++wst) {
            __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                dst + static_cast<size_t>(wst) * stream_bytes, 0, static_cast<int>(stream_bytes), 0x00020000);
            __builtin_amdgcn_raw_buffer_store_b128(acc, rs, off, 0, kStorePolicy);
        }
#pragma unroll
        for (int r = 0; r < NR; ++r) acc ^= v[r];
    }
    if (n_write == 0 && acc.x == 0x12345u && acc.y == 0x777u)
        reinterpret_cast<u32x4 *>(dst)[threadIdx.x] = acc;
}

// Occupies one wave for `ticks` of the device's constant-rate wall clock and does
// nothing else; gives up after max_iters polls whatever the clock says, so the
// wave always ends (each poll sleeps about a microsecond).
__global__ __launch_bounds__(64) void spin_kernel(unsigned long long ticks, unsigned max_iters)
{
    const unsigned long long t0 = wall_clock64();
    for (unsigned i = 0; i < max_iters; ++i) {
        if (wall_clock64() - t0 >= ticks) break;
        __builtin_amdgcn_s_sleep(32);
    }
}

template <int NR>
static tw_status launch_mixed(const void *src, void *dst, int64_t stream_bytes, int n_write, unsigned grid,
                              unsigned threads, hipStream_t stream)
{
    auto kern = probe_mixed_kernel<NR>;
    static std::atomic<int> allowed[kMaxDevices];
    TW_TRY(allow_dynamic_lds(reinterpret_cast<const void *>(kern), static_cast<int>(kProbePadBytes), allowed));
    TW_HIP(launch_kernel(kern, dim3(grid), dim3(threads), kProbePadBytes, stream,
                         static_cast<const char *>(src), static_cast<char *>(dst),
                         static_cast<unsigned>(stream_bytes), n_write));
    return TW_OK;
}

template <int NR>
static tw_status dispatch_mixed(int n_read, const void *src, void *dst, int64_t stream_bytes, int n_write,
                                unsigned grid, unsigned threads, hipStream_t stream)
{
    if (n_read == NR) return launch_mixed<NR>(src, dst, stream_bytes, n_write, grid, threads, stream);
    if constexpr (NR > 0)
        return dispatch_mixed<NR - 1>(n_read, src, dst, stream_bytes, n_write, grid, threads, stream);
    return TW_ERR_SHAPE;
}

template <int MODE, int DEPTH>
static tw_status launch_probe(const void *src, void *dst, int64_t bytes, unsigned grid, unsigned threads,
                              hipStream_t stream)
{
    auto kern = probe_kernel<MODE, DEPTH>;
    static std::atomic<int> allowed[kMaxDevices];
    TW_TRY(allow_dynamic_lds(reinterpret_cast<const void *>(kern), static_cast<int>(kProbePadBytes), allowed));
    TW_HIP(launch_kernel(kern, dim3(grid), dim3(threads), kProbePadBytes, stream,
                         static_cast<const u32x4 *>(src), static_cast<u32x4 *>(dst),
                         static_cast<long long>(bytes / 16)));
    return TW_OK;
}

template <int MODE>
static tw_status launch_probe_depth(int depth, const void *src, void *dst, int64_t bytes, unsigned grid,
                                    unsigned threads, hipStream_t stream)
{
    switch (depth) {
    case 1: return launch_probe<MODE, 1>(src, dst, bytes, grid, threads, stream);
    case 2: return launch_probe<MODE, 2>(src, dst, bytes, grid, threads, stream);
    case 4: return launch_probe<MODE, 4>(src, dst, bytes, grid, threads, stream);
    case 8: return launch_probe<MODE, 8>(src, dst, bytes, grid, threads, stream);
    case 16: return launch_probe<MODE, 16>(src, dst, bytes, grid, threads, stream);
    }
    return TW_ERR_UNSUPPORTED;
}

static bool probe_threads_ok(int threads) { return threads >= 64 && threads <= kProbeThreads && threads % 64 == 0; }

}  // namespace tw

using namespace tw;

extern "C" tw_status tw_hbm_probe_shaped(const void *src, void *dst, int64_t bytes, int mode, int cu_budget,
                                         int threads, int in_flight, void *stream)
{
    if (mode != TW_PROBE_READ && mode != TW_PROBE_COPY && mode != TW_PROBE_WRITE) return TW_ERR_SHAPE;
    if (!dst || (mode != TW_PROBE_WRITE && !src)) return TW_ERR_NULL;
    if (bytes < 0 || bytes % 16 != 0) return TW_ERR_SHAPE;
    if (!probe_threads_ok(threads)) return TW_ERR_SHAPE;
    if (in_flight != 1 && in_flight != 2 && in_flight != 4 && in_flight != 8 && in_flight != 16)
        return TW_ERR_UNSUPPORTED;
    if (!aligned16(dst) || (src && !aligned16(src))) return TW_ERR_ALIGN;
    if (mode == TW_PROBE_COPY && ranges_overlap(src, static_cast<uint64_t>(bytes), dst, static_cast<uint64_t>(bytes)))
        return TW_ERR_ALIAS;
    if (bytes == 0) return TW_OK;
    int cus = 0;
    TW_TRY(current_cu_count(&cus));
    const unsigned grid = static_cast<unsigned>(resolve_budget(cu_budget, cus));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned t = static_cast<unsigned>(threads);
    switch (mode) {
    case TW_PROBE_READ: return launch_probe_depth<TW_PROBE_READ>(in_flight, src, dst, bytes, grid, t, s);
    case TW_PROBE_COPY: return launch_probe_depth<TW_PROBE_COPY>(in_flight, src, dst, bytes, grid, t, s);
    default: return launch_probe_depth<TW_PROBE_WRITE>(in_flight, src, dst, bytes, grid, t, s);
    }
}

extern "C" tw_status tw_hbm_probe(const void *src, void *dst, int64_t bytes, int mode, int cu_budget,
                                  void *stream)
{
    return tw_hbm_probe_shaped(src, dst, bytes, mode, cu_budget, kProbeThreads, 8, stream);
}

extern "C" tw_status tw_hbm_probe_mixed_shaped(const void *src, void *dst, int64_t stream_bytes, int n_read,
                                               int n_write, int cu_budget, int threads, void *stream)
{
    if (n_read < 0 || n_read > TW_MAX_P + 1 || n_write < 0 || n_write > 4 || n_read + n_write == 0)
        return TW_ERR_SHAPE;
    if (!dst || (n_read > 0 && !src)) return TW_ERR_NULL;
    if (stream_bytes < 0 || stream_bytes % (kProbeThreads * 16) != 0 || stream_bytes > (int64_t(1) << 31))
        return TW_ERR_SHAPE;
    // a workgroup's row must divide the 16 KiB granule of stream_bytes
    if (!probe_threads_ok(threads) || kProbeThreads % threads != 0) return TW_ERR_SHAPE;
    if (!aligned16(dst) || (src && !aligned16(src))) return TW_ERR_ALIGN;
    if (n_read > 0 && n_write > 0 &&
        ranges_overlap(src, static_cast<uint64_t>(stream_bytes) * n_read, dst,
                       static_cast<uint64_t>(stream_bytes) * n_write))
        return TW_ERR_ALIAS;
    if (stream_bytes == 0) return TW_OK;
    int cus = 0;
    TW_TRY(current_cu_count(&cus));
    const unsigned grid = static_cast<unsigned>(resolve_budget(cu_budget, cus));
    return dispatch_mixed<TW_MAX_P + 1>(n_read, src, dst, stream_bytes, n_write, grid, static_cast<unsigned>(threads),
                                        static_cast<hipStream_t>(stream));
}

extern "C" tw_status tw_hbm_probe_mixed(const void *src, void *dst, int64_t stream_bytes, int n_read,
                                        int n_write, int cu_budget, void *stream)
{
    return tw_hbm_probe_mixed_shaped(src, dst, stream_bytes, n_read, n_write, cu_budget, kProbeThreads, stream);
}

extern "C" tw_status tw_streams_overlap(void *stream_a, void *stream_b, int *overlap)
{
    if (!overlap) return TW_ERR_NULL;
    *overlap = 0;
    if (stream_a == stream_b) return TW_OK;
    hipStream_t a = static_cast<hipStream_t>(stream_a), b = static_cast<hipStream_t>(stream_b);
    int dev = 0, khz = 0;
    TW_HIP(hipGetDevice(&dev));
    TW_HIP(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev));
    if (khz <= 0) khz = 100000;  // 100 MHz on this family
    const double spin_us = 300.0;
    const unsigned long long ticks = static_cast<unsigned long long>(spin_us * 1e-3 * khz);
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    tw_status st = TW_OK;
    float ms_a = 0.0f, ms_b = 0.0f;
    auto run = [&]() -> tw_status {
        for (auto &e : ev) TW_HIP(hipEventCreate(&e));
        // both kernels become runnable at the same point: after everything already on a
        TW_HIP(hipEventRecord(ev[0], a));
        TW_HIP(hipStreamWaitEvent(b, ev[0], 0));
        TW_HIP(launch_kernel(spin_kernel, dim3(1), dim3(64), 0u, a, ticks, 8192u));
        TW_HIP(hipEventRecord(ev[1], a));
        TW_HIP(launch_kernel(spin_kernel, dim3(1), dim3(64), 0u, b, ticks, 8192u));
        TW_HIP(hipEventRecord(ev[2], b));
        TW_HIP(hipEventSynchronize(ev[1]));
        TW_HIP(hipEventSynchronize(ev[2]));
        TW_HIP(hipEventElapsedTime(&ms_a, ev[0], ev[1]));
        TW_HIP(hipEventElapsedTime(&ms_b, ev[0], ev[2]));
        return TW_OK;
    };
    st = run();
    for (auto &e : ev)
        if (e) (void)hipEventDestroy(e);
    if (st != TW_OK) return st;
    // side by side both end about spin_us after the fork; one behind the other, the later ends at twice that
    const double later_us = 1e3 * (ms_a > ms_b ? ms_a : ms_b);
    *overlap = later_us < 1.6 * spin_us ? 1 : 0;
    return TW_OK;
}

extern "C" tw_status tw_stream_create_cu_masked(int first_cu, int n_cus, void **stream)
{
    if (!stream) return TW_ERR_NULL;
    *stream = nullptr;
    if (first_cu < 0 || n_cus < 1) return TW_ERR_SHAPE;
    int cus = 0;
    TW_TRY(current_cu_count(&cus));
    if (first_cu > cus - n_cus) return TW_ERR_SHAPE;
    constexpr int kMaxMaskWords = 32;  // 1024 compute units
    if (cus > 32 * kMaxMaskWords) return TW_ERR_UNSUPPORTED;
    uint32_t mask[kMaxMaskWords] = {};
    for (int b = first_cu; b < first_cu + n_cus; ++b) mask[b / 32] |= 1u << (b % 32);
    hipStream_t s = nullptr;
    TW_HIP(hipExtStreamCreateWithCUMask(&s, static_cast<uint32_t>((cus + 31) / 32), mask));
    *stream = s;
    return TW_OK;
}

extern "C" tw_status tw_stream_destroy(void *stream)
{
    if (!stream) return TW_ERR_NULL;
    TW_HIP(hipStreamDestroy(static_cast<hipStream_t>(stream)));
    return TW_OK;
}
