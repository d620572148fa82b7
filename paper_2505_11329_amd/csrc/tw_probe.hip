// Measurement aid: a streaming read / copy / write kernel launched with the same
// shape as the fused kernel (persistent grid of `budget` workgroups of 1024
// threads, one per compute unit, 16-byte accesses, several in flight per
// thread). It measures what a CU budget can move to and from HBM, the ceiling
// the fused kernel is compared with, and serves as the copy of known size that
// hardware byte counters are scaled against.
#include <atomic>

#include "tw_internal.h"

namespace tw {

static constexpr int kProbeThreads = 1024;
static constexpr unsigned kProbePadBytes = 96 * 1024;  // one workgroup per compute unit
static constexpr int kInFlight = 8;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int MODE>
__global__ __launch_bounds__(kProbeThreads) void probe_kernel(const u32x4 *src, u32x4 *dst, long long n_vec)
{
    const long long stride = static_cast<long long>(gridDim.x) * kProbeThreads;
    long long i = static_cast<long long>(blockIdx.x) * kProbeThreads + threadIdx.x;
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
        if ((threadIdx.x & 63) == 0) dst[blockIdx.x * (kProbeThreads / 64) + (threadIdx.x >> 6)] = acc;
    }
}

template <int MODE>
static tw_status launch_probe(const void *src, void *dst, int64_t bytes, unsigned grid, hipStream_t stream)
{
    auto kern = probe_kernel<MODE>;
    static std::atomic<int> allowed{0};
    if (!allowed.load(std::memory_order_acquire)) {
        TW_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                   hipFuncAttributeMaxDynamicSharedMemorySize,
                                   static_cast<int>(kProbePadBytes)));
        allowed.store(1, std::memory_order_release);
    }
    TW_HIP(launch_kernel(kern, dim3(grid), dim3(kProbeThreads), kProbePadBytes, stream,
                         static_cast<const u32x4 *>(src), static_cast<u32x4 *>(dst),
                         static_cast<long long>(bytes / 16)));
    return TW_OK;
}

}  // namespace tw

using namespace tw;

extern "C" tw_status tw_hbm_probe(const void *src, void *dst, int64_t bytes, int mode, int cu_budget,
                                  void *stream)
{
    if (mode != TW_PROBE_READ && mode != TW_PROBE_COPY && mode != TW_PROBE_WRITE) return TW_ERR_SHAPE;
    if (!dst || (mode != TW_PROBE_WRITE && !src)) return TW_ERR_NULL;
    if (bytes < 0 || bytes % 16 != 0) return TW_ERR_SHAPE;
    if (!aligned16(dst) || (src && !aligned16(src))) return TW_ERR_ALIGN;
    if (mode == TW_PROBE_COPY && ranges_overlap(src, static_cast<uint64_t>(bytes), dst, static_cast<uint64_t>(bytes)))
        return TW_ERR_ALIAS;
    if (bytes == 0) return TW_OK;
    int cus = 0;
    TW_TRY(current_cu_count(&cus));
    const unsigned grid = static_cast<unsigned>(resolve_budget(cu_budget, cus));
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (mode) {
    case TW_PROBE_READ: return launch_probe<TW_PROBE_READ>(src, dst, bytes, grid, s);
    case TW_PROBE_COPY: return launch_probe<TW_PROBE_COPY>(src, dst, bytes, grid, s);
    default: return launch_probe<TW_PROBE_WRITE>(src, dst, bytes, grid, s);
    }
}
