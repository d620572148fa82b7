// Internal declarations shared by libtw's translation units (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "tw.h"
#include "tw_measure.h"

namespace tw {

// Records e (and where it happened) as the calling thread's last HIP error and
// returns TW_ERR_HIP.
tw_status hip_fail(hipError_t e, const char *where);

#define TW_STR2(x) #x
#define TW_STR(x) TW_STR2(x)
#define TW_HIP(expr)                                  \
    do {                                              \
        hipError_t tw_e_ = (expr);                    \
        if (tw_e_ != hipSuccess)                      \
            return ::tw::hip_fail(tw_e_, __FILE_NAME__ ":" TW_STR(__LINE__) ": " #expr); \
    } while (0)

// Launches through the runtime's C entry point, whose return value belongs to
// this launch alone (the triple-chevron form reports through the thread's sticky
// "last error", which may be somebody else's).
template <typename... Params, typename... Args>
inline hipError_t launch_kernel(void (*kern)(Params...), dim3 grid, dim3 block, unsigned lds_bytes,
                                hipStream_t stream, Args... args)
{
    void *argv[] = {const_cast<void *>(static_cast<const void *>(&args))...};
    return hipLaunchKernel(reinterpret_cast<const void *>(kern), grid, block, argv, lds_bytes, stream);
}

// Kernels that ask for more than 64 KiB of dynamic LDS have to be allowed to,
// once per device. `done` is a per-kernel array of kMaxDevices flags.
static constexpr int kMaxDevices = 64;
tw_status allow_dynamic_lds(const void *kernel, int bytes, std::atomic<int> *done);

#define TW_TRY(expr)                                  \
    do {                                              \
        tw_status tw_s_ = (expr);                     \
        if (tw_s_ != TW_OK) return tw_s_;             \
    } while (0)

// Compute units of the current device (cached per device id).
tw_status current_cu_count(int *cu_count);

// Workgroups (= compute units) a budget stands for on a device with cu_count CUs.
inline int resolve_budget(int cu_budget, int cu_count)
{
    return (cu_budget <= 0 || cu_budget >= cu_count) ? cu_count : cu_budget;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Half-open byte ranges [a, a+alen) and [b, b+blen) intersect.
inline bool ranges_overlap(const void *a, uint64_t alen, const void *b, uint64_t blen)
{
    if (alen == 0 || blen == 0) return false;
    const uintptr_t pa = reinterpret_cast<uintptr_t>(a), pb = reinterpret_cast<uintptr_t>(b);
    return pa < pb + blen && pb < pa + alen;
}

// One launch addresses its tensors with 32-bit byte offsets; longer batches are
// cut into several launches on the host (rows are independent).
static constexpr int64_t kMaxLaunchBytes = int64_t(1) << 31;

// ---- fused reduce + residual add + RMSNorm (tw_fused.hip) ----
// Host-only argument checks; no HIP call.
tw_status validate_fused(const tw_fused_args &a);
// Launch geometry for H (hidden size): threads per row (power of two), vectors per
// thread, rows per workgroup iteration.
struct FusedGeometry {
    int hv;             // 16-byte vectors per row
    int tpr_log2;       // log2 of the row's vectors rounded up to a power of two (at most 1024)
    int vpt;            // vector columns per thread (1, 2, 4 or 8)
    int wpr;            // waves per row (rows wider than a wave), 0: 2^tpr_log2 lanes per row
    int rows_per_iter;  // rows one workgroup handles per loop trip
    int block;          // threads per workgroup: the waves that have columns to work on
};
FusedGeometry fused_geometry(int64_t H);
int64_t fused_grid_size(int64_t n_rows, const FusedGeometry &g, int budget_wgs);
// Enqueue rows [row_begin, row_end) of a (already validated) fused step.
tw_status launch_fused(const tw_fused_args &a, int64_t row_begin, int64_t row_end,
                       uint32_t *hw_ids, int64_t hw_ids_len, hipStream_t stream);

// ---- GEMM stand-in (tw_gemm.hip) ----
tw_status validate_gemm(const tw_gemm_args &g);
// `beside_other_kernels`: the launch is meant to overlap with another kernel (the
// fused step, a second GEMM): then the wide tiles are kept even where few of them
// fill the device.
tw_status launch_gemm(const tw_gemm_args &g, hipStream_t stream, bool beside_other_kernels = false);
static constexpr int kGemmTileM = 256, kGemmTileN = 128;


// ---- fork/join events (tw_host.hip) ----
// A small per-device pool of timing-disabled events used to order streams.
tw_status borrow_event(hipEvent_t *ev);

}  // namespace tw
