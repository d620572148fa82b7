// The pipeline the fused kernel replaces, kept as a measured ablation
// (TokenWeave, arXiv 2505.11329: Section 4.2 and Table 1 compare the fused
// kernel with "AllReduce, then RMSNorm"; Section 4.3 counts the standard
// RMSNorm's passes: two reads of the tensor and one write).
//
// Two launches, three passes over memory, bf16 tensors in between:
//   allreduce_kernel   t = bf16(p_0 + ... + p_{P-1})             P reads, 1 write
//   add_norm_kernel    x = t + residual; residual_out = bf16(x);  2 reads, 1 write
//                      s = rsqrt(mean(x^2) + eps)
//                      out = bf16((bf16(x) * s) * weight), with   1 read,  1 write
//                      bf16(x) read back from residual_out
// i.e. (P + 6) * 2H bytes per row against the fused kernel's (P + 3) * 2H. Both
// kernels run on the whole device with small workgroups; neither is confined to
// a CU budget. The results differ from the fused kernel's by the two extra
// roundings (t and the re-read x).
#include <mutex>

#include "tw_device.h"
#include "tw_internal.h"

namespace tw {

static constexpr int kUThreads = 256;
static constexpr int kUWaves = kUThreads / 64;

struct UnfusedParams {
    const void *partials[TW_MAX_P];
    const void *residual;
    const void *weight;
    void *sum;  // t
    void *out;
    void *residual_out;
    uint32_t n_bytes;  // rows of this launch * H * 2
    uint32_t n_rows;
    int hv;  // 16-byte vectors per row
    int P;
    float eps;
    float inv_h;
};

// Pass 1: elementwise over the launch's 16-byte vectors. PT > 0: P known at
// compile time, all P loads of a vector are issued together; PT == 0: any P.
template <int PT>
__global__ __launch_bounds__(kUThreads) void allreduce_kernel(const UnfusedParams prm)
{
    const __amdgpu_buffer_rsrc_t r_sum = make_rsrc(prm.sum, prm.n_bytes);
    const uint32_t stride = gridDim.x * kUThreads * 16u;
    for (uint32_t off = (blockIdx.x * kUThreads + threadIdx.x) * 16u; off < prm.n_bytes; off += stride) {
        float f[8];
        if constexpr (PT > 0) {
            u32x4 v[PT];
#pragma unroll
            for (int p = 0; p < PT; ++p) v[p] = ld(make_rsrc(prm.partials[p], prm.n_bytes), off);
            unpack8(v[0], f);
#pragma unroll
            for (int p = 1; p < PT; ++p) add8(v[p], f);
        } else {
            unpack8(ld(make_rsrc(prm.partials[0], prm.n_bytes), off), f);
            for (int p = 1; p < prm.P; ++p) add8(ld(make_rsrc(prm.partials[p], prm.n_bytes), off), f);
        }
        st(r_sum, off, pack8(f), false);
    }
}

// Passes 2 and 3: one workgroup per row at a time, Q vectors per thread.
template <int Q>
__global__ __launch_bounds__(kUThreads) void add_norm_kernel(const UnfusedParams prm)
{
    __shared__ float s_wave_sum[2][kUWaves];
    const int tid = threadIdx.x;
    const int hv = prm.hv;
    const __amdgpu_buffer_rsrc_t r_sum = make_rsrc(prm.sum, prm.n_bytes);
    const __amdgpu_buffer_rsrc_t r_res = make_rsrc(prm.residual, prm.n_bytes);
    const __amdgpu_buffer_rsrc_t r_out = make_rsrc(prm.out, prm.n_bytes);
    const __amdgpu_buffer_rsrc_t r_res_out = make_rsrc(prm.residual_out, prm.n_bytes);
    const __amdgpu_buffer_rsrc_t r_w = make_rsrc(prm.weight, static_cast<uint32_t>(hv) * 16u);

    uint32_t parity = 0;
    for (uint32_t row = blockIdx.x; row < prm.n_rows; row += gridDim.x, parity ^= 1u) {
        uint32_t off[Q];
        u32x4 a[Q], b[Q];
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            const int v = tid + j * kUThreads;
            off[j] = v < hv ? (row * static_cast<uint32_t>(hv) + v) * 16u : kOutOfRange;
            a[j] = ld(r_sum, off[j]);
            b[j] = ld(r_res, off[j]);
        }
        float ss = 0.0f;
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            float x[8];
            unpack8(a[j], x);
            add8(b[j], x);
#pragma unroll
            for (int e = 0; e < 8; ++e) ss = fmaf(x[e], x[e], ss);
            st(r_res_out, off[j], pack8(x), false);
        }
        ss = group_sum(ss, 6);
        if ((tid & 63) == 0) s_wave_sum[parity][tid >> 6] = ss;
        __syncthreads();
        float total = s_wave_sum[parity][0];
#pragma unroll
        for (int w = 1; w < kUWaves; ++w) total += s_wave_sum[parity][w];
        const float s = rsqrtf(total * prm.inv_h + prm.eps);

        // pass 3: the stored residual stream is read back, as a stand-alone
        // RMSNorm's second loop does
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            const int v = tid + j * kUThreads;
            const u32x4 xr = ld(r_res_out, off[j]);
            const u32x4 wv = __builtin_amdgcn_raw_buffer_load_b128(r_w, v < hv ? v * 16u : kOutOfRange, 0, 0);
            float x[8], w[8];
            unpack8(xr, x);
            unpack8(wv, w);
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = (x[e] * s) * w[e];
            st(r_out, off[j], pack8(x), false);
        }
    }
}

template <int PT>
static hipError_t launch_allreduce(const UnfusedParams &prm, unsigned grid, hipStream_t s)
{
    return launch_kernel(allreduce_kernel<PT>, dim3(grid), dim3(kUThreads), 0, s, prm);
}

template <int Q>
static hipError_t launch_add_norm(const UnfusedParams &prm, unsigned grid, hipStream_t s)
{
    return launch_kernel(add_norm_kernel<Q>, dim3(grid), dim3(kUThreads), 0, s, prm);
}


// Scratch of the entry point that allocates nothing: the all-reduce's bf16 output
// t lives in this file-scope array instead of a caller's buffer. Every GPU the
// library is loaded on holds its own copy until the process ends. In host code
// the array's name is only a handle for hipGetSymbolAddress: kernels and copies
// get the device address that call returned, kept per device.
static __device__ __align__(256) unsigned char scratch[TW_STATIC_SCRATCH_BYTES];

static std::mutex g_scratch_mu;
static void *g_scratch_ptr[kMaxDevices];  // nullptr = not looked up yet on that device

static tw_status static_scratch(void **ptr)
{
    int dev = 0;
    TW_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return hip_fail(hipErrorInvalidDevice, "tw_unfused.hip: device id out of range");
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        TW_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return hip_fail(hipErrorInvalidSymbol, "tw_unfused.hip: the scratch array has no device address");
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return TW_OK;
}

// Host-only checks of the unfused call that do not need the scratch address.
static tw_status validate_unfused(const tw_fused_args &a)
{
    TW_TRY(validate_fused(a));
    if (a.N > 0 && a.H > 8192) return TW_ERR_UNSUPPORTED;  // add_norm_kernel covers rows of up to 4 * 256 vectors
    return TW_OK;
}

// Both launches of the (already validated) pipeline, t going through sum_scratch.
static tw_status launch_unfused(const tw_fused_args &a, void *sum_scratch, hipStream_t s)
{
    const uint64_t bytes = static_cast<uint64_t>(a.N) * static_cast<uint64_t>(a.H) * 2u;
    for (int p = 0; p < a.P; ++p)
        if (ranges_overlap(sum_scratch, bytes, a.partials[p], bytes)) return TW_ERR_ALIAS;
    if (ranges_overlap(sum_scratch, bytes, a.residual, bytes) ||
        ranges_overlap(sum_scratch, bytes, a.weight, static_cast<uint64_t>(a.H) * 2u) ||
        ranges_overlap(sum_scratch, bytes, a.out, bytes) ||
        ranges_overlap(sum_scratch, bytes, a.residual_out, bytes))
        return TW_ERR_ALIAS;

    int cus = 0;
    TW_TRY(current_cu_count(&cus));
    const int hv = static_cast<int>(a.H / 8);
    const int64_t row_bytes = a.H * 2;
    const int64_t rows_per_launch = kMaxLaunchBytes / row_bytes;
    for (int64_t r0 = 0; r0 < a.N; r0 += rows_per_launch) {
        const int64_t n_rows = (a.N - r0 < rows_per_launch) ? a.N - r0 : rows_per_launch;
        const int64_t off = r0 * row_bytes;
        UnfusedParams prm;
        for (int p = 0; p < TW_MAX_P; ++p)
            prm.partials[p] = p < a.P ? static_cast<const char *>(a.partials[p]) + off : nullptr;
        prm.residual = static_cast<const char *>(a.residual) + off;
        prm.weight = a.weight;
        prm.sum = static_cast<char *>(sum_scratch) + off;
        prm.out = static_cast<char *>(a.out) + off;
        prm.residual_out = static_cast<char *>(a.residual_out) + off;
        prm.n_bytes = static_cast<uint32_t>(n_rows * row_bytes);
        prm.n_rows = static_cast<uint32_t>(n_rows);
        prm.hv = hv;
        prm.P = a.P;
        prm.eps = a.eps;
        prm.inv_h = 1.0f / static_cast<float>(a.H);

        // eight workgroups (32 waves) per compute unit fill it; fewer if the batch is small
        const int64_t n_vec = n_rows * hv;
        const int64_t wgs_full = static_cast<int64_t>(cus) * 8;
        int64_t g1 = (n_vec + kUThreads - 1) / kUThreads;
        if (g1 > wgs_full) g1 = wgs_full;
        switch (a.P) {
        case 1: TW_HIP(launch_allreduce<1>(prm, static_cast<unsigned>(g1), s)); break;
        case 2: TW_HIP(launch_allreduce<2>(prm, static_cast<unsigned>(g1), s)); break;
        case 4: TW_HIP(launch_allreduce<4>(prm, static_cast<unsigned>(g1), s)); break;
        case 8: TW_HIP(launch_allreduce<8>(prm, static_cast<unsigned>(g1), s)); break;
        default: TW_HIP(launch_allreduce<0>(prm, static_cast<unsigned>(g1), s)); break;
        }
        const int64_t g2 = n_rows < wgs_full ? n_rows : wgs_full;
        if (hv <= kUThreads) TW_HIP(launch_add_norm<1>(prm, static_cast<unsigned>(g2), s));
        else if (hv <= 2 * kUThreads) TW_HIP(launch_add_norm<2>(prm, static_cast<unsigned>(g2), s));
        else TW_HIP(launch_add_norm<4>(prm, static_cast<unsigned>(g2), s));
    }
    return TW_OK;
}

}  // namespace tw

using namespace tw;

extern "C" tw_status tw_reduce_add_rmsnorm_unfused(const tw_fused_args *args, void *sum_scratch, void *stream)
{
    if (!args) return TW_ERR_NULL;
    const tw_fused_args &a = *args;
    TW_TRY(validate_fused(a));
    if (a.N == 0) return TW_OK;
    if (!sum_scratch) return TW_ERR_NULL;
    if (!aligned16(sum_scratch)) return TW_ERR_ALIGN;
    TW_TRY(validate_unfused(a));
    return launch_unfused(a, sum_scratch, static_cast<hipStream_t>(stream));
}

extern "C" tw_status tw_reduce_add_rmsnorm_unfused_static(const tw_fused_args *args, void *stream)
{
    if (!args) return TW_ERR_NULL;
    const tw_fused_args &a = *args;
    TW_TRY(validate_unfused(a));
    // validate_fused has bounded N * H far below 2^62
    if (static_cast<uint64_t>(a.N) * static_cast<uint64_t>(a.H) * 2u > uint64_t(TW_STATIC_SCRATCH_BYTES))
        return TW_ERR_SHAPE;
    if (a.N == 0) return TW_OK;
    void *t = nullptr;
    TW_TRY(static_scratch(&t));
    return launch_unfused(a, t, static_cast<hipStream_t>(stream));
}
