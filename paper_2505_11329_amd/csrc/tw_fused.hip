// Fused reduce over P partials + residual add + RMSNorm for gfx950
// (TokenWeave, arXiv 2505.11329: Section 4.3 and Appendix A, Listing 1).
//
// Per token row: x = (p_0 + ... + p_{P-1}) + residual in fp32; residual_out =
// bf16(x); s = rsqrt(mean(x^2) + eps); out = bf16((x * s) * weight). The paper's
// kernel lets the switch do the sum and re-reads the residual for the second
// loop; here the reading compute unit does the sum and x stays in registers, so
// every input byte is read once and every output byte written once.
//
// Shape of the launch
//   - One workgroup of up to 1024 threads (16 wave64) per compute unit, a persistent
//     grid of `budget` workgroups striding over groups of rows (Listing 1's
//     "token_id = blockIdx.x + iter * gridDim.x"). Each workgroup asks for more
//     than half of a compute unit's LDS, so two can never share one: the grid
//     size IS the number of compute units occupied.
//   - A row wider than a wave is covered by WPR whole waves (2 ... 16), each
//     thread owning VPT 16-byte vector columns (8 bf16); a workgroup handles
//     16/WPR rows per loop trip and is launched with just those waves. A narrower
//     row takes a power-of-two group of lanes. The thread->column map and the
//     reduction tree depend on H only, never on N, the grid or the row's
//     position: the same row gives the same bits in any launch (split or not,
//     any budget).
//   - Loads are software-pipelined two "chunks" deep (a chunk = the P+1 vectors
//     that feed one output vector): the loads of chunk q+2 are issued as soon as
//     chunk q has been summed, before the row's reduction and barrier, so a
//     thread always has P+1 .. 2(P+1) 16-byte loads in flight.
//   - Both outputs of a row are stored together once its scale is known (the new
//     residual stream could go out as soon as a chunk is summed, but loads that
//     are not interleaved with stores come in 1-1.5 % faster); rows of more than
//     16384 elements store it at once, for want of registers.
//   - Row sum of squares: per-thread fp32 FMAs, xor-butterfly across the lanes of
//     a wave (every lane ends with the same bits), and for rows wider than a
//     wave one LDS slot per wave and one barrier; slots are double-buffered by
//     row parity so one barrier per row suffices.
#include <atomic>

#include "tw_device.h"
#include "tw_internal.h"

namespace tw {

static constexpr int kThreads = 1024;
static constexpr int kWaves = kThreads / 64;
// Dynamic LDS each workgroup requests so that only one fits on a compute unit
// (gfx950 has 160 KiB per CU).
static constexpr unsigned kOccupancyPadBytes = 96 * 1024;
static constexpr int64_t kLastLevelCacheBytes = int64_t(256) << 20;

struct FusedParams {
    const void *partials[TW_MAX_P];
    const void *residual;
    const void *weight;
    void *out;
    void *residual_out;
    uint32_t *hw_ids;
    uint32_t n_bytes;      // rows of this launch * H * 2
    uint32_t group_bytes;  // rows_per_iter * H * 2
    uint32_t n_groups;     // ceil(rows / rows_per_iter)
    int hv;                // 16-byte vectors per row
    int P;
    int tpr_log2;          // rows of at most 64 vectors (and the thin kernel): 2^tpr_log2 lanes per row
    int wpr;               // wide kernel, rows wider than a wave: waves per row; else 0
    float eps;
    float inv_h;
};

// The P+1 vectors that feed one output vector, in flight.
template <int PT>
struct Chunk {
    u32x4 v[PT + 1];
};

// How many chunks are kept in flight per thread (register budget: 128 VGPRs).
template <int PT, int VPT>
constexpr int buffers_in_flight()
{
    return (PT == 0) ? 1 : (((PT + 1) * 8 + 12 * VPT <= 100) ? 2 : 1);
}

template <int PT, int VPT, bool TRACE, bool STREAMED>
__global__ __launch_bounds__(kThreads) void fused_kernel(const FusedParams prm)
{
    constexpr bool streamed = STREAMED;  // see st()
    __shared__ float s_wave_sum[2][kWaves];
    constexpr int NB = buffers_in_flight<PT, VPT>();
    constexpr bool KEEP_W = VPT <= 2;     // weights unpacked to fp32 once, else kept packed,
    constexpr bool RELOAD_W = VPT >= 8;  // or (no registers left) re-read through the cache per row
    constexpr bool LATE_RES = VPT <= 2;  // the new residual stream is stored with the output (wide rows: at once, or registers run out)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int tpr_log2 = prm.tpr_log2;
    // Rows wider than a wave take wpr whole waves each (any number up to 16: the
    // workgroup is launched with just the waves that have columns to work on, an
    // idle wave's out-of-range loads and stores would still cost L1 request
    // slots); narrower rows take a power-of-two group of lanes.
    const int wpr = prm.wpr;
    const int tpr = wpr ? wpr << 6 : 1 << tpr_log2;
    const int row_in_iter = wpr ? __builtin_amdgcn_readfirstlane(wave / wpr) : tid >> tpr_log2;
    const int col0 = wpr ? tid - row_in_iter * tpr : tid & (tpr - 1);
    const int hv = prm.hv;

    if (TRACE && tid == 0) {
        // HW_ID (hwreg 4) and XCC_ID (hwreg 20), all 32 bits of each.
        prm.hw_ids[2 * blockIdx.x] = __builtin_amdgcn_s_getreg(4 | (0 << 6) | (31 << 11));
        prm.hw_ids[2 * blockIdx.x + 1] = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (31 << 11));
    }

    __amdgpu_buffer_rsrc_t r_part[PT > 0 ? PT : 1];
    if constexpr (PT > 0) {
#pragma unroll
        for (int p = 0; p < PT; ++p) r_part[p] = make_rsrc(prm.partials[p], prm.n_bytes);
    }
    const __amdgpu_buffer_rsrc_t r_res = make_rsrc(prm.residual, prm.n_bytes);
    const __amdgpu_buffer_rsrc_t r_out = make_rsrc(prm.out, prm.n_bytes);
    const __amdgpu_buffer_rsrc_t r_res_out = make_rsrc(prm.residual_out, prm.n_bytes);

    // Byte offset of this thread's vector j inside a row group; columns past the
    // end of the row are pushed out of range for good.
    uint32_t lane_off[VPT];
    bool cvalid[VPT];
    u32x4 wv[RELOAD_W ? 1 : VPT];
    float wf[KEEP_W ? VPT : 1][8];
    const __amdgpu_buffer_rsrc_t r_w = make_rsrc(prm.weight, static_cast<uint32_t>(hv) * 16u);
    auto load_w = [&](int j) {
        return __builtin_amdgcn_raw_buffer_load_b128(r_w, cvalid[j] ? (col0 + j * tpr) * 16u : kOutOfRange, 0, 0);
    };
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
        const int v = col0 + j * tpr;
        cvalid[j] = v < hv;
        lane_off[j] = static_cast<uint32_t>(row_in_iter * hv + v) * 16u;
        if constexpr (!RELOAD_W) wv[j] = load_w(j);
        if constexpr (KEEP_W) unpack8(wv[j], wf[j]);
    }

    const uint32_t stride = gridDim.x;
    const uint32_t n_groups = prm.n_groups;
    const uint32_t group_bytes = prm.group_bytes;

    // Offset of chunk (group, j). A group at or past n_groups lands at or past
    // n_bytes (the host keeps n_bytes + 2 * stride * group_bytes below 2^32), so
    // prefetching past the end reads zeros and never needs a branch.
    auto chunk_off = [&](uint32_t group, int j) -> uint32_t {
        return cvalid[j] ? lane_off[j] + group * group_bytes : kOutOfRange;
    };
    // The loads of one chunk are kept together and in program order (the
    // scheduling barriers): the wait for chunk q must not also wait for q + 1.
    auto issue = [&](Chunk<PT> &c, uint32_t off) {
        if constexpr (PT > 0) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int p = 0; p < PT; ++p) c.v[p] = ld(r_part[p], off);
            c.v[PT] = ld(r_res, off);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // x = (p_0 + p_1 + ... + p_{P-1}) + residual, left to right, fp32.
    auto reduce_chunk = [&](const Chunk<PT> &c, uint32_t off, float (&x)[8]) {
        if constexpr (PT > 0) {
            unpack8(c.v[0], x);
#pragma unroll
            for (int p = 1; p < PT; ++p) add8(c.v[p], x);
            add8(c.v[PT], x);
        } else {
            // P known only at run time: four loads at a time, padded with
            // zero-length descriptors (which read as +0.0 and fetch nothing).
            // (Eight at a time measured 4 % slower at P = 12 and 16.)
            constexpr int kBatch = 4;
            const u32x4 r = ld(r_res, off);
            for (int p0 = 0; p0 < prm.P; p0 += kBatch) {
                u32x4 t[kBatch];
#pragma unroll
                for (int i = 0; i < kBatch; ++i) {
                    const bool live = p0 + i < prm.P;
                    t[i] = ld(make_rsrc(prm.partials[live ? p0 + i : 0], live ? prm.n_bytes : 0u), off);
                }
                if (p0 == 0) unpack8(t[0], x); else add8(t[0], x);
#pragma unroll
                for (int i = 1; i < kBatch; ++i) add8(t[i], x);
            }
            add8(r, x);
        }
    };

    // Chunks are numbered q = trip * VPT + j; trip t handles row group
    // blockIdx.x + t * gridDim.x. NB chunk buffers rotate, chunk q sits in buffer
    // q % NB; a loop body covers a multiple of NB chunks (two trips when VPT == 1).
    constexpr int TRIPS = (VPT == 1 && NB == 2) ? 2 : 1;
    Chunk<PT> buf[NB];
    if constexpr (NB == 2) {
        if constexpr (VPT == 1) {
            issue(buf[0], chunk_off(blockIdx.x, 0));
            issue(buf[1], chunk_off(blockIdx.x + stride, 0));
        } else {
            issue(buf[0], chunk_off(blockIdx.x, 0));
            issue(buf[1], chunk_off(blockIdx.x, 1));
        }
    } else {
        issue(buf[0], chunk_off(blockIdx.x, 0));
    }

    int parity = 0;
    for (uint32_t g0 = blockIdx.x; g0 < n_groups; g0 += stride * TRIPS) {
#pragma unroll
        for (int t = 0; t < TRIPS; ++t) {
            const uint32_t group = g0 + t * stride;
            float x[VPT][8];
            float ss = 0.0f;
#pragma unroll
            for (int j = 0; j < VPT; ++j) {
                Chunk<PT> &b = buf[(t * VPT + j) % NB];
                const uint32_t off = chunk_off(group, j);
                reduce_chunk(b, off, x[j]);
                // refill this buffer with chunk q + NB
                const int nj = (j + NB) % VPT;
                const uint32_t ng = (VPT == 1) ? group + NB * stride : (j + NB >= VPT ? group + stride : group);
                issue(b, chunk_off(ng, nj));
                if constexpr (!LATE_RES) st(r_res_out, off, pack8(x[j]), streamed);
#pragma unroll
                for (int e = 0; e < 8; ++e) ss = __builtin_fmaf(x[j][e], x[j][e], ss);
            }

            // Row sum of squares: the row's lanes inside this wave, then (rows
            // wider than a wave) the row's waves through LDS.
            ss = group_sum(ss, wpr ? 6 : tpr_log2);
            if (wpr) {
                // the row's wave sums, padded with zeros to 16, through a 16-lane butterfly
                if (lane == 0) s_wave_sum[parity][wave] = ss;
                __syncthreads();
                const int k = lane & 15;
                const float part = k < wpr ? s_wave_sum[parity][row_in_iter * wpr + k] : 0.0f;
                ss = group_sum(part, 4);
                parity ^= 1;
            }
            const float s = rsqrtf(ss * prm.inv_h + prm.eps);

#pragma unroll
            for (int j = 0; j < VPT; ++j) {
                float y[8];
                if constexpr (KEEP_W) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) y[e] = (x[j][e] * s) * wf[j][e];
                } else {
                    float w[8];
                    if constexpr (RELOAD_W) unpack8(load_w(j), w);
                    else unpack8(wv[j], w);
#pragma unroll
                    for (int e = 0; e < 8; ++e) y[e] = (x[j][e] * s) * w[e];
                }
                if constexpr (LATE_RES) st(r_res_out, chunk_off(group, j), pack8(x[j]), streamed);
                st(r_out, chunk_off(group, j), pack8(y), streamed);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// The same arithmetic in workgroups small enough to sit NEXT TO a GEMM workgroup
// on the same compute unit (256 threads, at most 128 VGPRs, 128 bytes of LDS): the
// "shared" launch mode. Instead of taking a few compute units away from the
// GEMM, the fused kernel is spread thinly over all of them and uses the HBM
// bandwidth the matrix-core-bound GEMM leaves idle. (The GEMM's two waves per
// SIMD hold 2 x 167 registers per lane, which leaves room for one such wave.)
//
// Bits are identical to fused_kernel's: a thread here plays Q (a row's vectors
// over 256, rounded up: 1 ... 4) of the wide kernel's threads (columns tid,
// tid+256, ...), keeps one sum of squares
// per played thread, and the reduction runs the very same tree (64-lane
// butterfly per played wave, then the 16-lane butterfly over the row's wave
// sums in LDS). Only rows of at most 1024 vectors (H <= 8192) are handled.
// With an even Q two chunks of loads are in flight per thread (chunk c sits in
// buffer c & 1, which needs no run-time index because every row then starts on
// buffer 0), with an odd Q one. Both outputs of a row are stored together once
// its scale is known: a small launch is one wave of workgroups that all run in
// step, and reads that are not interleaved with stores come in faster (a
// 1024-row, H = 8192, P = 8 launch: 33.5 -> 32.2 us with both changes, 256 rows
// 10.6 -> 9.7 us).
// ---------------------------------------------------------------------------
static constexpr int kThinThreads = 256;
// The all-at-once form is taken by whole-device launches of at most one workgroup per compute
// unit whose inputs come to at most this many bytes. Measured on MI355X, H = 8192, trains of
// launches replayed from a graph: P = 8 up to 48 rows 4.4-4.7 us a launch against 5.0-5.2
// (-11 %), at 256 rows 7.1 against 6.5 (+8 %): beyond a few MB the requests of a launch queue up
// and two chunks at a time come in faster.
static constexpr int64_t kDeepInputBytes = 6 << 20;

// DEEP: the form for batches so small that a launch is one round trip to memory
// and back (decode steps, Appendix B): a workgroup has one row group only, every
// chunk of it is requested at once together with the weights, and nothing is
// refilled. It needs ~200 registers, so it is a kernel of its own
// (fused_deep_kernel) without the 128-register bound that lets the other one
// sit beside a GEMM workgroup. Same arithmetic in the same order: same bits.
template <int PT, int Q, bool TRACE, bool STREAMED, bool DEEP>
__device__ __forceinline__ void thin_body(const FusedParams &prm)
{
    constexpr bool streamed = STREAMED;  // see st()
    __shared__ float s_wave_sum[2][kWaves];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int tpr_log2 = prm.tpr_log2;
    const int tpr = 1 << tpr_log2;
    const int hv = prm.hv;
    // Q > 1: the whole workgroup covers one row, thread plays columns tid + 256 q.
    // Q == 1: rows of at most 256 vectors, 256 / tpr of them per workgroup.
    const int row_in_iter = (Q > 1) ? 0 : (tid >> tpr_log2);
    const int col0 = (Q > 1) ? tid : (tid & (tpr - 1));

    if (TRACE && tid == 0) {
        prm.hw_ids[2 * blockIdx.x] = __builtin_amdgcn_s_getreg(4 | (0 << 6) | (31 << 11));
        prm.hw_ids[2 * blockIdx.x + 1] = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (31 << 11));
    }

    // The weights are re-read for every row with ordinary (cached) loads: the
    // streamed tensors are loaded "nt" and do not displace them from the L1, and
    // neither registers nor LDS are spent on them, which is what lets this
    // workgroup fit beside a GEMM workgroup that uses 144 KiB of LDS.
    const __amdgpu_buffer_rsrc_t r_w = make_rsrc(prm.weight, static_cast<uint32_t>(hv) * 16u);

    __amdgpu_buffer_rsrc_t r_part[PT > 0 ? PT : 1];
    if constexpr (PT > 0) {
#pragma unroll
        for (int p = 0; p < PT; ++p) r_part[p] = make_rsrc(prm.partials[p], prm.n_bytes);
    }
    const __amdgpu_buffer_rsrc_t r_res = make_rsrc(prm.residual, prm.n_bytes);
    const __amdgpu_buffer_rsrc_t r_out = make_rsrc(prm.out, prm.n_bytes);
    const __amdgpu_buffer_rsrc_t r_res_out = make_rsrc(prm.residual_out, prm.n_bytes);

    uint32_t lane_off[Q];
    bool cvalid[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const int v = col0 + q * kThinThreads;
        cvalid[q] = v < hv;
        lane_off[q] = static_cast<uint32_t>(row_in_iter * hv + v) * 16u;
    }
    const uint32_t group_bytes = prm.group_bytes;
    auto chunk_off = [&](uint32_t group, int q) -> uint32_t {
        return cvalid[q] ? lane_off[q] + group * group_bytes : kOutOfRange;
    };
    auto issue = [&](Chunk<PT> &c, uint32_t off) {
        if constexpr (PT > 0) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int p = 0; p < PT; ++p) c.v[p] = ld(r_part[p], off);
            c.v[PT] = ld(r_res, off);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto reduce_chunk = [&](const Chunk<PT> &c, uint32_t off, float (&x)[8]) {
        if constexpr (PT > 0) {
            unpack8(c.v[0], x);
#pragma unroll
            for (int p = 1; p < PT; ++p) add8(c.v[p], x);
            add8(c.v[PT], x);
        } else {
            // any P: eight loads at a time, padded with zero-length descriptors; a
            // thread here has four times the wide kernel's work per row and fewer
            // waves to hide a round trip behind (four at a time: 10-25 % slower)
            constexpr int kBatch = 8;
            const u32x4 r = ld(r_res, off);
            for (int p0 = 0; p0 < prm.P; p0 += kBatch) {
                u32x4 t[kBatch];
#pragma unroll
                for (int i = 0; i < kBatch; ++i) {
                    const bool live = p0 + i < prm.P;
                    t[i] = ld(make_rsrc(prm.partials[live ? p0 + i : 0], live ? prm.n_bytes : 0u), off);
                }
                if (p0 == 0) unpack8(t[0], x); else add8(t[0], x);
#pragma unroll
                for (int i = 1; i < kBatch; ++i) add8(t[i], x);
            }
            add8(r, x);
        }
    };

    // This workgroup's row groups: blockIdx.x, blockIdx.x + gridDim.x, ... The
    // workgroups resident at one time then read neighbouring rows of every stream,
    // which the memory system likes better than each workgroup walking a block of
    // its own (4-9 % at 8K rows and more).
    const uint32_t first = blockIdx.x;
    const uint32_t gstride = gridDim.x;
    const uint32_t last = prm.n_groups;
    // Chunks in flight: NB. Chunk (group, q) sits in buffer q % NB and is refilled
    // with the chunk NB further on: the same row's, or the workgroup's next row's;
    // after its last row nothing is fetched.
    constexpr int NB = DEEP ? Q : (Q % 2 == 0) ? 2 : 1;
    static_assert(!DEEP || PT > 0, "the run-time loop over P keeps nothing in flight");
    auto off_or_none = [&](uint32_t group, int q) -> uint32_t {
        return group < last ? chunk_off(group, q) : kOutOfRange;
    };
    Chunk<PT> buf[NB];
    issue(buf[0], off_or_none(first, 0));
    if constexpr (NB >= 2) issue(buf[1], off_or_none(first, 1));
    if constexpr (NB >= 3) issue(buf[2], off_or_none(first, 2));
    if constexpr (NB >= 4) issue(buf[3], off_or_none(first, 3));
    static_assert(NB <= 4, "chunks issued above");
    u32x4 w_ahead[DEEP ? Q : 1];
    if constexpr (DEEP) {
#pragma unroll
        for (int q = 0; q < Q; ++q)
            w_ahead[q] = __builtin_amdgcn_raw_buffer_load_b128(
                r_w, cvalid[q] ? (col0 + q * kThinThreads) * 16u : kOutOfRange, 0, 0);
    }
    int parity = 0;
    for (uint32_t group = first; group < last; group += gstride) {
        float x[Q][8];
        float ss[Q];
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            Chunk<PT> &b = buf[q % NB];
            reduce_chunk(b, chunk_off(group, q), x[q]);
            if constexpr (!DEEP)
                issue(b, (q + NB < Q) ? chunk_off(group, q + NB) : off_or_none(group + gstride, q + NB - Q));
            float acc = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc = __builtin_fmaf(x[q][e], x[q][e], acc);
            ss[q] = group_sum(acc, tpr_log2 < 6 ? tpr_log2 : 6);
        }
        float total = ss[0];
        if (tpr_log2 > 6) {
            if (lane == 0) {
#pragma unroll
                for (int q = 0; q < Q; ++q) s_wave_sum[parity][wave + q * (kThinThreads / 64)] = ss[q];
            }
            __syncthreads();
            // the played waves' sums, padded with zeros to 16, as in the wide kernel
            const int waves_per_row = (Q > 1) ? Q * (kThinThreads / 64) : tpr >> 6;
            const int k = lane & 15;
            const float part = k < waves_per_row ? s_wave_sum[parity][row_in_iter * waves_per_row + k] : 0.0f;
            total = group_sum(part, 4);
            parity ^= 1;
        }
        const float s = rsqrtf(total * prm.inv_h + prm.eps);
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            float w[8], y[8];
            const int v = col0 + q * kThinThreads;
            if constexpr (DEEP) unpack8(w_ahead[q], w);
            else unpack8(__builtin_amdgcn_raw_buffer_load_b128(r_w, cvalid[q] ? v * 16u : kOutOfRange, 0, 0), w);
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] = (x[q][e] * s) * w[e];
            st(r_res_out, chunk_off(group, q), pack8(x[q]), streamed);
            st(r_out, chunk_off(group, q), pack8(y), streamed);
        }
    }
}

template <int PT, int Q, bool TRACE, bool STREAMED>
__global__ __launch_bounds__(kThinThreads) __attribute__((amdgpu_waves_per_eu(4)))
void fused_thin_kernel(const FusedParams prm)
{
    thin_body<PT, Q, TRACE, STREAMED, false>(prm);
}

template <int PT, int Q>
__global__ __launch_bounds__(kThinThreads) void fused_deep_kernel(const FusedParams prm)
{
    thin_body<PT, Q, false, false, true>(prm);
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

FusedGeometry fused_geometry(int64_t H)
{
    FusedGeometry g;
    g.hv = static_cast<int>(H / 8);
    int l2 = 0;
    while ((1 << l2) < g.hv && l2 < 10) ++l2;
    g.tpr_log2 = l2;
    if (g.hv <= 64) {  // several rows per wave, or one
        g.vpt = 1;
        g.wpr = 0;
        g.rows_per_iter = kThreads >> l2;
        g.block = kThreads;
        return g;
    }
    const int need = (g.hv + kThreads - 1) / kThreads;  // 1..8
    g.vpt = need <= 1 ? 1 : need <= 2 ? 2 : need <= 4 ? 4 : 8;
    g.wpr = (g.hv + 64 * g.vpt - 1) / (64 * g.vpt);  // 2..16
    g.rows_per_iter = kWaves / g.wpr;
    g.block = g.rows_per_iter * g.wpr * 64;
    return g;
}

int64_t fused_grid_size(int64_t n_rows, const FusedGeometry &g, int budget_wgs)
{
    if (n_rows <= 0) return 0;
    const int64_t groups = (n_rows + g.rows_per_iter - 1) / g.rows_per_iter;
    return groups < budget_wgs ? groups : budget_wgs;
}

tw_status validate_fused(const tw_fused_args &a)
{
    if (a.P < 1 || a.P > TW_MAX_P) return TW_ERR_SHAPE;
    if (a.N < 0 || a.H <= 0) return TW_ERR_SHAPE;
    if (!(a.eps >= 0.0f) || !(a.eps <= 3.402823466e+38f)) return TW_ERR_SHAPE;  // rejects NaN, Inf, < 0
    if (a.H % 8 != 0 || a.H > TW_MAX_H) return TW_ERR_UNSUPPORTED;
    if (a.N > (INT64_MAX / 2) / a.H) return TW_ERR_SHAPE;
    if (!a.weight) return TW_ERR_NULL;
    if (!aligned16(a.weight)) return TW_ERR_ALIGN;
    // The [N x H] tensors of an empty batch have no storage to point at.
    if (a.N == 0) return TW_OK;
    if (!a.partials || !a.residual || !a.out || !a.residual_out) return TW_ERR_NULL;
    for (int p = 0; p < a.P; ++p)
        if (!a.partials[p]) return TW_ERR_NULL;
    if (!aligned16(a.residual) || !aligned16(a.out) || !aligned16(a.residual_out)) return TW_ERR_ALIGN;
    for (int p = 0; p < a.P; ++p)
        if (!aligned16(a.partials[p])) return TW_ERR_ALIGN;

    const uint64_t tensor = static_cast<uint64_t>(a.N) * static_cast<uint64_t>(a.H) * 2u;
    const uint64_t wbytes = static_cast<uint64_t>(a.H) * 2u;
    if (ranges_overlap(a.out, tensor, a.residual_out, tensor)) return TW_ERR_ALIAS;
    const void *outs[2] = {a.out, a.residual_out};
    for (int o = 0; o < 2; ++o) {
        if (ranges_overlap(outs[o], tensor, a.weight, wbytes)) return TW_ERR_ALIAS;
        // residual: only residual_out may coincide with it, and only exactly
        if (ranges_overlap(outs[o], tensor, a.residual, tensor) &&
            !(o == 1 && a.residual_out == a.residual))
            return TW_ERR_ALIAS;
        // partials: only out may coincide with one, and only exactly
        for (int p = 0; p < a.P; ++p)
            if (ranges_overlap(outs[o], tensor, a.partials[p], tensor) &&
                !(o == 0 && a.out == a.partials[p]))
                return TW_ERR_ALIAS;
    }
    return TW_OK;
}

template <int PT, int VPT>
static tw_status launch_t(const FusedParams &prm, bool trace, bool streamed, int64_t grid, int block, hipStream_t stream)
{
    auto kern = trace ? fused_kernel<PT, VPT, true, false>
                      : streamed ? fused_kernel<PT, VPT, false, true> : fused_kernel<PT, VPT, false, false>;
    static std::atomic<int> allowed[2][kMaxDevices];
    TW_TRY(allow_dynamic_lds(reinterpret_cast<const void *>(kern), static_cast<int>(kOccupancyPadBytes),
                             allowed[trace]));
    TW_HIP(launch_kernel(kern, dim3(static_cast<unsigned>(grid)), dim3(static_cast<unsigned>(block)),
                         kOccupancyPadBytes, stream, prm));
    return TW_OK;
}

template <int PT, int Q>
static tw_status launch_thin_t(const FusedParams &prm, bool trace, bool streamed, int64_t grid,
                               hipStream_t stream)
{
    auto kern = trace ? fused_thin_kernel<PT, Q, true, false>
                      : streamed ? fused_thin_kernel<PT, Q, false, true> : fused_thin_kernel<PT, Q, false, false>;
    TW_HIP(launch_kernel(kern, dim3(static_cast<unsigned>(grid)), dim3(kThinThreads), 0u, stream, prm));
    return TW_OK;
}

template <int PT, int Q>
static tw_status launch_deep_t(const FusedParams &prm, int64_t grid, hipStream_t stream)
{
    if constexpr (PT > 0) {
        TW_HIP(launch_kernel(fused_deep_kernel<PT, Q>, dim3(static_cast<unsigned>(grid)), dim3(kThinThreads), 0u,
                             stream, prm));
        return TW_OK;
    }
    return TW_ERR_UNSUPPORTED;
}

template <int PT>
static tw_status launch_thin(const FusedParams &prm, int q, bool trace, bool streamed, bool deep, int64_t grid,
                             hipStream_t s)
{
    if (deep) {
        switch (q) {
        case 1: return launch_deep_t<PT, 1>(prm, grid, s);
        case 2: return launch_deep_t<PT, 2>(prm, grid, s);
        case 3: return launch_deep_t<PT, 3>(prm, grid, s);
        case 4: return launch_deep_t<PT, 4>(prm, grid, s);
        }
        return TW_ERR_UNSUPPORTED;
    }
    switch (q) {
    case 1: return launch_thin_t<PT, 1>(prm, trace, streamed, grid, s);
    case 2: return launch_thin_t<PT, 2>(prm, trace, streamed, grid, s);
    case 3: return launch_thin_t<PT, 3>(prm, trace, streamed, grid, s);
    case 4: return launch_thin_t<PT, 4>(prm, trace, streamed, grid, s);
    }
    return TW_ERR_UNSUPPORTED;
}

// Geometry of the shared (co-resident) mode: 256-thread workgroups, each striding
// over up to eight row groups; enough workgroups that the hardware dispatcher
// balances them over compute units that are busy to different degrees.
struct ThinGeometry {
    int q;              // wide-kernel threads played by one thread (1 ... 4)
    int rows_per_iter;  // rows per row group
};
static ThinGeometry thin_geometry(const FusedGeometry &g)
{
    ThinGeometry t;
    const int tpr = 1 << g.tpr_log2;
    t.q = g.hv > kThinThreads ? (g.hv + kThinThreads - 1) / kThinThreads : 1;
    t.rows_per_iter = tpr >= kThinThreads ? 1 : kThinThreads / tpr;
    return t;
}
static int64_t thin_grid(int64_t n_rows, const ThinGeometry &t, int cus)
{
    const int64_t n_groups = (n_rows + t.rows_per_iter - 1) / t.rows_per_iter;
    int64_t gpw = n_groups / (int64_t(8) * cus);  // row groups per workgroup
    gpw = gpw < 1 ? 1 : gpw > 8 ? 8 : gpw;
    return (n_groups + gpw - 1) / gpw;
}

template <int PT>
static tw_status launch_vpt(const FusedParams &prm, const FusedGeometry &g, bool trace, bool streamed, int64_t grid,
                            hipStream_t s)
{
    switch (g.vpt) {
    case 1: return launch_t<PT, 1>(prm, trace, streamed, grid, g.block, s);
    case 2: return launch_t<PT, 2>(prm, trace, streamed, grid, g.block, s);
    case 4: return launch_t<PT, 4>(prm, trace, streamed, grid, g.block, s);
    case 8:
        if constexpr (PT != 8) return launch_t<PT, 8>(prm, trace, streamed, grid, g.block, s);  // P = 8 goes to the any-P kernel
        break;
    }
    return TW_ERR_UNSUPPORTED;
}

// Which kernel a launch takes. Shared mode has a kernel for rows of up to 1024
// vectors; wider rows run on the wide kernel over the whole device. A small
// whole-device launch with P = 1, 2, 4 or 8 also takes the small workgroups: they
// are placed faster and put every row in flight at once, where the wide kernel's
// software pipeline has only a few rows per workgroup to run over. Measured on
// MI355X, small workgroups against the wide kernel on 255 compute units, trains
// of launches on rotating buffers. Rows of an even number of 256-vector pieces
// (H = 4096, 8192: two chunks in flight per thread): P = 8 faster up to 8192 rows
// (22 % at 512, 4 % at 4096, 1.5 % at 8192), P = 4 up to 2048 (level at 4096, 2 %
// slower at 8192), P = 2 at H = 4096 up to 4096 (level at 8192, 5 % slower at
// 16384), P = 1 up to 1024 (7 % slower at 4096). Other row widths (one chunk in
// flight) keep narrower limits found the same way. For P without a specialised
// kernel, whose loads go out eight at a time, the wide kernel is faster, by up
// to 40 % on small batches. Both kernels give the same bits.
static bool takes_thin_kernel(int cu_budget, int cus, const FusedGeometry &g, int64_t n_rows, int P)
{
    if (g.vpt != 1) return false;
    if (cu_budget == TW_CU_SHARED) return true;
    if (resolve_budget(cu_budget, cus) != cus) return false;
    const bool two_chunks = g.hv > kThinThreads && ((g.hv + kThinThreads - 1) / kThinThreads) % 2 == 0;
    int64_t rows_per_cu;
    if (two_chunks) rows_per_cu = P == 8 ? 16 : (P == 4 || P == 2) ? 8 : P == 1 ? 4 : 0;
    else rows_per_cu = P == 8 ? 8 : (P == 4 || P == 2) ? 2 : 0;
    return n_rows <= rows_per_cu * cus;
}

tw_status launch_fused(const tw_fused_args &a, int64_t row_begin, int64_t row_end, uint32_t *hw_ids,
                       int64_t hw_ids_len, hipStream_t stream)
{
    if (row_end <= row_begin) return TW_OK;
    int cus = 0;
    TW_TRY(current_cu_count(&cus));
    const FusedGeometry g = fused_geometry(a.H);
    const int budget = resolve_budget(a.cu_budget, cus);
    const bool trace = hw_ids != nullptr;

    // A launch addresses at most kMaxLaunchBytes per tensor; more rows than that
    // go out as consecutive launches on the same stream.
    const int64_t row_bytes = a.H * 2;
    int64_t rows_per_launch = kMaxLaunchBytes / row_bytes;
    rows_per_launch -= rows_per_launch % g.rows_per_iter;
    if (trace && row_end - row_begin > rows_per_launch) return TW_ERR_UNSUPPORTED;
    const bool thin = takes_thin_kernel(a.cu_budget, cus, g, row_end - row_begin, a.P);
    // outputs that do not fit the last-level cache are stored with the streaming policy (see st());
    // not under a CU budget, where that is 1 % slower
    const bool streamed = 2 * (row_end - row_begin) * row_bytes >= kLastLevelCacheBytes && (thin || budget == cus);
    const ThinGeometry tg = thin_geometry(g);
    const int rows_per_group = thin ? tg.rows_per_iter : g.rows_per_iter;

    for (int64_t r0 = row_begin; r0 < row_end; r0 += rows_per_launch) {
        const int64_t n_rows = (row_end - r0 < rows_per_launch) ? row_end - r0 : rows_per_launch;
        int64_t grid = 0;
        bool deep = false;
        if (thin) {
            grid = thin_grid(n_rows, tg, cus);
            // one row group per workgroup, at most one workgroup per compute unit, few
            // bytes: the launch is latency-bound, everything is requested at once. Not
            // in shared mode, whose workgroups must fit beside a GEMM's.
            const int64_t n_groups = (n_rows + rows_per_group - 1) / rows_per_group;
            deep = !trace && a.cu_budget != TW_CU_SHARED && (a.P == 1 || a.P == 2 || a.P == 4 || a.P == 8) &&
                   grid == n_groups && n_groups <= cus && n_rows * row_bytes * (a.P + 1) <= kDeepInputBytes;
        } else {
            grid = fused_grid_size(n_rows, g, budget);
            if (grid > 1024) return TW_ERR_UNSUPPORTED;  // offset arithmetic in the kernel assumes this
        }
        if (trace && hw_ids_len < grid) return TW_ERR_SHAPE;

        FusedParams prm;
        const int64_t off = r0 * row_bytes;
        for (int p = 0; p < TW_MAX_P; ++p)
            prm.partials[p] = p < a.P ? static_cast<const char *>(a.partials[p]) + off : nullptr;
        prm.residual = static_cast<const char *>(a.residual) + off;
        prm.weight = a.weight;
        prm.out = static_cast<char *>(a.out) + off;
        prm.residual_out = static_cast<char *>(a.residual_out) + off;
        prm.hw_ids = hw_ids;
        prm.n_bytes = static_cast<uint32_t>(n_rows * row_bytes);
        prm.group_bytes = static_cast<uint32_t>(rows_per_group * row_bytes);
        prm.n_groups = static_cast<uint32_t>((n_rows + rows_per_group - 1) / rows_per_group);
        prm.hv = g.hv;
        prm.P = a.P;
        prm.tpr_log2 = g.tpr_log2;
        prm.wpr = g.wpr;
        prm.eps = a.eps;
        prm.inv_h = 1.0f / static_cast<float>(a.H);

        if (thin) {
            switch (a.P) {
            case 1: TW_TRY((launch_thin<1>(prm, tg.q, trace, streamed, deep, grid, stream))); break;
            case 2: TW_TRY((launch_thin<2>(prm, tg.q, trace, streamed, deep, grid, stream))); break;
            case 4: TW_TRY((launch_thin<4>(prm, tg.q, trace, streamed, deep, grid, stream))); break;
            case 8: TW_TRY((launch_thin<8>(prm, tg.q, trace, streamed, deep, grid, stream))); break;
            default: TW_TRY((launch_thin<0>(prm, tg.q, trace, streamed, deep, grid, stream))); break;
            }
            continue;
        }
        // Rows of 8 vectors per thread with all 8 partials in flight would not fit
        // the 128 registers; the any-P kernel (4 loads at a time, same order of
        // additions) does.
        const int p_case = (a.P == 8 && g.vpt == 8) ? 0 : a.P;
        switch (p_case) {
        case 1: TW_TRY((launch_vpt<1>(prm, g, trace, streamed, grid, stream))); break;
        case 2: TW_TRY((launch_vpt<2>(prm, g, trace, streamed, grid, stream))); break;
        case 4: TW_TRY((launch_vpt<4>(prm, g, trace, streamed, grid, stream))); break;
        case 8: TW_TRY((launch_vpt<8>(prm, g, trace, streamed, grid, stream))); break;
        default: TW_TRY((launch_vpt<0>(prm, g, trace, streamed, grid, stream))); break;
        }
    }
    return TW_OK;
}

}  // namespace tw

using namespace tw;

extern "C" {

tw_status tw_reduce_add_rmsnorm(const void *const *partials, const void *residual,
                                const void *weight, float eps, int64_t N, int64_t H, int P,
                                int cu_budget, void *out, void *residual_out, void *stream)
{
    const tw_fused_args a = {partials, residual, weight, eps, N, H, P, cu_budget, out, residual_out};
    TW_TRY(validate_fused(a));
    return launch_fused(a, 0, N, nullptr, 0, static_cast<hipStream_t>(stream));
}

tw_status tw_reduce_add_rmsnorm_traced(const void *const *partials, const void *residual,
                                       const void *weight, float eps, int64_t N, int64_t H, int P,
                                       int cu_budget, void *out, void *residual_out,
                                       uint32_t *hw_ids, int64_t hw_ids_len, void *stream)
{
    const tw_fused_args a = {partials, residual, weight, eps, N, H, P, cu_budget, out, residual_out};
    TW_TRY(validate_fused(a));
    if (!hw_ids) return TW_ERR_NULL;
    if (hw_ids_len < 0) return TW_ERR_SHAPE;
    return launch_fused(a, 0, N, hw_ids, hw_ids_len, static_cast<hipStream_t>(stream));
}

tw_status tw_fused_layout(int64_t H, int *waves_per_row, int *vectors_per_thread, int *rows_per_trip,
                          int *threads_per_workgroup)
{
    if (H <= 0) return TW_ERR_SHAPE;
    if (H % 8 != 0 || H > TW_MAX_H) return TW_ERR_UNSUPPORTED;
    const FusedGeometry g = fused_geometry(H);
    if (waves_per_row) *waves_per_row = g.wpr;
    if (vectors_per_thread) *vectors_per_thread = g.vpt;
    if (rows_per_trip) *rows_per_trip = g.rows_per_iter;
    if (threads_per_workgroup) *threads_per_workgroup = g.block;
    return TW_OK;
}

int64_t tw_fused_grid(int64_t N, int64_t H, int P, int cu_budget)
{
    if (N < 0 || H <= 0 || H % 8 != 0 || H > TW_MAX_H || P < 1 || P > TW_MAX_P) return -1;
    if (N == 0) return 0;
    int cus = 0;
    if (current_cu_count(&cus) != TW_OK) return -1;
    const FusedGeometry g = fused_geometry(H);
    if (takes_thin_kernel(cu_budget, cus, g, N, P) && N * H * 2 <= kMaxLaunchBytes) {
        return thin_grid(N, thin_geometry(g), cus);
    }
    return fused_grid_size(N, g, resolve_budget(cu_budget, cus));
}

}  // extern "C"
