/*
 * tw_measure.h -- measurement and introspection aids of libtw. They live in the
 * same shared library as the entry points of tw.h but are NOT part of the
 * method's interface: they expose launch geometry and streaming probes so that
 * claims about the kernels (how many compute units a budget occupies, what a
 * compute unit can pull from HBM, which schedule a boundary takes) can be
 * evidenced from outside. Their signatures may change with the kernels; nothing
 * in tw.h depends on them. Conventions (device pointers, status codes, checks
 * before the first HIP call) are those of tw.h.
 */
#ifndef TW_MEASURE_H_
#define TW_MEASURE_H_

#include "tw.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Same as tw_reduce_add_rmsnorm, and in addition workgroup g of the launch
 * writes, once, the hardware placement it ran on to hw_ids[2*g] (the raw HW_ID
 * register) and hw_ids[2*g+1] (the raw XCC_ID register), so that "confined to
 * cu_budget compute units" can be evidenced (Section 4.3 / Fig. 9 vary the
 * number of SMs the kernel gets). hw_ids: device uint32 [2 * hw_ids_len];
 * hw_ids_len must be at least the grid size that tw_fused_grid() returns.
 */
tw_status tw_reduce_add_rmsnorm_traced(const void *const *partials, const void *residual,
                                       const void *weight, float eps, int64_t N, int64_t H,
                                       int P, int cu_budget, void *out, void *residual_out,
                                       uint32_t *hw_ids, int64_t hw_ids_len, void *stream);

/*
 * tw_gemm_bf16 (B stored [N x K], whole device) with a kernel that also counts,
 * per wave, the shader clocks it spends in each phase of its K loop: evidence for
 * where the cycles of the 256 x 256 tile's pipeline go. Only products that
 * tw_gemm_bf16 would run on 256 x 256 tiles are accepted (TW_ERR_UNSUPPORTED
 * otherwise). Wave w of workgroup g writes TW_GEMM_PHASES 64-bit sums to
 * phase_cycles[(g * 4 + w) * TW_GEMM_PHASES + i]:
 *   0  first sub-step of the K steps (64 MFMAs = 1024 clocks of matrix work each,
 *      with the loads of one operand and the fragment reads of the second)
 *   1  waiting for the next K step's loads to have landed
 *   2  the workgroup barrier of a K step
 *   3  second sub-step of the K steps (as 0, plus the bookkeeping of the next step)
 *   4  from the start of a tile to its first MFMA (the pipeline filling)
 *   5  the stores of a tile
 *   6  tiles this wave worked on
 *   7  the kernel from its first to its last instruction
 * Reading the clock costs a scalar memory read and a wait each time: the traced
 * kernel is a few percent slower than the plain one. phase_cycles: device memory,
 * phase_len entries, at least (workgroups, at most one per compute unit) * 4 *
 * TW_GEMM_PHASES (else TW_ERR_SHAPE). C receives the product as usual.
 */
#define TW_GEMM_PHASES 8
tw_status tw_gemm_bf16_traced(const void *A, const void *B, void *C, int64_t M, int64_t N, int64_t K,
                              unsigned long long *phase_cycles, int64_t phase_len, void *stream);

/* Number of workgroups the fused kernel is launched with for these sizes on the
 * current device (0 if N == 0; -1 if the arguments are invalid or no device). */
int64_t tw_fused_grid(int64_t N, int64_t H, int P, int cu_budget);

/*
 * How the budgeted fused kernel lays a row of H elements over a workgroup (host
 * arithmetic only, no device needed): waves per row (0: the row is narrower
 * than a wave and takes a power-of-two group of lanes), 16-byte vectors per
 * thread, rows per workgroup trip and threads per workgroup. Any pointer may be
 * NULL. Returns TW_ERR_UNSUPPORTED for an H the kernel does not take.
 */
tw_status tw_fused_layout(int64_t H, int *waves_per_row, int *vectors_per_thread, int *rows_per_trip,
                          int *threads_per_workgroup);

/*
 * The schedule tw_weave_layer takes for a split boundary of these sizes on a
 * device with `cus` compute units: TW_WEAVE_ORDERED or TW_WEAVE_CHAINS (the
 * `schedule` argument itself unless it is TW_WEAVE_AUTO). Host arithmetic only.
 * Returns -1 on bad arguments.
 */
int tw_weave_schedule(int64_t T, int64_t K1, int64_t H, int P, int64_t N2, int fused_cu_budget, int schedule,
                      int cus);

/* Rows and columns of the output tile a GEMM workgroup computes by default, and
 * always when the GEMM runs beside another kernel (a product launched on its own
 * may be cut into tiles of half or twice this width instead, see tw_gemm_bf16;
 * tw_smart_split_point counts in tiles of this shape). */
void tw_gemm_tile_shape(int *tile_m, int *tile_n);

/*
 * Measurement aid (not part of the method): a streaming kernel with the same
 * persistent, CU-budgeted launch shape as the fused kernel, used to measure
 * what a given number of compute units can pull from / push to HBM, and as the
 * copy of known size against which hardware byte counters are scaled.
 *   mode TW_PROBE_READ: reads `bytes` from src (dst gets one 16-byte word per
 *        wave so the loads cannot be dropped; dst needs 256 bytes per compute
 *        unit of the device, 64 KiB on a 256-CU part);
 *   mode TW_PROBE_COPY: dst[0..bytes) = src[0..bytes);
 *   mode TW_PROBE_WRITE: dst[0..bytes) = a constant pattern (src unused, may be NULL).
 * bytes must be a multiple of 16; pointers 16-byte aligned; src and dst must
 * not overlap.
 */
#define TW_PROBE_READ 0
#define TW_PROBE_COPY 1
#define TW_PROBE_WRITE 2
tw_status tw_hbm_probe(const void *src, void *dst, int64_t bytes, int mode, int cu_budget,
                       void *stream);

/*
 * Measurement aid: the fused kernel's traffic shape without its arithmetic.
 * With the same budgeted launch, every workgroup walks 16 KiB rows; per row it
 * reads n_read streams (src + r * stream_bytes, r < n_read) and writes n_write
 * streams (dst + w * stream_bytes) at the same offset. What
 * it reaches is the ceiling of any kernel with that mix of loads and stores on
 * that many compute units. stream_bytes: a multiple of 16384, at most 2 GiB;
 * 0 <= n_read <= TW_MAX_P + 1, 0 <= n_write <= 4, not both zero. With
 * n_write == 0, dst still needs 16 KiB. src and dst ranges must not overlap.
 */
tw_status tw_hbm_probe_mixed(const void *src, void *dst, int64_t stream_bytes, int n_read,
                             int n_write, int cu_budget, void *stream);

/*
 * tw_hbm_probe with the launch shape opened up, to show what the ceiling of a
 * compute unit does and does not depend on: `threads` per workgroup (a multiple
 * of 64, at most 1024; still one workgroup per compute unit) and `in_flight`
 * 16-byte accesses issued per thread before the first is consumed (1, 2, 4, 8 or
 * 16; others: TW_ERR_UNSUPPORTED). tw_hbm_probe is the case (1024, 8). In
 * TW_PROBE_READ mode dst needs 256 bytes per compute unit whatever `threads` is.
 */
tw_status tw_hbm_probe_shaped(const void *src, void *dst, int64_t bytes, int mode, int cu_budget, int threads,
                              int in_flight, void *stream);

/*
 * tw_hbm_probe_mixed with `threads` per workgroup (64, 128, 256, 512 or 1024: a
 * workgroup then walks rows of threads * 16 bytes; each thread still has n_read
 * loads in flight). tw_hbm_probe_mixed is the case 1024.
 */
tw_status tw_hbm_probe_mixed_shaped(const void *src, void *dst, int64_t stream_bytes, int n_read, int n_write,
                                    int cu_budget, int threads, void *stream);

/*
 * Do kernels on these two streams run side by side? Two streams of one process
 * only overlap when the HIP runtime has mapped them to different hardware queues,
 * and it has few of those (GPU_MAX_HW_QUEUES, 4 by default): of the streams a
 * process creates, every fourth shares a queue with the first, and work on two
 * such streams runs strictly one kernel after the other, whatever events say.
 * The split schedules of tw.h then still give correct results but hide nothing.
 * This call finds out by running a one-wave kernel that idles for 300 us on each
 * stream from a common starting point and timing both with events: *overlap is 1
 * if the later one ends well before 600 us, else 0 (also when stream_a ==
 * stream_b). Unlike the entry points of tw.h it creates and destroys three
 * events and BLOCKS until both kernels are done (about 0.3 to 0.6 ms after the
 * work already on stream_a): call it once when the streams are set up, not per
 * launch, and not during stream capture.
 */
tw_status tw_streams_overlap(void *stream_a, void *stream_b, int *overlap);

/*
 * A stream whose kernels the hardware confines to n_cus compute units: the other
 * way of giving the fused kernel "a few SMs" (Section 4.3; Fig. 9), enforced by
 * the dispatcher instead of by the launch shape (tw_fused_args.cu_budget: a
 * persistent grid of one workgroup per compute unit). The stream carries a
 * compute-unit mask with bits [first_cu, first_cu + n_cus) set. On MI355X the
 * dispatcher deals mask bit i to XCD i mod 8 (probed with the traced launch: bits
 * 0 ... 31 are four compute units in each of the eight XCDs), so a range whose
 * length is a multiple of 8 is spread evenly, and two disjoint ranges are
 * disjoint sets of compute units: [0, 32) for the fused kernel and [32, 256) for
 * the GEMM is the paper's partition in hardware. A mask that leaves an XCD
 * without a compute unit is refused by the runtime (TW_ERR_HIP).
 * Any grid may be launched on such a stream (also cu_budget = 0 or
 * TW_CU_SHARED); workgroups beyond what the masked units hold wait their turn.
 * What a confined kernel can pull from HBM is the same either way (one compute
 * unit sustains ~50-57 GB/s): 1.45-1.5 TB/s for the shared-mode grid on 32 masked
 * units against 1.6 for the persistent grid of 32 workgroups, which runs as fast
 * on a masked stream as on an ordinary one. Measured with the overlap demo's pair
 * (fused kernel on 32 units beside the GEMM on 224): kernels on two masked
 * streams do run side by side, but forked from and joined into a parent stream
 * with events the masked pair took 316-328 us against 264-295 on ordinary
 * streams with the same budgets, and the first dispatch on a new masked stream
 * starts late (run something on it before timing). So the launch-shape budget
 * stays the default and the mask is the cross-check that the budget confines
 * what it says.
 * The caller owns the stream: it is an ordinary hipStream_t of default priority
 * on a hardware queue of its own, to be destroyed with tw_stream_destroy (or
 * hipStreamDestroy) once its work is done. Not for use during stream capture.
 * Errors: TW_ERR_NULL; TW_ERR_SHAPE (first_cu < 0, n_cus < 1, range beyond the
 * device's compute units); TW_ERR_HIP.
 */
tw_status tw_stream_create_cu_masked(int first_cu, int n_cus, void **stream);
tw_status tw_stream_destroy(void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TW_MEASURE_H_ */
