/*
 * tw.h -- C ABI of libtw: the single-GPU hot path that TokenWeave (arXiv
 * 2505.11329) builds its compute-communication overlap around, written for
 * AMD Instinct MI355X (gfx950):
 *
 *   - the fused "reduce over the P tensor-parallel partials + residual add +
 *     RMSNorm" of one GPU's share of the token rows, in one pass over HBM
 *     (Section 4.3 and Appendix A, Listing 1), confined to a CU budget so it
 *     can co-run with compute (Section 4.3, last paragraph; Fig. 9);
 *   - the two-way token split launched on two streams (Section 4, Section
 *     4.1.2 "Overlapped Execution");
 *   - a bf16 GEMM standing in for the other split's projection, and the
 *     fused-kernel-next-to-GEMM launch that one step of the weave consists of
 *     (Fig. 7b).
 *
 * The in-switch reduction of the paper has no counterpart on this hardware:
 * the P peer partials are P buffers in local HBM and the reading compute unit
 * does the sum.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers unless a parameter says "host".
 *     bf16 tensors are row-major, contiguous, 16-byte aligned.
 *   - The caller owns all memory and all streams. libtw keeps no pointer after
 *     a call returns. Pointer arrays and argument structs are read on the host
 *     during the call and may live on the caller's stack.
 *   - Calls enqueue work on the given streams and return; nothing inside
 *     synchronises the device. `stream` arguments are hipStream_t values passed
 *     as void*; NULL means the default (null) stream.
 *   - Errors are reported through the return code only. Every argument check
 *     happens on the host before the first HIP call, so an invalid call
 *     launches nothing and works (returns its error) on a machine without a GPU.
 *   - Results are a pure function of each row's inputs: bits do not depend on
 *     cu_budget, on N, on the stream, or on whether and where rows were split.
 *   - HIP graphs: every entry point can be recorded into a stream capture
 *     (hipStreamBeginCapture on the caller's stream; the cross-stream entry
 *     points fork their second stream from `parent` and join it back, so a
 *     capture that begins and ends on `parent` holds the whole call). Nothing is
 *     allocated, freed or cleared with a memset per call, so a captured call or a
 *     captured train of calls replays as it was recorded, with the pointers it was
 *     recorded with. Make one eager call of each kind first (the first call on a
 *     device creates a few events and sets a kernel attribute, which a capture
 *     must not contain). Worth it for decode-sized batches (Appendix B, the
 *     decode paragraph): a train of 160 fused steps of 1 to 64 rows takes 5.1-6.1
 *     us per step launched eagerly and 4.5-5.6 us replayed from one graph, and the
 *     host is busy 0.5 instead of 4.1 us per step; from 256 rows on the kernels
 *     themselves fill the time and a graph gains nothing.
 *   - Thread safety: calls may be made from several host threads at once; work
 *     given to one stream is ordered by that stream as usual. The events the
 *     cross-stream entry points order their streams with come from a small ring
 *     per host thread and device, so one thread's record-then-wait pair can never
 *     pick up another thread's record. Nothing is allocated per call once a
 *     thread has made its first few calls on a device (16 events at most).
 */
#ifndef TW_H_
#define TW_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum tw_status {
    TW_OK = 0,
    TW_ERR_NULL = 1,        /* a required pointer is NULL                         */
    TW_ERR_SHAPE = 2,       /* a size is negative, zero where it must not be, or out of range */
    TW_ERR_ALIGN = 3,       /* a data pointer is not 16-byte aligned              */
    TW_ERR_ALIAS = 4,       /* buffers overlap in a way that is not allowed       */
    TW_ERR_UNSUPPORTED = 5, /* a valid request this build has no kernel for       */
    TW_ERR_SPLIT = 6,       /* split_row outside [0, N], cuts out of range or order, or the two streams are the same */
    TW_ERR_HIP = 7          /* a HIP call failed; see tw_last_hip_error()         */
} tw_status;

#define TW_MAX_P 16          /* most partial buffers one call can sum              */
#define TW_CU_SHARED (-1)    /* cu_budget value: co-resident ("shared") launch mode */
#define TW_MAX_H 65536       /* largest hidden size the fused kernel handles       */

/*
 * Arguments of one fused step (Appendix A, Listing 1; residual add fused as in
 * the footnote of Section 1). For every row r < N and column c < H:
 *
 *   x[r,c]            = (partials[0][r,c] + ... + partials[P-1][r,c]) + residual[r,c]
 *   residual_out[r,c] = bf16(x[r,c])
 *   out[r,c]          = bf16( x[r,c] * rsqrt(mean_c(x[r,c]^2) + eps) * weight[c] )
 *
 * Inputs are bf16; the sum is accumulated in fp32 in the order written above;
 * the mean of squares is taken over the UNROUNDED fp32 x, divided by H, with
 * eps inside the root; the scaling is (x * s) * weight in fp32; each output is
 * rounded once, to nearest even. NaN/Inf propagate by IEEE rules within their
 * row and never reach another row.
 *
 *   partials      host array of P device pointers, each bf16 [N x H]
 *   residual      device bf16 [N x H]
 *   weight        device bf16 [H]
 *   eps           finite, >= 0
 *   N             rows (tokens) >= 0; N == 0 is TW_OK, launches nothing, and the
 *                 [N x H] pointers are then not looked at (they may be NULL)
 *   H             hidden size: a multiple of 8 with 8 <= H <= TW_MAX_H
 *   P             1 <= P <= TW_MAX_P
 *   cu_budget     number of compute units the kernel may occupy: the launch is
 *                 a persistent grid of that many workgroups, each sized so that
 *                 no two share a compute unit. 0, or >= the device's CU count,
 *                 means the whole device. TW_CU_SHARED (-1) selects the shared
 *                 mode instead: many small workgroups (256 threads, <= 128
 *                 VGPRs, under 1 KiB LDS) spread over every compute unit, sized
 *                 to run NEXT TO a tw_gemm_bf16 workgroup on the same compute
 *                 unit rather than in place of one; for H > 8192 it falls back
 *                 to the whole device. Other negative values mean the whole
 *                 device. A small whole-device launch (P = 1, 2, 4 or 8; up to
 *                 4 to 16 rows per compute unit depending on P and H <= 8192) is
 *                 sent as those small workgroups too: same bits, lower latency;
 *                 and one of a few dozen rows (decode steps: inputs of at most
 *                 6 MiB) requests a whole row and the weights at once, one round
 *                 trip to memory instead of three.
 *   out           device bf16 [N x H]
 *   residual_out  device bf16 [N x H]
 *
 * Aliasing: residual_out may be the same buffer as residual (the paper updates
 * the residual stream in place) and out may be the same buffer as one of the
 * partials (the paper writes the result back into the communication buffer);
 * "the same buffer" means the same start address. Any other overlap between an
 * output and an input or between the two outputs is TW_ERR_ALIAS. Inputs may
 * overlap each other freely.
 */
typedef struct tw_fused_args {
    const void *const *partials;
    const void *residual;
    const void *weight;
    float eps;
    int64_t N;
    int64_t H;
    int P;
    int cu_budget;
    void *out;
    void *residual_out;
} tw_fused_args;

/* One fused step over all N rows, enqueued on `stream`. */
tw_status tw_reduce_add_rmsnorm(const void *const *partials, const void *residual,
                                const void *weight, float eps, int64_t N, int64_t H,
                                int P, int cu_budget, void *out, void *residual_out,
                                void *stream);

/*
 * Ablation: the pipeline the fused kernel replaces (Section 4.2 and Table 1:
 * all-reduce, then residual add + RMSNorm; Section 4.3: a stand-alone RMSNorm
 * reads the tensor twice and writes it once). Two launches on `stream`:
 *   t = bf16(p_0 + ... + p_{P-1}) into sum_scratch;
 *   x = t + residual, residual_out = bf16(x), s = rsqrt(mean(x^2) + eps), then
 *   out = bf16((bf16(x) * s) * weight) with bf16(x) read back from residual_out.
 * That moves (P + 6) * 2H bytes per row where tw_reduce_add_rmsnorm moves
 * (P + 3) * 2H, and rounds twice more, so its outputs are close to, not equal
 * to, the fused kernel's. Same arguments and rules as tw_reduce_add_rmsnorm,
 * except: args->cu_budget is ignored (both launches use the whole device);
 * H <= 8192 (else TW_ERR_UNSUPPORTED); sum_scratch is device bf16 [N x H],
 * 16-byte aligned, owned by the caller, overwritten, and must not overlap any
 * other tensor of the call (TW_ERR_ALIAS).
 */
tw_status tw_reduce_add_rmsnorm_unfused(const tw_fused_args *args, void *sum_scratch, void *stream);

/*
 * tw_reduce_add_rmsnorm_unfused for callers that cannot allocate device memory
 * or hand over a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc. Same two launches, same kernels, same bits;
 * the intermediate sum t goes through a buffer of TW_STATIC_SCRATCH_BYTES that
 * is part of the library's device image (one copy per GPU, held until the
 * process ends) instead of through sum_scratch. The call allocates and frees
 * nothing on host or device. Differences from tw_reduce_add_rmsnorm_unfused:
 *   - N * H * 2 must not exceed TW_STATIC_SCRATCH_BYTES, else TW_ERR_SHAPE
 *     (checked on the host before any HIP call; nothing is launched);
 *   - every call on one GPU uses that GPU's one buffer: two calls whose kernels
 *     may run at the same time on one GPU (different streams with no ordering
 *     between them) race on it and give undefined outputs. Calls on one stream,
 *     or ordered by events, are fine. The buffer keeps the previous call's
 *     contents; nothing in it has to start at zero, because the first launch
 *     writes every element of t that the second one reads.
 * The caller's tensors cannot overlap the buffer, so TW_ERR_ALIAS only reports
 * the overlaps tw_reduce_add_rmsnorm rejects.
 */
#define TW_STATIC_SCRATCH_BYTES (32u << 20) /* 32 MiB: e.g. 2048 rows of H = 8192 */
tw_status tw_reduce_add_rmsnorm_unfused_static(const tw_fused_args *args, void *stream);

/*
 * Two-way token split (Section 4: prefix split T_a, suffix split T_b; every
 * operation here is token-level, so the split is a pure row-range split).
 * Rows [0, split_row) are enqueued on stream_a and rows [split_row, N) on
 * stream_b, each as its own launch with args->cu_budget compute units.
 *
 *   parent         a stream whose already-enqueued work both halves must wait
 *                  for: an event is recorded on it and both streams wait on that
 *                  event. NULL is a valid value (the default stream), which is
 *                  why parent_is_set says whether there is a parent at all.
 *   parent_is_set  0: no fork and no join; `parent` is ignored.
 *   join           non-zero: after both launches `parent` is made to wait for
 *                  both halves.
 *
 * split_row == 0 or == N gives a single launch on stream_b or stream_a.
 * stream_a and stream_b must differ when both halves are non-empty
 * (TW_ERR_SPLIT otherwise). The results are bit-identical to the unsplit call.
 */
tw_status tw_split_launch(const tw_fused_args *args, int64_t split_row, void *stream_a,
                          void *stream_b, void *parent, int parent_is_set, int join);

/*
 * Where to cut N rows in two: ceil(N/2) rounded up to a multiple of `multiple`
 * (the prefix split takes the extra rows, Appendix A "Smart-Splitting"; split
 * offsets there are multiples of 64), clamped to N. A result equal to N means
 * "do not split". multiple <= 0 is treated as 1; N <= 0 gives 0. Host only.
 */
int64_t tw_split_point(int64_t N, int64_t multiple);

/*
 * GEMM stand-in for the other split's projection (the compute that overlaps
 * the fused kernel in Fig. 7b): C = A * B with bf16 inputs, fp32 accumulation,
 * one rounding to bf16 at the store.
 *
 *   A         device bf16 [M x K], row-major
 *   B         device bf16; b_layout says how B(k, n) is stored:
 *             TW_B_NK: [N x K] row-major, i.e. B(k,n) at B[n*K + k] -- the way a
 *                      linear layer's weight [out_features x in_features] is kept;
 *             TW_B_KN: [K x N] row-major, B(k,n) at B[k*N + n].
 *             Both layouts give bit-identical C.
 *   C         device bf16 [M x N], row-major; must not overlap A or B
 *   M, N, K   >= 0 (any zero: TW_OK, C untouched unless K == 0 and M*N > 0, in
 *             which case C is zero-filled); K must be a multiple of 8 and N a
 *             multiple of 8 (16-byte vectors), and K, N <= 2^22, M <= 2^40 (a
 *             tile's rows are addressed with 32-bit byte offsets), else
 *             TW_ERR_UNSUPPORTED
 *   cu_budget persistent grid of at most this many workgroups (one per compute
 *             unit); <= 0 or >= the CU count: whole device
 * The result bits depend on A, B and K only: not on the budget, the layout of B,
 * nor on the tile shape the launch picks (256 x 128 outputs per workgroup; 256 x
 * 64 when the wider tiles would fill at most half of the compute units; 256 x
 * 256 for a large product launched on its own, when such tiles fill the compute
 * units about as well). Every output element is the sum of its K / 32 partial
 * dot products of depth 32, accumulated in fp32 in the order of increasing k.
 */
#define TW_B_NK 0
#define TW_B_KN 1

typedef struct tw_gemm_args {
    const void *A;
    const void *B;
    void *C;
    int64_t M;
    int64_t N;
    int64_t K;
    int b_layout;
    int cu_budget;
} tw_gemm_args;

tw_status tw_gemm_bf16(const void *A, const void *B, void *C, int64_t M, int64_t N, int64_t K,
                       int b_layout, int cu_budget, void *stream);

/*
 * One step of the weave (Fig. 7b, Section 4.1.2): the fused kernel of one split
 * on stream_comm next to the GEMM of the other split on stream_compute. If
 * parent_is_set, both first wait for the work already enqueued on `parent`.
 * With a CU budget the fused kernel is enqueued first so that its few
 * workgroups are placed before the GEMM fills the remaining compute units; with
 * fused->cu_budget == TW_CU_SHARED the GEMM is enqueued first and the small
 * fused workgroups settle beside its workgroups. If join is non-zero,
 * `parent` then waits for both. The two streams must differ.
 * `fused` describes the rows of the split being normalised (its own pointers
 * and N); `gemm` the other split's product. Either may be NULL to leave that
 * side out.
 */
tw_status tw_overlap_launch(const tw_fused_args *fused, const tw_gemm_args *gemm,
                            void *stream_comm, void *stream_compute, void *parent,
                            int parent_is_set, int join);

/*
 * One tensor-parallel block boundary as the paper weaves it (Fig. 7b, Section
 * 4.1.2 "Overlapped Execution"), for one GPU's T token rows:
 *
 *   G1: partials[0] = X1 * W1^T   [T x K1] x [H x K1]^T  this GPU's projection output
 *   F : the fused step of tw_fused_args over all P partials and the residual
 *   G2: Y = out * W2^T            [T x H] x [N2 x H]^T   the next projection
 *
 * run for the two token splits a = [0, split_row) and b = [split_row, T), in one
 * of two schedules:
 *   TW_WEAVE_ORDERED  GEMMs go to stream_compute in the order G1(a) G1(b) G2(a)
 *       G2(b), fused kernels to stream_comm in the order F(a) F(b); events make
 *       F(s) wait for G1(s) and G2(s) wait for F(s), so F(a) runs next to G1(b)
 *       and F(b) next to G2(a). No two GEMMs ever compete, but three waits on
 *       another stream (15-20 us each on MI355X) lie on the critical path.
 *   TW_WEAVE_CHAINS   each split is a chain of its own: G1(a) F(a) G2(a) on
 *       stream_compute, G1(b) F(b) G2(b) on stream_comm. In a call that forks
 *       from a parent (both chains start at one point) the second chain is held
 *       back until G1(a) is done so that the two run out of step: one wait on
 *       another stream, off the critical path. A call without a parent adds no
 *       dependency between the streams. What overlaps with what is left to the
 *       hardware.
 *   TW_WEAVE_AUTO     chains when the fused kernel is not confined to a CU budget
 *       (shared mode or whole device): on the block boundaries of a 70B-class
 *       layer they are level to 13 % faster than the ordered schedule at 256 to
 *       16384 tokens, with one exception of 2.5 %; ordered when it is confined,
 *       because the GEMMs leave its compute units alone only while no two of them
 *       overlap.
 * With split_row == 0 or == T the chain G1, F, G2 runs unsplit on stream_compute
 * alone (nothing overlaps, no events; a fused step asked to share the compute
 * units, TW_CU_SHARED, has them to itself there and runs as a whole-device launch).
 * Results are bit-identical for every split_row and schedule.
 *
 *   X1, W1, K1   device bf16 [T x K1] and [H x K1] (TW_B_NK), K1 a multiple of 8
 *   fused        as for tw_reduce_add_rmsnorm with N = T; fused.partials[0] is
 *                WRITTEN by G1 (the const in the struct is cast away) and then
 *                read by F like the other partials; fused.cu_budget is F's budget
 *   W2, N2, Y    device bf16 [N2 x H] and [T x N2], N2 a multiple of 8
 *   gemm_cu_budget  persistent grid of the GEMMs; pass (CU count - fused.cu_budget)
 *                so that the fused kernel always finds its compute units free
 *   parent, parent_is_set, join   as for tw_split_launch
 * Consecutive boundaries (the next layer's, on the same two streams) need no fork
 * and join in between: pass parent_is_set = 1 on the first call only and join = 0
 * throughout, so that each split's chain runs on through the boundaries on its own
 * stream as in Fig. 7b, and join the second stream once at the end with an event.
 * A call without a parent adds no dependency between the two streams at all (one
 * chain per split; the compute/communication order keeps its events). Measured on
 * trains of eight 70B-class boundaries, per boundary: 2 to 11 % less than the
 * unsplit train from 3K to 32K tokens (7 % more at 2K), where a fork and a join
 * around every call is 3 % more to 5 % less; so an engine that runs through can
 * split from about 3K tokens (pass that as the threshold: the built-in one is
 * calibrated on single calls). Rows of one split must then depend only on rows of the same
 * split between the boundaries.
 * The two streams must differ. Buffers must satisfy the aliasing rules of the
 * three operations they take part in.
 */
#define TW_WEAVE_AUTO 0
#define TW_WEAVE_ORDERED 1
#define TW_WEAVE_CHAINS 2

typedef struct tw_layer_args {
    const void *X1;
    const void *W1;
    int64_t K1;
    tw_fused_args fused;
    const void *W2;
    int64_t N2;
    void *Y;
    int gemm_cu_budget;
    int schedule; /* TW_WEAVE_AUTO, TW_WEAVE_ORDERED or TW_WEAVE_CHAINS; others: TW_ERR_UNSUPPORTED */
} tw_layer_args;

tw_status tw_weave_layer(const tw_layer_args *layer, int64_t split_row, void *stream_compute,
                         void *stream_comm, void *parent, int parent_is_set, int join);

/*
 * The same boundary cut into more than two splits: rows [0, cuts[0]), [cuts[0],
 * cuts[1]), ..., [cuts[n_cuts - 1], T). The paper weaves two splits (Fig. 7b);
 * this is the same schedule carried on over a longer list, for callers whose
 * batches cut better into three or four pieces than into two (on MI355X that is
 * the case where a third or a quarter of the batch is a whole number of GEMM
 * tile waves and half of it is not: 3 % at 12K tokens and 2 % at 32K on a
 * 70B-class attention-side boundary; elsewhere two splits are level or better,
 * and more than four never paid). The splits are woven two at a time exactly as
 * tw_weave_layer weaves its pair, pair after pair on the same two streams (an
 * odd split at the end runs as a plain chain on stream_compute); nothing but
 * stream order links the pairs, so the end of one overlaps the start of the
 * next. n_cuts == 0 is the unsplit chain, n_cuts == 1 is tw_weave_layer.
 *   cuts     host array of n_cuts rows, strictly ascending, each in (0, T);
 *            read during the call only
 *   n_cuts   0 ... TW_MAX_CUTS
 * Results are bit-identical for every set of cuts. Errors as for
 * tw_weave_layer; TW_ERR_SPLIT for cuts out of order or out of range or too many.
 */
#define TW_MAX_CUTS 15
tw_status tw_weave_layer_cuts(const tw_layer_args *layer, const int64_t *cuts, int n_cuts, void *stream_compute,
                              void *stream_comm, void *parent, int parent_is_set, int join);

/*
 * A train of consecutive boundaries woven through (Fig. 7b from layer to layer,
 * as the paper's engine runs a model): boundary i is layers[i], all of the same
 * token count T and all cut at the same split_row; split a's chain G1 F G2, G1 F
 * G2, ... runs on stream_compute and split b's on stream_comm, forked from
 * `parent` before the first boundary and joined into it after the last (as for
 * tw_split_launch) and with no dependency between the two streams in between
 * (one chain per split; the compute/communication order keeps its events). That
 * is where the weave pays on this part: 2 to 11 % less per boundary than the
 * unsplit train from 3K to 32K tokens on 70B-class boundaries, where a fork and
 * a join around every boundary is 3 % more to 5 % less.
 * Stream order is the only thing that orders boundary i + 1 after boundary i:
 * what boundary i + 1 reads of boundary i's outputs (typically its X1 is computed
 * from Y, its residual is residual_out) must, for the rows of one split, depend
 * on rows of that same split only. (A caller with work of its own between the
 * boundaries, attention for instance, gets the same schedule from tw_weave_layer
 * calls without a parent, enqueueing that work on the stream of the split it
 * belongs to.)
 *   layers     host array of n_layers descriptions, read during the call only
 *   n_layers   0 ... TW_MAX_TRAIN (0: TW_OK, nothing launched)
 *   split_row  0 or T: every boundary unsplit, on stream_compute
 * All layers are checked before anything is launched. Errors: as for
 * tw_weave_layer; TW_ERR_SHAPE also when the token counts differ or n_layers is
 * out of range.
 */
#define TW_MAX_TRAIN 4096
#define TW_TRAIN_SPLIT_THRESHOLD 3072 /* tokens from which a train of 70B-class boundaries gains when woven (MI355X) */
tw_status tw_weave_train(const tw_layer_args *layers, int n_layers, int64_t split_row, void *stream_compute,
                         void *stream_comm, void *parent, int parent_is_set, int join);

/*
 * Wave-aware choice of the split row (Section 4.1.1 and Appendix A
 * "Smart-Splitting"; Algorithm 1 finds the offset by profiling because its GEMMs
 * are closed source, here the GEMM's tile grid is known, so the same sweep is
 * evaluated analytically). A GEMM over r rows with output width n runs
 * ceil(r / 256) * ceil(n / 128) workgroups (the GEMM's output tile), i.e. ceil(that / cus) waves on
 * `cus` compute units, and a wave lasts in proportion to the GEMM's depth k. The
 * cost of a cut is the sum over both splits and all n_gemms GEMMs of waves * k
 * (gemm_k == NULL: every GEMM weighs 1, the cost is the plain wave count). Among
 * the candidates k = tw_split_point(T, multiple) + j * multiple (j = 0, 1, 2,
 * ..., k < T, offset at most 512 rows as in Algorithm 1) the cheapest wins; ties
 * go to the cut that leaves the fewest 256-row GEMM tiles over both splits (a cut
 * inside a tile makes both splits work on that tile), then to the smallest offset. Returns T ("do not split") only when tw_split_point
 * already does, i.e. for batches too small to cut at that multiple. If not NULL,
 * *cost_split receives the winner's cost and *cost_unsplit that of the whole
 * batch, so the caller can apply the paper's criterion (split waves <= unsplit
 * waves) or its own threshold. Host only. gemm_n_out, gemm_k: host arrays of
 * n_gemms output widths and depths. Returns -1 on bad arguments (T < 0,
 * n_gemms < 1, cus < 1, NULL widths, a width or depth < 1).
 */
int64_t tw_smart_split_point(int64_t T, int64_t multiple, const int64_t *gemm_n_out, const int64_t *gemm_k,
                             int n_gemms, int cus, int64_t *cost_split, int64_t *cost_unsplit);

/*
 * Selective enabling (Fig. 3 and Appendix A "Selective Enabling of Splitting and
 * Overlap"): split and overlap only when the batch has at least `threshold`
 * tokens, otherwise run the fused kernel unsplit. threshold <= 0 takes the
 * built-in default for MI355X, TW_DEFAULT_SPLIT_THRESHOLD, found by profiling
 * tw_weave_layer against the unsplit chain on the attention-side block boundary
 * of a 70B-class layer, which breaks even between 6K and 8K tokens (the paper's
 * own thresholds, 1K and 4K tokens, are for its 8xH100 system). Returns 1 to
 * split, 0 not to. Host only.
 */
#define TW_DEFAULT_SPLIT_THRESHOLD 8192
int tw_should_split(int64_t num_tokens, int64_t threshold);

/*
 * Token threshold for ONE block boundary G1 -> F -> G2 of the given sizes on a
 * device with `cus` compute units, for callers without a profile of their own
 * (the paper finds its thresholds by offline profiling, per model: Appendix A
 * "Selective Enabling of Splitting and Overlap"; tw_weave_tune below is that
 * profiling step). TW_NEVER_SPLIT when the GEMM after the fused step is shorter
 * than the fused step itself (per token 2 H N2 flop at 1 PFLOP/s against
 * (P + 3) * 2H bytes at 5 TB/s, i.e. N2 < 200 (P + 3)): the second split's fused
 * kernel then has nothing to hide behind. Otherwise the larger of two bounds,
 * rounded up to whole GEMM row tiles:
 *   - the fused step of the whole batch, (P + 3) * 2H bytes per row at 5 TB/s,
 *     must take at least 290 us: below that the cross-stream waits, the
 *     contention between co-resident kernels and the smaller GEMM tiles of the
 *     split schedule cost more than hiding it gains;
 *   - half the batch must still cut the narrower of the two GEMM outputs
 *     (min(H, N2) columns) into tiles for at least half of the compute units.
 * On MI355X this gives 8192 for [T x 1024] x [1024 x 8192] -> F(H = 8192, P = 8)
 * -> [T x 8192] x [8192 x 3584] and TW_NEVER_SPLIT for the MLP-side boundary
 * with K1 = 3584, N2 = 1280. Profiling agrees on the whole and not in every
 * point: the first boundary gains 5 % at 8K tokens and 10 to 14 % from 14K to
 * 24K, is level to 3 % behind at 12K, and loses 2 to 5 % at 32K, where the
 * unsplit GEMMs happen to fill the device with whole waves of their largest
 * tiles; the second stays within +4 and -6 % of break-even throughout. What a split gains here comes as much from how the tiles of the
 * halves and of the whole batch fall on the compute units as from the overlap,
 * which no single threshold captures: tw_weave_tune measures it.
 * Host only. Returns -1 on bad arguments (any size < 1).
 */
#define TW_NEVER_SPLIT INT64_MAX
int64_t tw_split_threshold(int64_t K1, int64_t H, int P, int64_t N2, int cus);

/*
 * The decision of the per-iteration policy (Fig. 3; Appendix A "Selective Enabling
 * of Splitting and Overlap" and "Smart-Splitting") for a batch of T tokens at one
 * block boundary G1 [T x K1] x [K1 x H] -> F(H, P) -> G2 [T x H] x [H x N2] whose
 * GEMMs run on `cus` compute units: the row to cut at, or T for "do not split".
 *   threshold > 0 (the caller's, e.g. from tw_weave_tune runs): T < threshold runs
 *     unsplit, anything else is cut at the row tw_smart_split_point picks
 *     (candidates at multiples of `multiple`, widths {H, N2}, depths {K1, H}).
 *   threshold <= 0 (built in): with t = tw_split_threshold() of the boundary, never
 *     when t is TW_NEVER_SPLIT; always at that row from t tokens up; and for
 *     t / 2 < T < t only when the cut costs no GEMM waves, i.e. when the cost
 *     tw_smart_split_point reports for the cut does not exceed that of the whole
 *     batch (Section 4.1.1's criterion). In that band the unsplit GEMMs' own wave
 *     quantisation decides: on MI355X, for K1 = 1024, H = 8192, P = 8, N2 = 3584
 *     and T = 4096 ... 8192 in steps of 256, the policy stays within 0.8 % of the
 *     best timed candidate on average (2.9 % at worst), against 1.5 % (4.5 %)
 *     for the threshold alone and 1.5 % (5.6 %) for always splitting; where it
 *     picks the slower of the two, the two are within 3 % of each other.
 * multiple <= 0: 64. Host only. Returns -1 on bad arguments (T < 0, another size
 * < 1).
 */
int64_t tw_policy_split_row(int64_t T, int64_t K1, int64_t H, int P, int64_t N2, int cus, int64_t threshold,
                            int64_t multiple);

/*
 * The per-iteration policy of Fig. 3 as one call, for one block boundary: the
 * batch is cut at the row tw_policy_split_row names for it (on the GEMMs'
 * compute units) and woven by tw_weave_layer in the schedule layer->schedule
 * names, or, when that row is T, runs the chain G1, F, G2 unsplit on
 * stream_compute (the fused kernel is still used; only splitting and overlap are
 * switched off). threshold, multiple: as for tw_policy_split_row. *split_row
 * (may be NULL) receives the row taken, T meaning
 * "not split"; it is written before anything is enqueued, also when the launch
 * then fails. Everything else as for tw_weave_layer, whose bit-exactness across
 * split rows makes the policy invisible in the results. The row is chosen per
 * boundary from its shapes: a train of boundaries woven through without joins
 * (see tw_weave_layer) needs ONE row for all of them, so take it once (e.g. from
 * tw_policy_split_row for the first boundary) and call tw_weave_layer.
 */
tw_status tw_weave_layer_auto(const tw_layer_args *layer, int64_t threshold, int64_t multiple, void *stream_compute,
                              void *stream_comm, void *parent, int parent_is_set, int join, int64_t *split_row);

/*
 * The offline search of Algorithm 1 (Appendix A "Smart-Splitting") and of the
 * thresholds of Appendix A "Selective Enabling of Splitting and Overlap", for one
 * block boundary and one batch size: the paper takes both from timing candidate
 * configurations before serving, not from a formula. Runs the boundary `layer`
 * unsplit and woven at every candidate row, `reps` rounds with the candidates in
 * rotating order after one untimed round, timed with events on stream_compute
 * (fork and join included), and reports the medians:
 *   us[0]      the unsplit chain
 *   us[1]      the row tw_smart_split_point picks (multiple, widths {H, N2},
 *              depths {K1, H}, the GEMMs' compute units)
 *   us[2 + i]  row tw_split_point(T, multiple) + offsets[i], i < n_offsets
 * A candidate row outside (0, T), or equal to an earlier candidate, is not run
 * and reports a negative time. *best_row receives the fastest candidate's row, T
 * when that is the unsplit chain: pass it to tw_weave_layer for batches of this
 * size (callers keep such results per token count, as the paper's engine does).
 * Unlike every other entry point this one WAITS for the device (it synchronises
 * both streams before returning and between candidates) and creates and destroys
 * two events: call it at start-up, never under stream capture. The layer's
 * outputs are left as any tw_weave_layer call leaves them.
 *   multiple <= 0: 64. offsets may be NULL with n_offsets == 0; n_offsets <= 16.
 *   reps in 1 .. 64. us: host array of 2 + n_offsets floats. best_row, us: not NULL.
 * Errors: TW_ERR_NULL, TW_ERR_SHAPE (reps, n_offsets out of range), and whatever
 * tw_weave_layer returns for the layer; on error *best_row and us are unspecified.
 */
tw_status tw_weave_tune(const tw_layer_args *layer, int64_t multiple, const int64_t *offsets, int n_offsets, int reps,
                        void *stream_compute, void *stream_comm, int64_t *best_row, float *us);

/* Compute units of the current device; -1 when no device can be queried. */
int tw_device_cu_count(void);
/* Static, NUL-terminated description of a status code (never NULL). */
const char *tw_status_str(tw_status s);
/* Static version string. */
const char *tw_version(void);
/* Raw hipError_t behind the last TW_ERR_HIP returned on the calling thread (0 if none). */
int tw_last_hip_error(void);
/* Source location and expression of that failing HIP call ("" if none). Static storage. */
const char *tw_last_hip_error_where(void);

#ifdef __cplusplus
}
#endif
#endif /* TW_H_ */
