/*
 * tw_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, fp64 CPU statement of what the fused reduce + residual-add +
 * RMSNorm path computes, and of the GEMM used as the overlapped compute
 * stand-in. It exists so that the HIP library can be checked against
 * something that is obviously the definition. It shares no code with the HIP
 * library (own bf16 codec, own loops) and nothing in the product path may
 * call it: only tests, the smoke check and the benchmark's cpu_baseline leg.
 *
 * What is followed (TokenWeave, arXiv 2505.11329):
 *   - Appendix A, Listing 1 (fused AllReduce-RMSNorm kernel): per token row,
 *     x = (sum over the tensor-parallel ranks of their partial) + residual;
 *     the residual stream is replaced by x; var = sum_c x[c]^2;
 *     s = rsqrt(var / hidden_size + epsilon); out = x * s * weight.
 *   - Section 4.3: the sum of squares is taken on the just-reduced values,
 *     the residual add is fused in, and the normalised values are what is
 *     distributed.
 *   - Section 4.2: RMSNorm is a token-level operation, so every row is
 *     independent of every other row (this is what allows the token split of
 *     Section 4 to be a pure row-range split).
 *   The in-switch reduction of the paper is replaced by an explicit sum over
 *   P buffers; the sum itself is the same mathematical object.
 *
 * Readings taken (the paper's precision statements are in Listing 1 only):
 *   - tw_oracle_fused: x used for the sum of squares and for the scaling is the
 *     UNROUNDED sum (fp32 accumulation throughout on the device; this is the
 *     reading the device path is held to).
 *   - tw_oracle_fused_rounded_x: Listing 1 as printed keeps the summed vector in
 *     bf16, takes the sum of squares of that bf16 vector, stores it to the
 *     residual stream and scales what it reads back from there, i.e. the
 *     bf16-ROUNDED x feeds the norm. That literal reading is provided too, with
 *     pins of its own, so tests can bound the difference between the two.
 *   - epsilon sits inside the square root; the mean divides by H.
 *   - bf16 encoding is round-to-nearest-even, NaN stays NaN, overflow -> Inf.
 *   - tw_oracle_unfused: the all-reduce's bf16 output is the exact sum rounded
 *     once (the paper does not state the reduction's internal precision);
 *     tw_oracle_unfused_f32sum is a second, labelled reading in which that sum
 *     is accumulated in binary32 in rank order before the rounding.
 *
 * All pins for this file live in tests/test_oracle_pins.py (closed forms,
 * invariants, worked examples, exact rational brute force, library RMSNorm
 * and matmul special cases). Nothing here is "parity unpinned".
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- bf16 codec (own copy; bf16 = top 16 bits of an IEEE binary32) ---- */

static double bf16_to_f64(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f; /* binary32 -> binary64 is exact */
}

/* Round a binary64 to the nearest bf16 (ties to even) in ONE rounding step:
 * going through binary32 first would round twice. Works on the binary64 bit
 * pattern: a bf16 has 8 significand bits (7 stored), binary64 has 53. */
uint16_t tw_oracle_f64_to_bf16(double v)
{
    if (isnan(v))
        return 0x7FC0;
    uint16_t sign = signbit(v) ? 0x8000 : 0;
    double a = fabs(v);
    if (isinf(a))
        return sign | 0x7F80;
    if (a == 0.0)
        return sign;
    /* Largest finite bf16 is (2 - 2^-7) * 2^127; halfway to 2^128 rounds to
     * even = overflow. */
    const double max_bf16 = 0x1.FEp127;
    const double half_ulp_top = 0x1p119; /* ulp at the top binade = 2^120 */
    if (a >= max_bf16 + half_ulp_top)
        return sign | 0x7F80;
    int e;
    (void)frexp(a, &e); /* a = m * 2^e, m in [0.5, 1) */
    int exp2 = e - 1;   /* a in [2^exp2, 2^(exp2+1)) */
    if (exp2 < -126)
        exp2 = -126;           /* subnormal range: fixed quantum 2^-133 */
    double quantum = ldexp(1.0, exp2 - 7); /* spacing of bf16 values near a */
    double q = a / quantum;                /* exact: power-of-two scaling */
    double fl = floor(q);
    double frac = q - fl; /* exact */
    if (frac > 0.5 || (frac == 0.5 && fmod(fl, 2.0) == 1.0))
        fl += 1.0;
    double r = fl * quantum; /* exact, representable in binary32 */
    float f = (float)r;
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return sign | (uint16_t)(u >> 16);
}

double tw_oracle_bf16_to_f64(uint16_t h) { return bf16_to_f64(h); }

/* ---- the fused path, one row (Listing 1, body of the token loop) ---- */

static void fused_row(const uint16_t *const *partials, const uint16_t *residual,
                      const uint16_t *weight, double eps, int64_t H, int P,
                      int64_t r, int rounded_x, double *x /* scratch [H] */,
                      double *ref_out, double *ref_res)
{
    const int64_t base = r * H;
    double sumsq = 0.0;
    for (int64_t c = 0; c < H; ++c) {
        double acc = 0.0;
        for (int p = 0; p < P; ++p) /* reduction over ranks */
            acc += bf16_to_f64(partials[p][base + c]);
        acc += bf16_to_f64(residual[base + c]); /* residual add */
        x[c] = acc;
        ref_res[base + c] = acc; /* new residual stream, unrounded */
        double xn = rounded_x ? bf16_to_f64(tw_oracle_f64_to_bf16(acc)) : acc;
        sumsq += xn * xn;
    }
    const double s = 1.0 / sqrt(sumsq / (double)H + eps);
    for (int64_t c = 0; c < H; ++c) {
        double xn = rounded_x ? bf16_to_f64(tw_oracle_f64_to_bf16(x[c])) : x[c];
        ref_out[base + c] = xn * s * bf16_to_f64(weight[c]);
    }
}

static int fused_rows(const uint16_t *const *partials, const uint16_t *residual,
                      const uint16_t *weight, double eps, int64_t row_begin,
                      int64_t row_end, int64_t H, int P, int rounded_x,
                      double *ref_out, double *ref_res)
{
    double *x = (double *)malloc((size_t)(H > 0 ? H : 1) * sizeof(double));
    if (!x)
        return -1;
    for (int64_t r = row_begin; r < row_end; ++r)
        fused_row(partials, residual, weight, eps, H, P, r, rounded_x, x,
                  ref_out, ref_res);
    free(x);
    return 0;
}

/* partials: P pointers to bf16 [N*H]; residual bf16 [N*H]; weight bf16 [H];
 * ref_out, ref_res: fp64 [N*H], the UNROUNDED expected outputs.
 * Returns 0, or -1 on bad arguments / allocation failure. */
int tw_oracle_fused(const uint16_t *const *partials, const uint16_t *residual,
                    const uint16_t *weight, float eps, int64_t N, int64_t H,
                    int P, double *ref_out, double *ref_res)
{
    if (N < 0 || H <= 0 || P < 1)
        return -1;
    return fused_rows(partials, residual, weight, (double)eps, 0, N, H, P, 0,
                      ref_out, ref_res);
}

/* Alternative reading: the bf16-rounded x feeds the sum of squares and the
 * scaling (ref_res stays the unrounded sum). */
int tw_oracle_fused_rounded_x(const uint16_t *const *partials,
                              const uint16_t *residual, const uint16_t *weight,
                              float eps, int64_t N, int64_t H, int P,
                              double *ref_out, double *ref_res)
{
    if (N < 0 || H <= 0 || P < 1)
        return -1;
    return fused_rows(partials, residual, weight, (double)eps, 0, N, H, P, 1,
                      ref_out, ref_res);
}

/* ---- the unfused pipeline the paper measures its kernel against (Section 4.2,
 * Table 1: all-reduce, then residual add + RMSNorm; Section 4.3 describes the
 * standard RMSNorm as two reads of the tensor and one write). Three stages,
 * each a pass over memory with bf16 tensors in between:
 *   1. t = bf16(p_0 + ... + p_{P-1}), the all-reduce's bf16 output: the sum as
 *      a real number (binary64 holds it exactly for operands whose exponents
 *      span fewer than 45 binades), rounded once to nearest even. With
 *      f32_sum != 0 the second reading: the sum accumulated in binary32 in the
 *      order p = 0 .. P-1, then rounded;
 *   2. x = t + residual (exact in binary64); the new residual stream is x
 *      (ref_res, unrounded; what is stored is bf16(x)); the sum of squares is
 *      taken over the unrounded x;
 *   3. the stored residual stream is read back: out = bf16(x) * s * w.
 * ref_out is the unrounded result of stage 3. ---- */
static int unfused_rows(const uint16_t *const *partials, const uint16_t *residual,
                        const uint16_t *weight, double eps, int64_t N, int64_t H,
                        int P, int f32_sum, double *ref_out, double *ref_res)
{
    for (int64_t r = 0; r < N; ++r) {
        const int64_t base = r * H;
        double sumsq = 0.0;
        for (int64_t c = 0; c < H; ++c) {
            double sum;
            if (f32_sum) {
                volatile float acc = 0.0f; /* volatile: no excess precision, no contraction */
                for (int p = 0; p < P; ++p)
                    acc = acc + (float)bf16_to_f64(partials[p][base + c]);
                sum = (double)acc;
            } else {
                sum = 0.0;
                for (int p = 0; p < P; ++p)
                    sum += bf16_to_f64(partials[p][base + c]);
            }
            const double t = bf16_to_f64(tw_oracle_f64_to_bf16(sum));
            const double x = t + bf16_to_f64(residual[base + c]);
            ref_res[base + c] = x;
            sumsq += x * x;
        }
        const double s = 1.0 / sqrt(sumsq / (double)H + eps);
        for (int64_t c = 0; c < H; ++c) {
            const double stored = bf16_to_f64(tw_oracle_f64_to_bf16(ref_res[base + c]));
            ref_out[base + c] = stored * s * bf16_to_f64(weight[c]);
        }
    }
    return 0;
}

int tw_oracle_unfused(const uint16_t *const *partials, const uint16_t *residual,
                      const uint16_t *weight, float eps, int64_t N, int64_t H,
                      int P, double *ref_out, double *ref_res)
{
    if (N < 0 || H <= 0 || P < 1)
        return -1;
    return unfused_rows(partials, residual, weight, (double)eps, N, H, P, 0, ref_out, ref_res);
}

/* Second reading of stage 1: binary32 accumulation in rank order. */
int tw_oracle_unfused_f32sum(const uint16_t *const *partials, const uint16_t *residual,
                             const uint16_t *weight, float eps, int64_t N, int64_t H,
                             int P, double *ref_out, double *ref_res)
{
    if (N < 0 || H <= 0 || P < 1)
        return -1;
    return unfused_rows(partials, residual, weight, (double)eps, N, H, P, 1, ref_out, ref_res);
}

/* ---- row-parallel wrapper: same per-row code, rows dealt out in contiguous
 * blocks to nthreads POSIX threads. Only used to time the oracle on all host
 * cores; results are identical to the single-threaded call because rows are
 * independent. ---- */

typedef struct {
    const uint16_t *const *partials;
    const uint16_t *residual;
    const uint16_t *weight;
    double eps;
    int64_t row_begin, row_end, H;
    int P;
    double *ref_out, *ref_res;
    int status;
} fused_job;

static void *fused_worker(void *arg)
{
    fused_job *j = (fused_job *)arg;
    j->status = fused_rows(j->partials, j->residual, j->weight, j->eps,
                           j->row_begin, j->row_end, j->H, j->P, 0, j->ref_out,
                           j->ref_res);
    return NULL;
}

int tw_oracle_fused_mt(const uint16_t *const *partials,
                       const uint16_t *residual, const uint16_t *weight,
                       float eps, int64_t N, int64_t H, int P, double *ref_out,
                       double *ref_res, int nthreads)
{
    if (N < 0 || H <= 0 || P < 1 || nthreads < 1)
        return -1;
    if (nthreads > 1024)
        nthreads = 1024;
    pthread_t *tid = (pthread_t *)calloc((size_t)nthreads, sizeof *tid);
    fused_job *job = (fused_job *)calloc((size_t)nthreads, sizeof *job);
    if (!tid || !job) {
        free(tid);
        free(job);
        return -1;
    }
    int64_t per = (N + nthreads - 1) / nthreads;
    int started = 0, rc = 0;
    for (int t = 0; t < nthreads; ++t) {
        int64_t b = per * t, e = b + per;
        if (b > N)
            b = N;
        if (e > N)
            e = N;
        job[t] = (fused_job){partials, residual, weight, (double)eps, b, e, H,
                             P, ref_out, ref_res, 0};
        if (pthread_create(&tid[t], NULL, fused_worker, &job[t]) != 0) {
            rc = -1;
            break;
        }
        ++started;
    }
    for (int t = 0; t < started; ++t) {
        pthread_join(tid[t], NULL);
        if (job[t].status != 0)
            rc = -1;
    }
    free(tid);
    free(job);
    return rc;
}

/* ---- GEMM stand-in: C = A * B, textbook triple loop in fp64.
 * A is bf16 [M x K] row-major. B is given as bf16 with explicit strides so
 * that either storage order can be described without two loops:
 * element B(k, n) lives at B[k * b_stride_k + n * b_stride_n]. ---- */

static double gemm_elem(const uint16_t *A, const uint16_t *B, int64_t K,
                        int64_t b_stride_k, int64_t b_stride_n, int64_t m,
                        int64_t n)
{
    double acc = 0.0;
    for (int64_t k = 0; k < K; ++k)
        acc += bf16_to_f64(A[m * K + k]) *
               bf16_to_f64(B[k * b_stride_k + n * b_stride_n]);
    return acc;
}

int tw_oracle_gemm(const uint16_t *A, const uint16_t *B, int64_t M, int64_t N,
                   int64_t K, int64_t b_stride_k, int64_t b_stride_n,
                   double *C /* [M x N] row-major */)
{
    if (M < 0 || N < 0 || K < 0)
        return -1;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n)
            C[m * N + n] = gemm_elem(A, B, K, b_stride_k, b_stride_n, m, n);
    return 0;
}

/* The same definition evaluated only at the listed (m, n) pairs, so that a
 * large product can be spot-checked one output at a time. */
int tw_oracle_gemm_samples(const uint16_t *A, const uint16_t *B, int64_t M,
                           int64_t N, int64_t K, int64_t b_stride_k,
                           int64_t b_stride_n, const int64_t *ms,
                           const int64_t *ns, int64_t count, double *vals)
{
    if (M < 0 || N < 0 || K < 0 || count < 0)
        return -1;
    for (int64_t i = 0; i < count; ++i) {
        if (ms[i] < 0 || ms[i] >= M || ns[i] < 0 || ns[i] >= N)
            return -1;
        vals[i] = gemm_elem(A, B, K, b_stride_k, b_stride_n, ms[i], ns[i]);
    }
    return 0;
}

/* Array forms of the codec, for the tests that decode GPU outputs and that
 * produce the rounded expected values. */
void tw_oracle_bf16_to_f64_array(const uint16_t *src, int64_t n, double *dst)
{
    for (int64_t i = 0; i < n; ++i)
        dst[i] = bf16_to_f64(src[i]);
}

void tw_oracle_f64_to_bf16_array(const double *src, int64_t n, uint16_t *dst)
{
    for (int64_t i = 0; i < n; ++i)
        dst[i] = tw_oracle_f64_to_bf16(src[i]);
}
