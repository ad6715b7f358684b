/*
 * dlion_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain, slow, one-coordinate-at-a-time CPU implementation of one iteration of
 * Distributed Lion (Algorithm 1; Section 3.2), used only by the tests, the
 * smoke check and the benchmark's CPU-baseline leg.  It shares no code with
 * the HIP library and nothing in the product path may call it.
 *
 * Precision: the build's target fixes fp32 state and fp32 arithmetic with
 * every multiply, add, subtract and divide rounded on its own (no fused
 * multiply-add), so this file must be compiled with -ffp-contract=off and
 * without any fast-math or flush-to-zero option.  Gradients may be bf16; they
 * are widened to fp32 exactly (bit pattern << 16) before use.
 *
 * Readings where the paper is silent (each also listed in the design notes):
 *   - the worker's sign maps 0 and -0 to +1, so the update is truly one bit;
 *   - the integer the server works with is p = number of +1 votes in {0..N};
 *     the sum of the +-1 votes is S = 2p - N;
 *   - majority vote of a tie (S = 0) is 0;
 *   - bit j%64 of word j/64 (LSB first) carries coordinate j, +1 -> 1,
 *     -1 -> 0, bits past d are 0;
 *   - (1 - beta) is formed once, in fp32;
 *   - expressions are evaluated in the literal form the equations are written.
 *
 * Parity pins: every function here is pinned by the CPU tests (N=1 against a
 * separately written single-worker Lion, hand-worked dyadic vectors, closed
 * forms, brute force over all sign patterns, invariants).  Nothing is
 * "parity unpinned".
 */
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_VOTE = 0, ORACLE_AVG = 1 };
enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

static float bf16_bits_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static float grad_at(const void *g, int g_dtype, int64_t idx)
{
    if (g_dtype == ORACLE_BF16)
        return bf16_bits_to_f32(((const uint16_t *)g)[idx]);
    return ((const float *)g)[idx];
}

/*
 * Worker side (Section 3.2, first display; Algorithm 1, worker-side lines):
 *   delta_i = sign(beta1 * m_i + (1 - beta1) * g_i)
 *   m_i    <- beta2 * m_i + (1 - beta2) * g_i          (old m_i on the right)
 * Worker i lives at m + i*m_stride, g + i*g_stride (strides in elements),
 * its packed update at packed + i*packed_stride (uint64 words).
 * delta (may be NULL) receives the same update as +-1 bytes, [N][d] dense,
 * so that the packing can be cross-checked.
 */
void oracle_worker_step(float *m, int64_t m_stride, const void *g, int64_t g_stride,
                        int g_dtype, uint64_t *packed, int64_t packed_stride,
                        int8_t *delta, int64_t d, int32_t N, float beta1, float beta2)
{
    const float one_minus_beta1 = 1.0f - beta1;
    const float one_minus_beta2 = 1.0f - beta2;
    const int64_t W = (d + 63) / 64;

    for (int32_t i = 0; i < N; ++i) {
        float *mi = m + (int64_t)i * m_stride;
        uint64_t *pi = packed + (int64_t)i * packed_stride;
        for (int64_t w = 0; w < W; ++w)
            pi[w] = 0;
        for (int64_t j = 0; j < d; ++j) {
            float gij = grad_at(g, g_dtype, (int64_t)i * g_stride + j);
            float a = beta1 * mi[j];
            float b = one_minus_beta1 * gij;
            float c = a + b;
            int plus = !(c < 0.0f); /* sign(0) -> +1 */
            if (plus)
                pi[j / 64] |= (uint64_t)1 << (j % 64);
            if (delta)
                delta[(int64_t)i * d + j] = plus ? 1 : -1;
            float a2 = beta2 * mi[j];
            float b2 = one_minus_beta2 * gij;
            mi[j] = a2 + b2;
        }
    }
}

/*
 * Server side, first half (Section 3.2: S_t = sum_i delta_i): the count of +1
 * votes per coordinate, read back out of the packed words.
 */
void oracle_aggregate_packed(const uint64_t *packed, int64_t packed_stride, int64_t d,
                             int32_t N, uint16_t *counts)
{
    for (int64_t j = 0; j < d; ++j) {
        uint32_t p = 0;
        for (int32_t i = 0; i < N; ++i) {
            uint64_t word = packed[(int64_t)i * packed_stride + j / 64];
            p += (uint32_t)((word >> (j % 64)) & 1u);
        }
        counts[j] = (uint16_t)p;
    }
}

/* Same count, taken from the +-1 bytes instead of the packed words. */
void oracle_aggregate_signs(const int8_t *delta, int64_t d, int32_t N, uint16_t *counts)
{
    for (int64_t j = 0; j < d; ++j) {
        int32_t S = 0;
        for (int32_t i = 0; i < N; ++i)
            S += delta[(int64_t)i * d + j];
        /* S = 2p - N */
        counts[j] = (uint16_t)((S + N) / 2);
    }
}

/*
 * Server side, second half, and the weight update (Section 3.2, second and
 * third displays; Algorithm 1, server-side):
 *   Delta = S / N (averaging)  or  sign(S) (majority vote, tie -> 0)
 *   x    <- x - lr * (Delta + lambda * x)
 * delta_out (may be NULL) receives Delta as fp32.
 */
void oracle_apply(float *x, const uint16_t *counts, int64_t d, int32_t N, int mode,
                  float lr, float lambda, float *delta_out)
{
    for (int64_t j = 0; j < d; ++j) {
        int32_t S = 2 * (int32_t)counts[j] - N;
        float Delta;
        if (mode == ORACLE_AVG)
            Delta = (float)S / (float)N;
        else
            Delta = (float)((S > 0) - (S < 0));
        float t = lambda * x[j];
        float u = Delta + t;
        float v = lr * u;
        x[j] = x[j] - v;
        if (delta_out)
            delta_out[j] = Delta;
    }
}

/*
 * One whole iteration for N workers: worker step, count, aggregate, apply.
 * packed must hold N*packed_stride words and counts d entries (both are
 * outputs the caller may inspect).
 */
void oracle_step(float *x, float *m, int64_t m_stride, const void *g, int64_t g_stride,
                 int g_dtype, int64_t d, int32_t N, int mode, float beta1, float beta2,
                 float lr, float lambda, uint64_t *packed, int64_t packed_stride,
                 uint16_t *counts)
{
    oracle_worker_step(m, m_stride, g, g_stride, g_dtype, packed, packed_stride, NULL, d, N,
                       beta1, beta2);
    oracle_aggregate_packed(packed, packed_stride, d, N, counts);
    oracle_apply(x, counts, d, N, mode, lr, lambda, NULL);
}

/*
 * The same iteration with the coordinate range cut into word-aligned pieces,
 * one per thread.  Coordinates never interact and every piece starts on a
 * 64-coordinate boundary, so each thread simply runs oracle_step on shifted
 * pointers; the result is identical for any thread count.
 */
struct piece {
    float *x, *m;
    const void *g;
    uint64_t *packed;
    uint16_t *counts;
    int64_t m_stride, g_stride, packed_stride, d;
    int32_t N;
    int g_dtype, mode;
    float beta1, beta2, lr, lambda;
};

static void *run_piece(void *arg)
{
    struct piece *p = (struct piece *)arg;
    if (p->d > 0)
        oracle_step(p->x, p->m, p->m_stride, p->g, p->g_stride, p->g_dtype, p->d, p->N, p->mode,
                    p->beta1, p->beta2, p->lr, p->lambda, p->packed, p->packed_stride, p->counts);
    return NULL;
}

int oracle_step_threads(float *x, float *m, int64_t m_stride, const void *g, int64_t g_stride,
                        int g_dtype, int64_t d, int32_t N, int mode, float beta1, float beta2,
                        float lr, float lambda, uint64_t *packed, int64_t packed_stride,
                        uint16_t *counts, int nthreads)
{
    if (nthreads < 1)
        nthreads = 1;
    const int64_t W = (d + 63) / 64;
    const int64_t words_per_piece = (W + nthreads - 1) / nthreads;
    struct piece *pieces = (struct piece *)calloc((size_t)nthreads, sizeof *pieces);
    pthread_t *tids = (pthread_t *)calloc((size_t)nthreads, sizeof *tids);
    char *started = (char *)calloc((size_t)nthreads, 1);
    if (!pieces || !tids || !started) {
        free(pieces);
        free(tids);
        free(started);
        return -1;
    }
    const int64_t g_elem = (g_dtype == ORACLE_BF16) ? 2 : 4;
    for (int t = 0; t < nthreads; ++t) {
        int64_t w0 = (int64_t)t * words_per_piece;
        int64_t w1 = w0 + words_per_piece;
        if (w0 > W) w0 = W;
        if (w1 > W) w1 = W;
        int64_t j0 = w0 * 64;
        int64_t j1 = w1 * 64;
        if (j1 > d) j1 = d;
        struct piece *p = &pieces[t];
        p->x = x + j0;
        p->m = m + j0;
        p->g = (const char *)g + j0 * g_elem;
        p->packed = packed + w0;
        p->counts = counts + j0;
        p->m_stride = m_stride;
        p->g_stride = g_stride;
        p->packed_stride = packed_stride;
        p->d = (j1 > j0) ? (j1 - j0) : 0;
        p->N = N;
        p->g_dtype = g_dtype;
        p->mode = mode;
        p->beta1 = beta1;
        p->beta2 = beta2;
        p->lr = lr;
        p->lambda = lambda;
    }
    int rc = 0;
    for (int t = 0; t < nthreads; ++t) {
        if (pthread_create(&tids[t], NULL, run_piece, &pieces[t]) == 0) {
            started[t] = 1;
        } else {
            run_piece(&pieces[t]); /* no thread available: do the piece here */
            rc = 1;
        }
    }
    for (int t = 0; t < nthreads; ++t)
        if (started[t])
            pthread_join(tids[t], NULL);
    free(pieces);
    free(tids);
    free(started);
    return rc;
}

/* ------------------------------------------------------------------------- *
 * Server -> worker message for Delta ("Communication Cost" paragraph; Table 1).
 *
 * The aggregated update is sent as bit-planes over the same 64-coordinate
 * words as the workers' messages (bit j%64 of word j/64 = coordinate j):
 *   majority vote : plane 0 ("plus")  bit = 1 iff S > 0;
 *                   plane 1 ("tie")   bit = 1 iff S == 0, present only when N
 *                   is even (an odd N cannot tie), so the message is d bits
 *                   for odd N as in Table 1 and 2d bits for even N (the
 *                   price of reading a tie as 0);
 *   averaging     : plane b holds bit b of the count p in {0..N}, for
 *                   b < bits(N) = ceil(log2(N+1)) -- the "log(N) d" of Table 1.
 * Bits past d are 0.
 * ------------------------------------------------------------------------- */
int oracle_delta_planes(int32_t N, int mode)
{
    if (mode == ORACLE_AVG) {
        int bits = 0;
        while (((int64_t)1 << bits) <= (int64_t)N)
            ++bits;
        return bits;
    }
    return (N % 2 == 0) ? 2 : 1;
}

void oracle_encode_delta(const uint16_t *counts, int64_t d, int32_t N, int mode, uint64_t *planes,
                         int64_t plane_stride)
{
    const int P = oracle_delta_planes(N, mode);
    const int64_t W = (d + 63) / 64;
    for (int b = 0; b < P; ++b)
        for (int64_t w = 0; w < W; ++w)
            planes[(int64_t)b * plane_stride + w] = 0;
    for (int64_t j = 0; j < d; ++j) {
        const uint64_t bit = (uint64_t)1 << (j % 64);
        if (mode == ORACLE_AVG) {
            for (int b = 0; b < P; ++b)
                if ((counts[j] >> b) & 1u)
                    planes[(int64_t)b * plane_stride + j / 64] |= bit;
        } else {
            int32_t S = 2 * (int32_t)counts[j] - N;
            if (S > 0)
                planes[j / 64] |= bit;
            if (S == 0)
                planes[plane_stride + j / 64] |= bit; /* S == 0 needs N even, so plane 1 exists */
        }
    }
}

/* What a worker does with the message: rebuild Delta and take the step
 * x <- x - lr*(Delta + lambda*x) (Section 3.2, third display). */
void oracle_apply_encoded(float *x, const uint64_t *planes, int64_t plane_stride, int64_t d, int32_t N,
                          int mode, float lr, float lambda, float *delta_out)
{
    const int P = oracle_delta_planes(N, mode);
    for (int64_t j = 0; j < d; ++j) {
        float Delta;
        if (mode == ORACLE_AVG) {
            int32_t p = 0;
            for (int b = 0; b < P; ++b)
                p |= (int32_t)((planes[(int64_t)b * plane_stride + j / 64] >> (j % 64)) & 1u) << b;
            Delta = (float)(2 * p - N) / (float)N;
        } else {
            int plus = (int)((planes[j / 64] >> (j % 64)) & 1u);
            int tie = (P > 1) ? (int)((planes[plane_stride + j / 64] >> (j % 64)) & 1u) : 0;
            Delta = plus ? 1.0f : (tie ? 0.0f : -1.0f);
        }
        float t = lambda * x[j];
        float u = Delta + t;
        float v = lr * u;
        x[j] = x[j] - v;
        if (delta_out)
            delta_out[j] = Delta;
    }
}

/* ------------------------------------------------------------------------- *
 * Worker step with each worker's own beta1, beta2 (footnote of Algorithm 1:
 * every worker may set its individual coefficients).  Same arithmetic as
 * oracle_worker_step with beta1[i], beta2[i] in place of the shared scalars.
 * With beta1[i] == beta2[i] this is the sign-momentum (SIGNUM) worker of the
 * D-SIGNUM comparison in Section 5.
 * ------------------------------------------------------------------------- */
void oracle_worker_step_pw(float *m, int64_t m_stride, const void *g, int64_t g_stride, int g_dtype,
                           uint64_t *packed, int64_t packed_stride, int64_t d, int32_t N,
                           const float *beta1, const float *beta2)
{
    const int64_t W = (d + 63) / 64;
    for (int32_t i = 0; i < N; ++i) {
        const float one_minus_beta1 = 1.0f - beta1[i];
        const float one_minus_beta2 = 1.0f - beta2[i];
        float *mi = m + (int64_t)i * m_stride;
        uint64_t *pi = packed + (int64_t)i * packed_stride;
        for (int64_t w = 0; w < W; ++w)
            pi[w] = 0;
        for (int64_t j = 0; j < d; ++j) {
            float gij = grad_at(g, g_dtype, (int64_t)i * g_stride + j);
            float a = beta1[i] * mi[j];
            float b = one_minus_beta1 * gij;
            float c = a + b;
            if (!(c < 0.0f))
                pi[j / 64] |= (uint64_t)1 << (j % 64);
            float a2 = beta2[i] * mi[j];
            float b2 = one_minus_beta2 * gij;
            mi[j] = a2 + b2;
        }
    }
}

/* ------------------------------------------------------------------------- *
 * Global Lion (Appendix, "Global Lion Convergence", the displayed scheme; the
 * G-Lion baseline of Section 5): every worker forms its blend
 *   c_i = beta1*m_i + (1-beta1)*g_i,  m_i <- beta2*m_i + (1-beta2)*g_i,
 * the full-precision blends are averaged, and
 *   x <- x - lr*(sign(mean_i c_i) + lambda*x).
 * Readings: the mean is the fp32 sum over i = 0..N-1 in that order, divided by
 * (float)N; the sign maps 0 to +1 like the worker sign, so that N = 1 is the
 * same single-worker Lion that Distributed Lion reduces to.
 * sign_bits (may be NULL) receives the W words of sign(mean c), packed like a
 * worker's message.
 * ------------------------------------------------------------------------- */
void oracle_global_lion_step(float *x, float *m, int64_t m_stride, const void *g, int64_t g_stride,
                             int g_dtype, int64_t d, int32_t N, float beta1, float beta2, float lr,
                             float lambda, uint64_t *sign_bits)
{
    const float one_minus_beta1 = 1.0f - beta1;
    const float one_minus_beta2 = 1.0f - beta2;
    const int64_t W = (d + 63) / 64;
    if (sign_bits)
        for (int64_t w = 0; w < W; ++w)
            sign_bits[w] = 0;
    for (int64_t j = 0; j < d; ++j) {
        float sum = 0.0f;
        for (int32_t i = 0; i < N; ++i) {
            float *mij = m + (int64_t)i * m_stride + j;
            float gij = grad_at(g, g_dtype, (int64_t)i * g_stride + j);
            float a = beta1 * (*mij);
            float b = one_minus_beta1 * gij;
            float c = a + b;
            sum = sum + c;
            float a2 = beta2 * (*mij);
            float b2 = one_minus_beta2 * gij;
            *mij = a2 + b2;
        }
        float mean = sum / (float)N;
        float Delta = (mean < 0.0f) ? -1.0f : 1.0f;
        if (sign_bits && !(mean < 0.0f))
            sign_bits[j / 64] |= (uint64_t)1 << (j % 64);
        float t = lambda * x[j];
        float u = Delta + t;
        float v = lr * u;
        x[j] = x[j] - v;
    }
}
