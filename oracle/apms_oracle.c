/*
 * APMSqueeze reference oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow CPU statement of what one step of the
 * compression stage of APMSqueeze computes (Algorithm 1, lines 3-12, in the
 * parameter-server form of the supplement, "Proof to the Updating Form",
 * steps 1-3, applied to every chunk independently), of the 1-bit
 * compression operator (Section 5.1, "Compression Method"), and of one step
 * of the Adam warm-up (Section 3.2, "Original Adam").
 *
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may call
 * this file.  It shares no code, header, table or helper with the HIP
 * library and includes none of its headers.
 *
 * Arithmetic contract (the paper is silent on all of it; these are the
 * readings this build fixes):
 *   - every elementwise operation is one IEEE-754 binary32 operation, rounded
 *     to nearest-even, in the order written below; no fused multiply-add
 *     (compile with -ffp-contract=off, no -ffast-math); denormals are kept;
 *   - the squared l2 norm behind a scale is the exact sum of the exact
 *     squares: each square is formed in a wider type where it is exact and
 *     the sum is carried in `long double`.  THIS ASSUMES x86-64, where long
 *     double is the x87 80-bit format (64-bit significand): the sum's error is
 *     then far below one binary64 ulp for any chunk length used here.  On a
 *     host whose long double is binary64 the sum is an ordinary binary64
 *     accumulation and "exact" weakens to a relative error of about L * 1e-16
 *     (the file refuses to compile there, see the check below);
 *     it is rounded to binary64 once, divided by the chunk length and square
 *     rooted in binary64, then rounded once to binary32;
 *   - sign(0) = +1: the sign bit sent is (u >= 0), so -0.0 maps to +1;
 *   - sign words are packed LSB-first: element j of a worker's vector is bit
 *     (j & 31) of word (j >> 5); bit 1 means +scale, bit 0 means -scale;
 *   - the server sums the n decoded values in worker order 0..n-1 and then
 *     multiplies by fl(1/n).
 *
 * Threads: single-threaded unless apms_oracle_set_threads() asks for more (and
 * the file was compiled with OpenMP).  Only independent work is spread: whole
 * (worker, chunk) problems, whole chunks, or single elements of a loop that has
 * no carried value; every sum runs in one thread in index order, so the results
 * are the same bits for any thread count.
 *
 * Parity status: the trajectory VALUES have no printed worked example in the
 * paper ("parity unpinned" for those); every function here is pinned by the
 * invariants, closed forms, special cases and brute-force checks in
 * tests/test_oracle_pins.py.
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#if LDBL_MANT_DIG < 64
#error "the norm accumulator needs a long double with a 64-bit significand (x86-64)"
#endif

/* Threads the loops over independent work may use (1 = serial, the default). */
static int oracle_threads = 1;

void apms_oracle_set_threads(int threads)
{
    oracle_threads = threads > 1 ? threads : 1;
}

#define APMS_ORACLE_ONEBIT 0   /* sign + l2 scale, Section 5.1            */
#define APMS_ORACLE_IDENTITY 1 /* C[u] = u: the "uncompressed" variant of  */
                               /* Section 5.3 (freeze v, no compression)   */

/* ------------------------------------------------------------------------ */
/* The compression operator C[.] on one chunk, and its decoder.             */
/* ------------------------------------------------------------------------ */

/*
 * Section 5.1: keep the sign of every element and one scaling factor equal to
 * (magnitude of the compensated vector) / (magnitude of the quantized one).
 * With the l2 norm of the paper's notation the quantized vector (all +-1) has
 * norm sqrt(L), so scale = ||u||_2 / sqrt(L) = sqrt(sum u^2 / L).
 *
 * u[0..L)        chunk to compress
 * words[0..L/32) packed signs (written only for ONEBIT)
 * *scale         scaling factor (ONEBIT), 1.0f for IDENTITY
 * c[0..L)        decoded value C[u], what a receiver reconstructs
 */
static void compress_chunk(int compressor, const float *u, int64_t L,
                           uint32_t *words, float *scale, float *c)
{
    if (compressor == APMS_ORACLE_IDENTITY) {
        for (int64_t j = 0; j < L; ++j)
            c[j] = u[j];
        *scale = 1.0f;
        return;
    }
    long double S = 0.0L;
    for (int64_t j = 0; j < L; ++j)
        S += (long double)u[j] * (long double)u[j];
    double mean_sq = (double)S / (double)L;
    float s = (float)sqrt(mean_sq);
    *scale = s;
    for (int64_t w = 0; w < L / 32; ++w)
        words[w] = 0u;
    for (int64_t j = 0; j < L; ++j) {
        int positive = (u[j] >= 0.0f);
        if (positive)
            words[j >> 5] |= (uint32_t)1u << (j & 31);
        c[j] = positive ? s : -s;
    }
}

/* Decoded value of element j of a chunk, from its wire form. */
static float decode_elem(int compressor, const uint32_t *words, float scale,
                         const float *dense, int64_t j)
{
    if (compressor == APMS_ORACLE_IDENTITY)
        return dense[j];
    return ((words[j >> 5] >> (j & 31)) & 1u) ? scale : -scale;
}

/* ------------------------------------------------------------------------ */
/* Worker side: supplement step 1 (Algorithm 1, lines 6-7).                 */
/* ------------------------------------------------------------------------ */

/*
 * For every worker i and chunk k:
 *     m_i   = beta * m + (1 - beta) * g_i          (local momentum)
 *     u     = m_i + delta_i                        (error compensation)
 *     send C[u];   delta_i <- u - C[u]
 *
 * d       vector length, a multiple of L;  L a multiple of 32
 * m       [n][d] momentum slices (read only: the local m_i is never stored,
 *         the gather of step 3 overwrites it).  NULL selects the APGSqueeze
 *         variant of Section 5.3 (item 4), which error-compensates and
 *         compresses the GRADIENT instead of the momentum: u = g_i + delta_i.
 * g       [n][d] local stochastic gradients
 * werr    [n][d] worker errors delta_i, updated in place
 * packed  [n][d/32] sign words out            (ONEBIT)
 * scales  [n][d/L] one scale per worker chunk (ONEBIT; 1.0f for IDENTITY)
 * dense   [n][d] decoded messages out (required for IDENTITY, where it IS the
 *         wire form; optional, may be NULL, for ONEBIT)
 * Returns 0, or -1 when the temporary chunk buffers cannot be allocated.
 */
int apms_oracle_compress(int compressor, int64_t d, int32_t n, int64_t L,
                         const float *m, const float *g, float *werr,
                         uint32_t *packed, float *scales, float *dense,
                         float beta)
{
    if (d == 0)
        return 0;
    const int64_t C = d / L;
    const float one_minus_beta = 1.0f - beta;
    int failed = 0;
    /* every (worker, chunk) pair is a problem of its own */
#pragma omp parallel for schedule(dynamic) num_threads(oracle_threads) reduction(| : failed)
    for (int64_t pair = 0; pair < (int64_t)n * C; ++pair) {
        const int32_t i = (int32_t)(pair / C);
        const int64_t k = pair % C;
        float *u = (float *)malloc((size_t)L * sizeof(float));
        float *c = (float *)malloc((size_t)L * sizeof(float));
        if (!u || !c) {
            free(u);
            free(c);
            failed = 1;
            continue;
        }
        const int64_t base = (int64_t)i * d + k * L;
        for (int64_t j = 0; j < L; ++j) {
            if (!m) {
                u[j] = g[base + j] + werr[base + j];
                continue;
            }
            float bm = beta * m[base + j];
            float bg = one_minus_beta * g[base + j];
            float mi = bm + bg;
            u[j] = mi + werr[base + j];
        }
        uint32_t *words = packed ? packed + base / 32 : NULL;
        compress_chunk(compressor, u, L, words, &scales[(int64_t)i * C + k], c);
        for (int64_t j = 0; j < L; ++j) {
            werr[base + j] = u[j] - c[j];
            if (dense)
                dense[base + j] = c[j];
        }
        free(u);
        free(c);
    }
    return failed ? -1 : 0;
}

/* ------------------------------------------------------------------------ */
/* Server side: supplement step 2 (Algorithm 1, line 9).                    */
/* ------------------------------------------------------------------------ */

/*
 * For every chunk k (served by worker k in the paper; here just chunk k):
 *     a     = (1/n) * sum_{i=0}^{n-1} C[u_i]        (average of the n messages)
 *     ubar  = a + deltabar
 *     send C[ubar];   deltabar <- ubar - C[ubar]
 *
 * packed, scales, dense   the n workers' messages as written by
 *                         apms_oracle_compress
 * serr     [d] server error deltabar, updated in place
 * spacked  [d/32] server sign words out (ONEBIT)
 * sscales  [d/L]  server scales out     (ONEBIT; 1.0f for IDENTITY)
 * sdense   [d]    decoded server message out (required for IDENTITY)
 */
int apms_oracle_server_reduce(int compressor, int64_t d, int32_t n, int64_t L,
                              const uint32_t *packed, const float *scales,
                              const float *dense, float *serr,
                              uint32_t *spacked, float *sscales, float *sdense)
{
    if (d == 0)
        return 0;
    const int64_t C = d / L;
    const float inv_n = 1.0f / (float)n;
    int failed = 0;
    /* chunks are independent; with fewer chunks than threads the threads share the elements of the
       averaging loop instead (no value is carried from one element to the next) */
#pragma omp parallel for schedule(dynamic) num_threads(oracle_threads) reduction(| : failed) if (C >= oracle_threads)
    for (int64_t k = 0; k < C; ++k) {
        float *ubar = (float *)malloc((size_t)L * sizeof(float));
        float *c = (float *)malloc((size_t)L * sizeof(float));
        if (!ubar || !c) {
            free(ubar);
            free(c);
            failed = 1;
            continue;
        }
        const int64_t base = k * L;
#pragma omp parallel for num_threads(oracle_threads)
        for (int64_t j = 0; j < L; ++j) {
            float acc = 0.0f;
            for (int32_t i = 0; i < n; ++i) {
                const int64_t wbase = (int64_t)i * d + base;
                acc = acc + decode_elem(compressor,
                                        packed ? packed + wbase / 32 : NULL,
                                        scales[(int64_t)i * C + k],
                                        dense ? dense + wbase : NULL, j);
            }
            float avg = acc * inv_n;
            ubar[j] = avg + serr[base + j];
        }
        compress_chunk(compressor, ubar, L, spacked ? spacked + base / 32 : NULL,
                       &sscales[k], c);
        for (int64_t j = 0; j < L; ++j) {
            serr[base + j] = ubar[j] - c[j];
            if (sdense)
                sdense[base + j] = c[j];
        }
        free(ubar);
        free(c);
    }
    return failed ? -1 : 0;
}

/* ------------------------------------------------------------------------ */
/* Gather + model update: supplement step 3 (Algorithm 1, lines 10-11).     */
/* ------------------------------------------------------------------------ */

/*
 * Every worker replaces its momentum by the server's decoded message and
 * takes the step preconditioned by the variance frozen at the end of the
 * warm-up:
 *     m_i <- C[ubar]   for all i
 *     x   <- x - lr * m / (sqrt(v) + eps)
 * The paper's update has no eps (it divides by sqrt(v)); eps = 0 reproduces
 * it literally, eps > 0 is the guard Adam itself carries (Section 3.2).
 * No bias correction in this stage.
 *
 * v [d] frozen variance (read only);  x [d] model, in place;
 * m [n][d] momentum slices, all n overwritten with the same values.
 */
int apms_oracle_apply(int compressor, int64_t d, int32_t n, int64_t L,
                      const uint32_t *spacked, const float *sscales,
                      const float *sdense, const float *v, float *x, float *m,
                      float lr, float eps)
{
#pragma omp parallel for num_threads(oracle_threads)
    for (int64_t j = 0; j < d; ++j) {
        const int64_t k = j / L;
        const int64_t base = k * L;
        float mj = decode_elem(compressor, spacked ? spacked + base / 32 : NULL,
                               sscales[k], sdense ? sdense + base : NULL,
                               j - base);
        for (int32_t i = 0; i < n; ++i)
            m[(int64_t)i * d + j] = mj;
        float root = sqrtf(v[j]);
        float denom = root + eps;
        float ratio = mj / denom;
        float step = lr * ratio;
        x[j] = x[j] - step;
    }
    return 0;
}

/*
 * APGSqueeze (Section 5.3, item 4) after the gather: the decoded server message is the averaged,
 * doubly compressed GRADIENT ghat; every worker then takes the momentum step itself,
 *     m_i <- beta * m_i + (1 - beta) * ghat      for all i
 *     x   <- x - lr * m / (sqrt(v) + eps)         (worker 0's m; all slices agree if they started equal)
 * The paper gives the variant one sentence; that the momentum is formed from the decoded gradient and
 * the variance stays frozen is this build's reading.
 */
int apms_oracle_apply_gradient(int compressor, int64_t d, int32_t n, int64_t L,
                               const uint32_t *spacked, const float *sscales,
                               const float *sdense, const float *v, float *x, float *m,
                               float lr, float beta, float eps)
{
    const float one_minus_beta = 1.0f - beta;
    for (int64_t j = 0; j < d; ++j) {
        const int64_t k = j / L;
        const int64_t base = k * L;
        const uint32_t *chunk_words = spacked ? spacked + base / 32 : NULL;
        const float *chunk_dense = sdense ? sdense + base : NULL;
        float ghat = decode_elem(compressor, chunk_words, sscales[k], chunk_dense, j - base);
        for (int32_t i = 0; i < n; ++i) {
            float keep = beta * m[(int64_t)i * d + j];
            float inc = one_minus_beta * ghat;
            m[(int64_t)i * d + j] = keep + inc;
        }
        float root_v = sqrtf(v[j]);
        float precond = root_v + eps;
        float direction = m[j] / precond;
        float delta_x = lr * direction;
        x[j] = x[j] - delta_x;
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Warm-up: one step of the original Adam (Section 3.2) on the average of   */
/* the n workers' gradients (Algorithm 1, line 2).                          */
/* ------------------------------------------------------------------------ */

/*
 *     gbar = (1/n) sum_i g_i           (full-precision average, worker order)
 *     m <- beta1 m + (1-beta1) gbar ;  v <- beta2 v + (1-beta2) gbar^2
 *     mhat = m / (1-beta1^t) ;  vhat = v / (1-beta2^t)
 *     x <- x - lr * mhat / (sqrt(vhat) + eps)
 * t is the 1-based index of this step.  The two bias-correction denominators
 * are formed in binary64 and rounded to binary32 once.
 * x, m, v are [d]; g is [n][d].
 */
int apms_oracle_warmup_step(int64_t d, int32_t n, float *x, float *m, float *v,
                            const float *g, float lr, float beta1, float beta2,
                            float eps, int64_t t)
{
    const float inv_n = 1.0f / (float)n;
    const float omb1 = 1.0f - beta1;
    const float omb2 = 1.0f - beta2;
    const float bc1 = (float)(1.0 - pow((double)beta1, (double)t));
    const float bc2 = (float)(1.0 - pow((double)beta2, (double)t));
#pragma omp parallel for num_threads(oracle_threads)
    for (int64_t j = 0; j < d; ++j) {
        float acc = 0.0f;
        for (int32_t i = 0; i < n; ++i)
            acc = acc + g[(int64_t)i * d + j];
        float gbar = acc * inv_n;
        float m_new = beta1 * m[j];
        float m_inc = omb1 * gbar;
        m_new = m_new + m_inc;
        float gsq = gbar * gbar;
        float v_new = beta2 * v[j];
        float v_inc = omb2 * gsq;
        v_new = v_new + v_inc;
        m[j] = m_new;
        v[j] = v_new;
        float mhat = m_new / bc1;
        float vhat = v_new / bc2;
        float root = sqrtf(vhat);
        float denom = root + eps;
        float ratio = mhat / denom;
        float step = lr * ratio;
        x[j] = x[j] - step;
    }
    return 0;
}

/*
 * Hand-over from the warm-up to the compression stage (Algorithm 1, line 1
 * initialisation of the errors, and line 3): the warm-up momentum becomes
 * every worker's momentum, both error vectors start at zero, v is frozen as
 * it stands (raw, not bias-corrected).
 * m_warm [d] in;  m [n][d], werr [n][d], serr [d] out.
 */
int apms_oracle_freeze(int64_t d, int32_t n, const float *m_warm, float *m,
                       float *werr, float *serr)
{
    for (int32_t i = 0; i < n; ++i) {
        memmove(m + (int64_t)i * d, m_warm, (size_t)d * sizeof(float));
        memset(werr + (int64_t)i * d, 0, (size_t)d * sizeof(float));
    }
    memset(serr, 0, (size_t)d * sizeof(float));
    return 0;
}

/* ------------------------------------------------------------------------ */
/* 16-bit gradient inputs (Section 5.1 trains in a 16-bit float type).       */
/* ------------------------------------------------------------------------ */

#define APMS_ORACLE_GRAD_F16 1  /* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits */
#define APMS_ORACLE_GRAD_BF16 2 /* bfloat16: 1 sign, 8 exponent (bias 127), 7 fraction bits     */

/*
 * Widen 16-bit gradient values to binary32.  Every binary16 / bfloat16 value is
 * exactly representable in binary32, so this is the value map of the formats'
 * definitions, written out with ldexp; the step itself then runs on the widened
 * values with the arithmetic stated at the top of this file.  NaN payloads are
 * not preserved (NaN is outside the contract).
 */
int apms_oracle_widen_g16(int format, int64_t count, const uint16_t *in, float *out)
{
    const int exp_bits = (format == APMS_ORACLE_GRAD_F16) ? 5 : 8;
    const int frac_bits = 15 - exp_bits;
    const int bias = (1 << (exp_bits - 1)) - 1;
    const int exp_max = (1 << exp_bits) - 1;
    if (format != APMS_ORACLE_GRAD_F16 && format != APMS_ORACLE_GRAD_BF16)
        return -1;
    for (int64_t j = 0; j < count; ++j) {
        const unsigned h = in[j];
        const int negative = (h >> 15) & 1;
        const int e = (h >> frac_bits) & exp_max;
        const int f = h & ((1 << frac_bits) - 1);
        double value;
        if (e == exp_max)
            value = f ? NAN : INFINITY;
        else if (e == 0)
            value = ldexp((double)f, 1 - bias - frac_bits);              /* zero and subnormals */
        else
            value = ldexp((double)((1 << frac_bits) + f), e - bias - frac_bits);
        out[j] = (float)(negative ? -value : value);
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Top-k compressor (Section 5.1, second bullet) under the same             */
/* error-compensated worker / server / gather structure.                    */
/* ------------------------------------------------------------------------ */

/*
 * Top-k operator of Section 5.1, second bullet: C[u] keeps the K elements of
 * largest |u| of a chunk (K = the stated percentage of its length) and zeroes
 * the rest.  The paper
 * does not say what happens between equal magnitudes; this build keeps the
 * LOWER index first, which makes the result unique.  The wire form of a
 * chunk is K (index, value) pairs, indices local to the chunk, ascending.
 * Here: order all L indices by (|u| descending, index ascending) with the
 * library sort, take the first K, and list them by ascending index.
 */
static const float *topk_sort_values; /* qsort has no context argument */

static int topk_by_magnitude(const void *pa, const void *pb)
{
    const uint32_t a = *(const uint32_t *)pa, b = *(const uint32_t *)pb;
    const float ma = fabsf(topk_sort_values[a]), mb = fabsf(topk_sort_values[b]);
    if (ma > mb) return -1;
    if (ma < mb) return 1;
    return (a < b) ? -1 : (a > b);
}

static int topk_by_index(const void *pa, const void *pb)
{
    const uint32_t a = *(const uint32_t *)pa, b = *(const uint32_t *)pb;
    return (a < b) ? -1 : (a > b);
}

/* u[0..L) in; idx[0..K), val[0..K) wire form out; c[0..L) decoded C[u] out. */
static int compress_chunk_topk(const float *u, int64_t L, int64_t K, uint32_t *idx, float *val, float *c)
{
    uint32_t *order = (uint32_t *)malloc((size_t)L * sizeof(uint32_t));
    if (!order)
        return -1;
    for (int64_t j = 0; j < L; ++j)
        order[j] = (uint32_t)j;
    topk_sort_values = u;
    qsort(order, (size_t)L, sizeof(uint32_t), topk_by_magnitude);
    qsort(order, (size_t)K, sizeof(uint32_t), topk_by_index);
    for (int64_t j = 0; j < L; ++j)
        c[j] = 0.0f;
    for (int64_t t = 0; t < K; ++t) {
        idx[t] = order[t];
        val[t] = u[order[t]];
        c[order[t]] = u[order[t]];
    }
    free(order);
    return 0;
}

/* Value of element j of a chunk decoded from its (idx, val) list (0 if absent). */
static float decode_topk_elem(const uint32_t *idx, const float *val, int64_t K, int64_t j)
{
    for (int64_t t = 0; t < K; ++t)
        if ((int64_t)idx[t] == j)
            return val[t];
    return 0.0f;
}

/*
 * Worker step with the top-k compressor (same equations as apms_oracle_compress):
 *   u = beta*m_i + (1-beta)*g_i + delta_i ;  send C[u] ;  delta_i <- u - C[u]
 * idx, val: [n][d/L][K] out.  1 <= K <= L.
 */
int apms_oracle_topk_compress(int64_t d, int32_t n, int64_t L, int64_t K, const float *m, const float *g,
                              float *werr, uint32_t *idx, float *val, float beta)
{
    if (d == 0)
        return 0;
    const int64_t C = d / L;
    const float one_minus_beta = 1.0f - beta;
    float *u = (float *)malloc((size_t)L * sizeof(float));
    float *sent = (float *)malloc((size_t)L * sizeof(float));
    int rc = (u && sent) ? 0 : -1;
    for (int32_t i = 0; i < n && !rc; ++i) {
        for (int64_t k = 0; k < C && !rc; ++k) {
            const int64_t base = (int64_t)i * d + k * L;
            for (int64_t j = 0; j < L; ++j) {
                float keep_m = beta * m[base + j];
                float new_g = one_minus_beta * g[base + j];
                float local_m = keep_m + new_g;
                u[j] = local_m + werr[base + j];
            }
            const int64_t out = ((int64_t)i * C + k) * K;
            rc = compress_chunk_topk(u, L, K, idx + out, val + out, sent);
            for (int64_t j = 0; j < L && !rc; ++j)
                werr[base + j] = u[j] - sent[j];
        }
    }
    free(u);
    free(sent);
    return rc;
}

/*
 * Server step with the top-k compressor: ubar = (1/n) sum_i C[u_i] + deltabar (the n decoded messages
 * summed in worker order, zeros included) ; send C[ubar] ; deltabar <- ubar - C[ubar].
 * idx, val: [n][C][K] in;  sidx, sval: [C][K] out.
 */
int apms_oracle_topk_server_reduce(int64_t d, int32_t n, int64_t L, int64_t K, const uint32_t *idx,
                                   const float *val, float *serr, uint32_t *sidx, float *sval)
{
    if (d == 0)
        return 0;
    const int64_t C = d / L;
    const float inv_n = 1.0f / (float)n;
    float *ubar = (float *)malloc((size_t)L * sizeof(float));
    float *sent = (float *)malloc((size_t)L * sizeof(float));
    float *dense = (float *)malloc((size_t)L * sizeof(float));
    int rc = (ubar && sent && dense) ? 0 : -1;
    for (int64_t k = 0; k < C && !rc; ++k) {
        const int64_t base = k * L;
        for (int64_t j = 0; j < L; ++j)
            ubar[j] = 0.0f;
        for (int32_t i = 0; i < n; ++i) {
            /* decode worker i's message densely, then add it: ubar holds the running sum */
            const int64_t in = ((int64_t)i * C + k) * K;
            for (int64_t j = 0; j < L; ++j)
                dense[j] = 0.0f;
            for (int64_t t = 0; t < K; ++t)
                dense[idx[in + t]] = val[in + t];
            for (int64_t j = 0; j < L; ++j)
                ubar[j] = ubar[j] + dense[j];
        }
        for (int64_t j = 0; j < L; ++j) {
            float mean = ubar[j] * inv_n;
            ubar[j] = mean + serr[base + j];
        }
        rc = compress_chunk_topk(ubar, L, K, sidx + k * K, sval + k * K, sent);
        for (int64_t j = 0; j < L && !rc; ++j)
            serr[base + j] = ubar[j] - sent[j];
    }
    free(ubar);
    free(sent);
    free(dense);
    return rc;
}

/*
 * Gather + model update with the top-k compressor: m_i <- C[ubar] (dense: zero outside the K kept
 * positions of each chunk), x <- x - lr * m / (sqrt(v) + eps).
 */
int apms_oracle_topk_apply(int64_t d, int32_t n, int64_t L, int64_t K, const uint32_t *sidx,
                           const float *sval, const float *v, float *x, float *m, float lr, float eps)
{
    for (int64_t j = 0; j < d; ++j) {
        const int64_t k = j / L;
        float gathered = decode_topk_elem(sidx + k * K, sval + k * K, K, j - k * L);
        for (int32_t i = 0; i < n; ++i)
            m[(int64_t)i * d + j] = gathered;
        float root_of_v = sqrtf(v[j]);
        float divisor = root_of_v + eps;
        float scaled = gathered / divisor;
        float move = lr * scaled;
        x[j] = x[j] - move;
    }
    return 0;
}
