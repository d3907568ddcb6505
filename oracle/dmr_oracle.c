/*
 * CPU oracle for the weight-only INT4 (W4A16) linear layer of a low-precision routed step,
 * and for its bf16 high-precision twin.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU library is
 * checked against.  It shares no code, header, table or helper with the HIP path, is never
 * linked into it, and only the test-suite, the smoke check and the benchmark's CPU-baseline
 * leg may call it.
 *
 * What the paper fixes (Sec. 5.1 "Experimental Models and Precision"; App. E "Per-cell
 * configuration"): the low-precision copy of the model stores every Linear weight in 4 bits
 * and keeps 16-bit activations; the high-precision copy is bf16.  The paper does not fix the
 * storage format, so the format below is this build's reading of it:
 *
 *   - codes q[n][k] in 0..15, eight per 32-bit word along k, code j of a word in bits
 *     [4j, 4j+4)                                                 ("canonical packing")
 *   - the 3-bit variant (the W3A16 group-128 cell of Sec. 5.1 / App. E, for which the paper had
 *     no kernel and projected T_W3 = T_W4 / 1.15 in App. A): codes 0..7, 32 per three 32-bit
 *     words along k, code j in bits [3j, 3j+3) of the 96-bit little-endian number formed by the
 *     three words; everything else is the same with 7 in place of 15.  Functions that take
 *     `bits` accept 3 or 4.
 *   - one bf16 scale s[n][G] and one bf16 zero point z[n][G] (an integer code 0..15 held
 *     in bf16) per group G = k / g of g consecutive k
 *   - w^[n][k] = (q[n][k] - z[n][G]) * s[n][G]                     (exact in fp64)
 *   - dequantize gives RNE_bf16(w^)                                (one correct answer)
 *   - forward gives  y[m][n] = sum_k x[m][k] * w^[n][k]   in fp64, k ascending
 *   - bf16 twin      y[m][n] = sum_k x[m][k] * W[n][k]    in fp64, k ascending
 *
 *   - decoder glue between the Linear layers of one routed step (the models of Sec. 5.1 are
 *     pre-norm decoders with RMSNorm and a SwiGLU MLP; the paper does not restate these
 *     operations, so they are written out here in their textbook form, all arithmetic in fp64
 *     with one rounding to bf16 at the end, because the next Linear takes bf16 activations):
 *       rmsnorm  out[m][k] = RNE_bf16( x[m][k] * gamma[k] / sqrt(mean_k(x[m][k]^2) + eps) )
 *       swiglu   out[m][i] = RNE_bf16( silu(in[m][i]) * in[m][I + i] ),  silu(a) = a / (1 + exp(-a))
 *     (the fused gate+up projection writes the gate half first, then the up half)
 *
 * Everything is row-major and contiguous.  bf16 values travel as uint16_t bit patterns.
 * All functions return 0 on success and a negative number on a bad argument.
 *
 * Parity status: every function here is pinned by the CPU tests (hand-worked 2x2 and 4x8
 * examples, pack/unpack bijection, zero-point-only and power-of-two-scale exact cases,
 * integer-matmul special case, closed-form quantiser error bound, an independent numpy
 * twin on tiny shapes; the glue by hand-worked vectors, closed forms and invariances).  oracle_forward on the large random configurations has no printed
 * value anywhere in the paper to compare with: beyond those pins it is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- bf16 <-> real ------------------------------------------------------------------ */

/* bf16 is the upper half of an IEEE binary32: 1 sign, 8 exponent, 7 fraction bits. */
double oracle_bf16_to_f64(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Round-to-nearest-even from the exact real value v (no intermediate binary32 rounding). */
uint16_t oracle_f64_to_bf16(double v)
{
    if (isnan(v)) return 0x7FC0;
    uint16_t sign = signbit(v) ? 0x8000 : 0;
    double a = fabs(v);
    if (a == 0.0) return sign;
    if (isinf(a)) return (uint16_t)(sign | 0x7F80);
    int e;
    (void)frexp(a, &e);             /* a = m * 2^e, m in [0.5,1)  ->  a in [2^(e-1), 2^e)   */
    int ex = e - 1;                 /* a = m' * 2^ex, m' in [1,2)                            */
    if (ex < -126) ex = -126;       /* subnormal range keeps the spacing of the last binade */
    double quantum = ldexp(1.0, ex - 7);          /* spacing of bf16 values around a        */
    double r = nearbyint(a / quantum);            /* exact scaling, then ties-to-even       */
    double rounded = r * quantum;                 /* exactly representable in binary32      */
    if (rounded >= ldexp(1.0, 128)) return (uint16_t)(sign | 0x7F80);
    float f = (float)rounded;
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return (uint16_t)(sign | (u >> 16));
}

uint16_t oracle_f32_to_bf16(float v) { return oracle_f64_to_bf16((double)v); }

void oracle_f32_to_bf16_array(int64_t count, const float *in, uint16_t *out)
{
    for (int64_t i = 0; i < count; ++i) out[i] = oracle_f32_to_bf16(in[i]);
}

void oracle_f64_to_bf16_array(int64_t count, const double *in, uint16_t *out)
{
    for (int64_t i = 0; i < count; ++i) out[i] = oracle_f64_to_bf16(in[i]);
}

/* ---- argument checks ---------------------------------------------------------------- */

static int bad_shape(int64_t K, int64_t N, int64_t g)
{
    return K <= 0 || N <= 0 || g <= 0 || (K % 8) != 0 || (K % g) != 0;
}

/* ---- quantiser: fp32 weights -> codes, scales, zero points --------------------------- */

/*
 * Asymmetric round-to-nearest per (row n, group G):
 *   lo = min(min_G w, 0), hi = max(max_G w, 0)        the range always contains 0
 *   s  = RNE_bf16( float32( (hi - lo) / 15 ) ),  s = 1 if that is 0
 *   z  = clamp( rint(-lo / s), 0, 15 )
 *   q  = clamp( rint(w / s) + z, 0, 15 )
 * with (hi - lo), the divisions and rint (ties to even) in fp64, and with the scale that is
 * actually stored (already rounded to bf16), so codes are the best ones for that scale.
 * q: uint8 [N][K] (one code per byte), s and z: bf16 bits [N][K/g].
 */
int oracle_quantize_bits(int64_t K, int64_t N, int64_t g, int bits, const float *w,
                         uint8_t *q, uint16_t *s_bits, uint16_t *z_bits)
{
    if (bad_shape(K, N, g) || (bits != 3 && bits != 4) || !w || !q || !s_bits || !z_bits) return -1;
    const double qmax = (double)((1 << bits) - 1);     /* 15 or 7 */
    const int64_t groups = K / g;
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t G = 0; G < groups; ++G) {
            const float *wg = w + n * K + G * g;
            float lo = 0.0f, hi = 0.0f;
            for (int64_t i = 0; i < g; ++i) {
                if (wg[i] < lo) lo = wg[i];
                if (wg[i] > hi) hi = wg[i];
            }
            float s32 = (float)(((double)hi - (double)lo) / qmax);
            uint16_t sb = oracle_f32_to_bf16(s32);
            double s = oracle_bf16_to_f64(sb);
            if (s == 0.0) { s = 1.0; sb = 0x3F80; }
            double z = nearbyint(-(double)lo / s);
            if (z <= 0.0) z = 0.0;          /* also turns the -0 of an all-positive group into code 0 */
            if (z > qmax) z = qmax;
            for (int64_t i = 0; i < g; ++i) {
                double c = nearbyint((double)wg[i] / s) + z;
                if (c < 0.0) c = 0.0;
                if (c > qmax) c = qmax;
                q[n * K + G * g + i] = (uint8_t)c;
            }
            s_bits[n * groups + G] = sb;
            z_bits[n * groups + G] = oracle_f64_to_bf16(z);
        }
    }
    return 0;
}

int oracle_quantize(int64_t K, int64_t N, int64_t g, const float *w,
                    uint8_t *q, uint16_t *s_bits, uint16_t *z_bits)
{
    return oracle_quantize_bits(K, N, g, 4, w, q, s_bits, z_bits);
}

/* ---- canonical packing -------------------------------------------------------------- */

/* q uint8 [N][K]  ->  qweight uint32 [N][K/8]; code 8i+j goes to bits [4j,4j+4) of word i. */
int oracle_pack(int64_t K, int64_t N, const uint8_t *q, uint32_t *qweight)
{
    if (bad_shape(K, N, 1) || !q || !qweight) return -1;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t i = 0; i < K / 8; ++i) {
            uint32_t word = 0;
            for (int j = 0; j < 8; ++j) {
                uint8_t c = q[n * K + 8 * i + j];
                if (c > 15) return -2;
                word |= (uint32_t)c << (4 * j);
            }
            qweight[n * (K / 8) + i] = word;
        }
    return 0;
}

int oracle_unpack(int64_t K, int64_t N, const uint32_t *qweight, uint8_t *q)
{
    if (bad_shape(K, N, 1) || !q || !qweight) return -1;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            q[n * K + k] = (uint8_t)((qweight[n * (K / 8) + k / 8] >> (4 * (k % 8))) & 0xFu);
    return 0;
}

/* 3-bit: q uint8 [N][K] (0..7) -> qweight uint32 [N][3K/32]; K % 32 == 0.  Code j of a run of 32
 * occupies bits [3j, 3j+3) of the 96-bit number word0 + 2^32 word1 + 2^64 word2. */
int oracle_pack3(int64_t K, int64_t N, const uint8_t *q, uint32_t *qweight)
{
    if (K <= 0 || N <= 0 || (K % 32) != 0 || !q || !qweight) return -1;
    const int64_t wpr = K / 32 * 3;      /* words per row */
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t i = 0; i < wpr; ++i) qweight[n * wpr + i] = 0;
        for (int64_t k = 0; k < K; ++k) {
            uint8_t c = q[n * K + k];
            if (c > 7) return -2;
            for (int b = 0; b < 3; ++b) {
                int64_t bit = (k / 32) * 96 + 3 * (k % 32) + b;     /* position in the row's bit stream */
                if ((c >> b) & 1) qweight[n * wpr + bit / 32] |= (uint32_t)1 << (bit % 32);
            }
        }
    }
    return 0;
}

static int code3(const uint32_t *row_words, int64_t k)
{
    int c = 0;
    for (int b = 0; b < 3; ++b) {
        int64_t bit = (k / 32) * 96 + 3 * (k % 32) + b;
        c |= (int)((row_words[bit / 32] >> (bit % 32)) & 1u) << b;
    }
    return c;
}

int oracle_unpack3(int64_t K, int64_t N, const uint32_t *qweight, uint8_t *q)
{
    if (K <= 0 || N <= 0 || (K % 32) != 0 || !q || !qweight) return -1;
    const int64_t wpr = K / 32 * 3;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) q[n * K + k] = (uint8_t)code3(qweight + n * wpr, k);
    return 0;
}

/* ---- dequantisation ----------------------------------------------------------------- */

static double weight_exact_bits(int64_t K, int64_t g, int bits, const uint32_t *qweight,
                                const uint16_t *s_bits, const uint16_t *z_bits,
                                int64_t n, int64_t k)
{
    const int64_t groups = K / g;
    int code = bits == 4 ? (int)((qweight[n * (K / 8) + k / 8] >> (4 * (k % 8))) & 0xFu)
                         : code3(qweight + n * (K / 32 * 3), k);
    double s = oracle_bf16_to_f64(s_bits[n * groups + k / g]);
    double z = oracle_bf16_to_f64(z_bits[n * groups + k / g]);
    return ((double)code - z) * s;
}

static double weight_exact(int64_t K, int64_t g, const uint32_t *qweight,
                           const uint16_t *s_bits, const uint16_t *z_bits,
                           int64_t n, int64_t k)
{
    return weight_exact_bits(K, g, 4, qweight, s_bits, z_bits, n, k);
}

static int bad_shape_bits(int64_t K, int64_t N, int64_t g, int bits)
{
    if (bits == 4) return bad_shape(K, N, g);
    return bits != 3 || K <= 0 || N <= 0 || g <= 0 || (K % 32) != 0 || (K % g) != 0;
}

/* 3- or 4-bit versions of the three functions below (same definitions, `bits` picks the packing). */
int oracle_dequantize_exact_bits(int64_t K, int64_t N, int64_t g, int bits, const uint32_t *qweight,
                                 const uint16_t *s_bits, const uint16_t *z_bits, double *w_hat)
{
    if (bad_shape_bits(K, N, g, bits) || !qweight || !s_bits || !z_bits || !w_hat) return -1;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            w_hat[n * K + k] = weight_exact_bits(K, g, bits, qweight, s_bits, z_bits, n, k);
    return 0;
}

int oracle_dequantize_bits(int64_t K, int64_t N, int64_t g, int bits, const uint32_t *qweight,
                           const uint16_t *s_bits, const uint16_t *z_bits, uint16_t *w_bf16)
{
    if (bad_shape_bits(K, N, g, bits) || !qweight || !s_bits || !z_bits || !w_bf16) return -1;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            w_bf16[n * K + k] =
                oracle_f64_to_bf16(weight_exact_bits(K, g, bits, qweight, s_bits, z_bits, n, k));
    return 0;
}

int oracle_forward_bits(int64_t K, int64_t N, int64_t g, int bits, int64_t M, const uint32_t *qweight,
                        const uint16_t *s_bits, const uint16_t *z_bits, const uint16_t *x_bits,
                        double *y, int threads)
{
    if (bad_shape_bits(K, N, g, bits) || M < 0 || !qweight || !s_bits || !z_bits || (M && (!x_bits || !y)))
        return -1;
    int used = 1;
#ifdef _OPENMP
    if (threads > 1) used = threads;
#pragma omp parallel for num_threads(used) schedule(static)
#endif
    for (int64_t n = 0; n < N; ++n)
        for (int64_t m = 0; m < M; ++m) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += oracle_bf16_to_f64(x_bits[m * K + k]) *
                       weight_exact_bits(K, g, bits, qweight, s_bits, z_bits, n, k);
            y[m * N + n] = acc;
        }
    return used;
}

/* w^ as fp64 [N][K] (the mathematical weight; exact). */
int oracle_dequantize_exact(int64_t K, int64_t N, int64_t g, const uint32_t *qweight,
                            const uint16_t *s_bits, const uint16_t *z_bits, double *w_hat)
{
    if (bad_shape(K, N, g) || !qweight || !s_bits || !z_bits || !w_hat) return -1;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            w_hat[n * K + k] = weight_exact(K, g, qweight, s_bits, z_bits, n, k);
    return 0;
}

/* RNE_bf16(w^) as bf16 bits [N][K]: the result of the library's dequantize call. */
int oracle_dequantize(int64_t K, int64_t N, int64_t g, const uint32_t *qweight,
                      const uint16_t *s_bits, const uint16_t *z_bits, uint16_t *w_bf16)
{
    if (bad_shape(K, N, g) || !qweight || !s_bits || !z_bits || !w_bf16) return -1;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            w_bf16[n * K + k] =
                oracle_f64_to_bf16(weight_exact(K, g, qweight, s_bits, z_bits, n, k));
    return 0;
}

/* ---- forward ------------------------------------------------------------------------ */

/*
 * y[m][n] = sum_{k<K} x[m][k] * w^[n][k], fp64, k ascending.
 * rounded_weights = 0: w^ exact (the reference).  = 1: RNE_bf16(w^) widened back to fp64
 * (a diagnostic that separates weight-rounding error from accumulation error).
 * threads <= 1 runs serially; otherwise rows n are shared among that many OpenMP threads
 * (each y element is still one serial sum, so results do not depend on the thread count).
 * Returns the thread count used (>= 1) or a negative error.
 */
int oracle_forward(int64_t K, int64_t N, int64_t g, int64_t M, const uint32_t *qweight,
                   const uint16_t *s_bits, const uint16_t *z_bits, const uint16_t *x_bits,
                   double *y, int rounded_weights, int threads)
{
    if (bad_shape(K, N, g) || M < 0 || !qweight || !s_bits || !z_bits || (M && (!x_bits || !y)))
        return -1;
    int used = 1;
#ifdef _OPENMP
    if (threads > 1) used = threads;
#endif
    int failed = 0;
#ifdef _OPENMP
#pragma omp parallel for num_threads(used) schedule(static)
#endif
    for (int64_t n = 0; n < N; ++n) {
        double *row = (double *)malloc((size_t)K * sizeof(double));
        if (!row) { failed = 1; continue; }
        for (int64_t k = 0; k < K; ++k) {
            double v = weight_exact(K, g, qweight, s_bits, z_bits, n, k);
            row[k] = rounded_weights ? oracle_bf16_to_f64(oracle_f64_to_bf16(v)) : v;
        }
        for (int64_t m = 0; m < M; ++m) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) acc += oracle_bf16_to_f64(x_bits[m * K + k]) * row[k];
            y[m * N + n] = acc;
        }
        free(row);
    }
    return failed ? -3 : used;
}

/* Same sum for chosen (m, n) pairs only: out[i] = y[ms[i]][ns[i]].  For outputs too many to
 * compute in full (prefill sizes). */
int oracle_forward_sampled(int64_t K, int64_t N, int64_t g, int64_t M, const uint32_t *qweight,
                           const uint16_t *s_bits, const uint16_t *z_bits,
                           const uint16_t *x_bits, int64_t count, const int64_t *ms,
                           const int64_t *ns, double *out)
{
    if (bad_shape(K, N, g) || M <= 0 || count < 0 || !qweight || !s_bits || !z_bits || !x_bits ||
        (count && (!ms || !ns || !out)))
        return -1;
    for (int64_t i = 0; i < count; ++i) {
        int64_t m = ms[i], n = ns[i];
        if (m < 0 || m >= M || n < 0 || n >= N) return -2;
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k)
            acc += oracle_bf16_to_f64(x_bits[m * K + k]) *
                   weight_exact(K, g, qweight, s_bits, z_bits, n, k);
        out[i] = acc;
    }
    return 0;
}

/* bf16 twin: y[m][n] = sum_k x[m][k] * W[n][k], W bf16 [N][K], fp64, k ascending. */
int oracle_bf16_forward(int64_t K, int64_t N, int64_t M, const uint16_t *w_bits,
                        const uint16_t *x_bits, double *y, int threads)
{
    if (K <= 0 || N <= 0 || M < 0 || !w_bits || (M && (!x_bits || !y))) return -1;
    int used = 1;
#ifdef _OPENMP
    if (threads > 1) used = threads;
#pragma omp parallel for num_threads(used) schedule(static)
#endif
    for (int64_t n = 0; n < N; ++n)
        for (int64_t m = 0; m < M; ++m) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += oracle_bf16_to_f64(x_bits[m * K + k]) * oracle_bf16_to_f64(w_bits[n * K + k]);
            y[m * N + n] = acc;
        }
    return used;
}

int oracle_bf16_forward_sampled(int64_t K, int64_t N, int64_t M, const uint16_t *w_bits,
                                const uint16_t *x_bits, int64_t count, const int64_t *ms,
                                const int64_t *ns, double *out)
{
    if (K <= 0 || N <= 0 || M <= 0 || count < 0 || !w_bits || !x_bits ||
        (count && (!ms || !ns || !out)))
        return -1;
    for (int64_t i = 0; i < count; ++i) {
        int64_t m = ms[i], n = ns[i];
        if (m < 0 || m >= M || n < 0 || n >= N) return -2;
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k)
            acc += oracle_bf16_to_f64(x_bits[m * K + k]) * oracle_bf16_to_f64(w_bits[n * K + k]);
        out[i] = acc;
    }
    return 0;
}

/* ---- decoder glue (see the header) ----------------------------------------------------- */

int oracle_rmsnorm(int64_t M, int64_t K, const uint16_t *x_bits, const uint16_t *gamma_bits, double eps,
                   uint16_t *out_bits)
{
    if (M < 0 || K <= 0 || !x_bits || !gamma_bits || !out_bits || !(eps >= 0.0)) return -1;
    for (int64_t m = 0; m < M; ++m) {
        double ss = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double v = oracle_bf16_to_f64(x_bits[m * K + k]);
            ss += v * v;
        }
        const double denom = sqrt(ss / (double)K + eps);
        for (int64_t k = 0; k < K; ++k) {
            const double v = oracle_bf16_to_f64(x_bits[m * K + k]);
            const double gma = oracle_bf16_to_f64(gamma_bits[k]);
            /* an all-zero row with eps = 0 is 0 / 0: defined as 0 */
            out_bits[m * K + k] = oracle_f64_to_bf16(denom > 0.0 ? v * gma / denom : 0.0);
        }
    }
    return 0;
}

int oracle_swiglu(int64_t M, int64_t I, const uint16_t *in_bits, uint16_t *out_bits)
{
    if (M < 0 || I <= 0 || !in_bits || !out_bits) return -1;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t i = 0; i < I; ++i) {
            const double a = oracle_bf16_to_f64(in_bits[m * 2 * I + i]);
            const double b = oracle_bf16_to_f64(in_bits[m * 2 * I + I + i]);
            out_bits[m * I + i] = oracle_f64_to_bf16(a / (1.0 + exp(-a)) * b);
        }
    return 0;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
