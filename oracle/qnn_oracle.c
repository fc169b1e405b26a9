/*
 * qnn_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, scalar CPU statement of what the quantized-inference hot path
 * computes, written from the whitepaper "Quantizing deep convolutional networks
 * for efficient inference" (arXiv 1806.08342).  It exists to check the GPU
 * library and to be timed as a CPU baseline; nothing in the product may call it.
 * It shares no code, header, table or helper with the HIP implementation.
 *
 * Conventions
 *   activations : uint8, NHWC, one (scale Delta_x, zero-point z_x) per tensor   (Sec. 2.1, Sec. 2.6)
 *   weights     : int8 (or two signed 4-bit values per byte), one kernel per output
 *                 channel stored contiguously ([C_out][kh][kw][C_in]); per-channel
 *                 scale Delta_c and optional per-channel zero-point z_w        (Sec. 2.2, Sec. 2.6)
 *   accumulator : int64 here (the product uses int32; overflow of the int32 range
 *                 is reported as an error by the oracle, never wrapped)
 *   output      : uint8 after the two-stage fixed-point rescale defined below.
 *
 * The paper defines the quantizer (eq. 1-3) and the integer convolution with
 * its zero-point expansion (eq. 4-6).  It does not define how the accumulator
 * is scaled back to 8 bits; that step follows the build's stated reading:
 * a saturating rounding-doubling high multiply by an int32 multiplier followed
 * by a rounding right shift (ties: first stage toward +infinity, second stage
 * away from zero).
 *
 * Parity status: every function below is pinned by tests that do not re-use
 * this code (closed forms, exact rational arithmetic, fp64 brute force, the
 * paper's worked example), except oracle_qadd whose structure cannot be
 * pinned to the paper (the rescale-add figure of Sec. 3.2.1 is missing from
 * the text): it is pinned to real arithmetic within 1 LSB and to the identity
 * case only -- "parity unpinned" with respect to the paper.
 *
 * Loops are parallelised with OpenMP over independent outputs only; there is
 * no blocking, fusion or re-ordering of the arithmetic.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_EINVAL 1
#define ORACLE_EOVERFLOW 4 /* |acc + bias| left the int32 range */

/* ------------------------------------------------------------------ helpers */

static int64_t clamp_i64(int64_t lo, int64_t hi, int64_t x)
{
    /* three-case clamp of Sec. 2.1 (below eq. 2) */
    if (x <= lo) return lo;
    if (x >= hi) return hi;
    return x;
}

/* round to nearest integer, ties away from zero (double argument) */
static double round_half_away(double v)
{
    return (v < 0.0) ? -floor(-v + 0.5) : floor(v + 0.5);
}

static int64_t floor_div_i64(int64_t p, int64_t d) /* d > 0 */
{
    int64_t q = p / d;
    if ((p % d) != 0 && p < 0) q -= 1;
    return q;
}

/* ------------------------------------------ quantizer parameters (Sec. 2.1) */

/* Range (xmin, xmax) is first relaxed to contain 0 (Sec. 2.1, second paragraph),
 * then Delta = (xmax - xmin) / (2^bits - 1) and z = round(-xmin / Delta),
 * clamped to the integer grid so that real 0 maps to z with no error. */
int oracle_choose_qparams(double xmin, double xmax, int bits, float *scale, int32_t *zero_point)
{
    if (!scale || !zero_point || bits < 2 || bits > 16 || !(xmin <= xmax)) return ORACLE_EINVAL;
    if (xmin > 0.0) xmin = 0.0;
    if (xmax < 0.0) xmax = 0.0;
    const int64_t top = ((int64_t)1 << bits) - 1;
    if (xmax == xmin) {
        *scale = 1.0f;
        *zero_point = 0;
        return ORACLE_OK;
    }
    const float delta = (float)((xmax - xmin) / (double)top);
    const double z = round_half_away(-xmin / (double)delta);
    *scale = delta;
    *zero_point = (int32_t)clamp_i64(0, top, (int64_t)z);
    return ORACLE_OK;
}

/* ReLU / ReLU6 expressed as a clamp range in the quantized output domain
 * (Sec. 3.2.1 last paragraph: the activation is fused into the producing op).
 * kind 0: none -> [0,255]; 1: ReLU -> [z,255]; 2: ReLU6 -> [z, min(255, z + round(6/s))] */
int oracle_act_range(int kind, float s_out, int32_t z_out, int32_t *lo, int32_t *hi)
{
    if (!lo || !hi || kind < 0 || kind > 2 || !(s_out > 0.0f) || z_out < 0 || z_out > 255) return ORACLE_EINVAL;
    *lo = 0;
    *hi = 255;
    if (kind >= 1) *lo = z_out;
    if (kind == 2) {
        const double six = round_half_away(6.0 / (double)s_out);
        int64_t h = (int64_t)z_out + (six > 1e9 ? (int64_t)1000000000 : (int64_t)six);
        *hi = (int32_t)clamp_i64(*lo, 255, h);
    }
    return ORACLE_OK;
}

/* --------------------------------- quantize / de-quantize (Sec. 2.1, eq. 1-3) */

/* eq. 1-2 with the clamp range [qmin, qmax] (0..255 for 8 bits):
 *   t = x / Delta in IEEE binary32, r = round(t) ties away from zero,
 *   q = clamp(qmin, qmax, r + z).  NaN quantizes like 0.0 (to z). */
int oracle_quantize(const float *x, uint8_t *q, size_t n, float scale, int32_t zero_point, int32_t qmin, int32_t qmax)
{
    if ((n && (!x || !q)) || !(scale > 0.0f) || isinf(scale)) return ORACLE_EINVAL;
    if (qmin < 0 || qmax > 255 || qmin > qmax || zero_point < qmin || zero_point > qmax) return ORACLE_EINVAL;
    const float lo = (float)(qmin - zero_point);
    const float hi = (float)(qmax - zero_point);
#pragma omp parallel for schedule(static)
    for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i) {
        volatile float t = x[i] / scale; /* volatile: force a binary32 result */
        float r;
        if (t != t) {
            r = 0.0f;
        } else {
            r = roundf(t);
        }
        if (r < lo) r = lo;
        if (r > hi) r = hi;
        q[i] = (uint8_t)((int32_t)r + zero_point);
    }
    return ORACLE_OK;
}

/* eq. 3: x = (q - z) * Delta, one binary32 multiply */
int oracle_dequantize(const uint8_t *q, float *x, size_t n, float scale, int32_t zero_point)
{
    if ((n && (!x || !q)) || !(scale > 0.0f) || isinf(scale)) return ORACLE_EINVAL;
    if (zero_point < 0 || zero_point > 255) return ORACLE_EINVAL;
#pragma omp parallel for schedule(static)
    for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i) {
        volatile float d = (float)((int32_t)q[i] - zero_point);
        volatile float v = d * scale;
        x[i] = v;
    }
    return ORACLE_OK;
}

/* The same two maps for code ranges wider than a byte (up to 16 bits: the lower- and higher-precision
 * activation experiments of Sec. 3.3 use 4-bit and 16-bit codes).  Same arithmetic, codes in uint16. */
int oracle_quantize_wide(const float *x, uint16_t *q, size_t n, float scale, int32_t zero_point, int32_t qmin,
                         int32_t qmax)
{
    if ((n && (!x || !q)) || !(scale > 0.0f) || isinf(scale)) return ORACLE_EINVAL;
    if (qmin < 0 || qmax > 65535 || qmin > qmax || zero_point < qmin || zero_point > qmax) return ORACLE_EINVAL;
    const float lo = (float)(qmin - zero_point);
    const float hi = (float)(qmax - zero_point);
#pragma omp parallel for schedule(static)
    for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i) {
        volatile float t = x[i] / scale;
        float r = (t != t) ? 0.0f : roundf(t);
        if (r < lo) r = lo;
        if (r > hi) r = hi;
        q[i] = (uint16_t)((int32_t)r + zero_point);
    }
    return ORACLE_OK;
}

int oracle_dequantize_wide(const uint16_t *q, float *x, size_t n, float scale, int32_t zero_point)
{
    if ((n && (!x || !q)) || !(scale > 0.0f) || isinf(scale)) return ORACLE_EINVAL;
    if (zero_point < 0 || zero_point > 65535) return ORACLE_EINVAL;
#pragma omp parallel for schedule(static)
    for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i) {
        volatile float d = (float)((int32_t)q[i] - zero_point);
        volatile float v = d * scale;
        x[i] = v;
    }
    return ORACLE_OK;
}

/* ------------------------- symmetric per-channel weight quantizer (Sec. 2.2) */

/* w is [channels][per_channel] fp32.  Delta_c = max|w_c| / (2^(bits-1) - 1)
 * (restricted range, eq. 10), w_Q = clamp(round(w / Delta_c)) with the clamp
 * range of eq. 8 (full, [-2^(bits-1), 2^(bits-1)-1]) or eq. 10 (restricted).
 * Rounding ties away from zero, division in double. */
int oracle_quantize_weights(const float *w, size_t channels, size_t per_channel, int bits, int restricted,
                            int8_t *wq, float *delta)
{
    if (!w || !wq || !delta || (bits != 8 && bits != 4)) return ORACLE_EINVAL;
    const int64_t top = ((int64_t)1 << (bits - 1)) - 1;
    const int64_t lo = restricted ? -top : -top - 1;
    for (size_t c = 0; c < channels; ++c) {
        double amax = 0.0;
        for (size_t i = 0; i < per_channel; ++i) {
            double a = fabs((double)w[c * per_channel + i]);
            if (a > amax) amax = a;
        }
        float d = (amax == 0.0) ? 1.0f : (float)(amax / (double)top);
        delta[c] = d;
        for (size_t i = 0; i < per_channel; ++i) {
            double r = round_half_away((double)w[c * per_channel + i] / (double)d);
            wq[c * per_channel + i] = (int8_t)clamp_i64(lo, top, (int64_t)r);
        }
    }
    return ORACLE_OK;
}

/* ------------------------------------------------ 4-bit weight storage */

/* Two's-complement nibbles, element 2j in the low nibble of byte j, element
 * 2j+1 in the high nibble (Sec. 3.3 uses 4-bit per-channel weights; the
 * storage order is this build's choice). */
int oracle_pack_int4(const int8_t *v, size_t n, uint8_t *packed)
{
    if (!v || !packed || (n & 1)) return ORACLE_EINVAL;
    for (size_t i = 0; i < n; ++i)
        if (v[i] < -8 || v[i] > 7) return ORACLE_EINVAL;
    for (size_t j = 0; j < n / 2; ++j) {
        unsigned lo = (unsigned)(v[2 * j] & 0xF);
        unsigned hi = (unsigned)(v[2 * j + 1] & 0xF);
        packed[j] = (uint8_t)(lo | (hi << 4));
    }
    return ORACLE_OK;
}

static int32_t nibble_value(unsigned nib) /* nib in 0..15 -> -8..7 */
{
    return (int32_t)((nib ^ 8u)) - 8;
}

int oracle_unpack_int4(const uint8_t *packed, size_t n, int8_t *v)
{
    if (!v || !packed || (n & 1)) return ORACLE_EINVAL;
    for (size_t j = 0; j < n / 2; ++j) {
        v[2 * j] = (int8_t)nibble_value(packed[j] & 0xFu);
        v[2 * j + 1] = (int8_t)nibble_value((packed[j] >> 4) & 0xFu);
    }
    return ORACLE_OK;
}

/* weight element `idx` of a tensor stored with `bits` bits per element */
static int32_t weight_at(const void *w, int bits, size_t idx)
{
    if (bits == 8) return (int32_t)((const int8_t *)w)[idx];
    const uint8_t b = ((const uint8_t *)w)[idx >> 1];
    return nibble_value((idx & 1) ? ((b >> 4) & 0xFu) : (b & 0xFu));
}

/* ------------------------------------- fixed-point rescale (build's reading) */

/* real multiplier M > 0  ->  (mult, shift) with M ~= mult * 2^(-31 - shift),
 * mult in [2^30, 2^31).  shift > 0 is a right shift, shift < 0 a left shift. */
int oracle_quantize_multiplier(double real_mult, int32_t *mult, int32_t *shift)
{
    if (!mult || !shift || !(real_mult >= 0.0) || isinf(real_mult)) return ORACLE_EINVAL;
    if (real_mult == 0.0) {
        *mult = 0;
        *shift = 0;
        return ORACLE_OK;
    }
    int e = 0;
    const double m = frexp(real_mult, &e); /* m in [0.5, 1) */
    int64_t q = (int64_t)llround(m * 2147483648.0);
    if (q == ((int64_t)1 << 31)) {
        q >>= 1;
        e += 1;
    }
    int s = -e;
    if (s > 31) { /* M < 2^-32: every int32 input rescales to 0 */
        *mult = 0;
        *shift = 0;
        return ORACLE_OK;
    }
    if (s < -31) return ORACLE_EINVAL;
    *mult = (int32_t)q;
    *shift = (int32_t)s;
    return ORACLE_OK;
}

static int32_t sat32(int64_t v)
{
    if (v > INT32_MAX) return INT32_MAX;
    if (v < INT32_MIN) return INT32_MIN;
    return (int32_t)v;
}

/* saturating rounding doubling high multiply: nearest integer to a*b/2^31,
 * ties toward +infinity; the single overflow case saturates. */
static int32_t srdhm(int32_t a, int32_t b)
{
    if (a == INT32_MIN && b == INT32_MIN) return INT32_MAX;
    const int64_t p = (int64_t)a * (int64_t)b + ((int64_t)1 << 30);
    return (int32_t)floor_div_i64(p, (int64_t)1 << 31);
}

/* divide by 2^n, nearest, ties away from zero */
static int32_t rshift_round(int32_t h, int n)
{
    if (n == 0) return h;
    const int64_t a = (h < 0) ? -(int64_t)h : (int64_t)h;
    const int64_t q = floor_div_i64(a + ((int64_t)1 << (n - 1)), (int64_t)1 << n);
    return (int32_t)((h < 0) ? -q : q);
}

/* the rescale primitive: a -> nearest(a * mult * 2^(-31-shift)) in two stages */
int32_t oracle_rescale(int32_t a, int32_t mult, int32_t shift)
{
    if (shift < 0) a = sat32((int64_t)a * ((int64_t)1 << (-shift)));
    const int32_t h = srdhm(a, mult);
    return rshift_round(h, shift > 0 ? shift : 0);
}

static uint8_t finish_u8(int64_t acc, int32_t mult, int32_t shift, int32_t z_out, int32_t act_min, int32_t act_max)
{
    const int64_t r = (int64_t)oracle_rescale((int32_t)acc, mult, shift) + (int64_t)z_out;
    return (uint8_t)clamp_i64(act_min, act_max, r);
}

static int bad_out_range(int32_t z_out, int32_t act_min, int32_t act_max)
{
    return act_min < 0 || act_max > 255 || act_min > act_max || z_out < 0 || z_out > 255;
}

/* stand-alone requantize of an int32 tensor [rows][channels] */
int oracle_requantize(const int32_t *acc, uint8_t *y, size_t rows, size_t channels, const int32_t *mult,
                      const int32_t *shift, int per_channel, int32_t z_out, int32_t act_min, int32_t act_max)
{
    if (!acc || !y || !mult || !shift || bad_out_range(z_out, act_min, act_max)) return ORACLE_EINVAL;
    for (size_t c = 0; c < (per_channel ? channels : 1); ++c)
        if (shift[c] < -31 || shift[c] > 31) return ORACLE_EINVAL;
#pragma omp parallel for schedule(static)
    for (ptrdiff_t r = 0; r < (ptrdiff_t)rows; ++r)
        for (size_t c = 0; c < channels; ++c) {
            const size_t p = per_channel ? c : 0;
            y[(size_t)r * channels + c] = finish_u8(acc[(size_t)r * channels + c], mult[p], shift[p], z_out, act_min, act_max);
        }
    return ORACLE_OK;
}

/* ------------------------------------------------ integer GEMM (eq. 4) */

/* C[m][n] = clamp(z_out + rescale(bias[n] + sum_k (A[m][k]-z_a)(B[k][n]-z_w[n])))
 * A is [M][K] row-major uint8 (lda).  B holds the K weights of output column n
 * contiguously: element (k, n) at B[n*ldb + k] (ldb counted in elements).
 * z_w may be NULL (symmetric weights).  bias may be NULL. */
int oracle_qgemm(const uint8_t *A, int64_t lda, int32_t z_a, const void *B, int64_t ldb, int weight_bits,
                 const int32_t *z_w, int64_t M, int64_t N, int64_t K, const int32_t *bias, const int32_t *mult,
                 const int32_t *shift, int32_t z_out, int32_t act_min, int32_t act_max, uint8_t *C, int64_t ldc)
{
    if (!A || !B || !mult || !shift || !C || M <= 0 || N <= 0 || K <= 0 || lda < K || ldb < K || ldc < N)
        return ORACLE_EINVAL;
    if ((weight_bits != 8 && weight_bits != 4) || (weight_bits == 4 && ((K | ldb) & 1))) return ORACLE_EINVAL;
    if (z_a < 0 || z_a > 255 || bad_out_range(z_out, act_min, act_max)) return ORACLE_EINVAL;
    int overflow = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            const int64_t zw = z_w ? z_w[n] : 0;
            int64_t acc = 0;
            for (int64_t k = 0; k < K; ++k) {
                const int64_t xa = (int64_t)A[m * lda + k] - z_a;
                const int64_t wb = (int64_t)weight_at(B, weight_bits, (size_t)(n * ldb + k)) - zw;
                acc += xa * wb;
            }
            if (bias) acc += bias[n];
            if (acc > INT32_MAX || acc < INT32_MIN) overflow = 1;
            C[m * ldc + n] = finish_u8(acc, mult[n], shift[n], z_out, act_min, act_max);
        }
    return overflow ? ORACLE_EOVERFLOW : ORACLE_OK;
}

/* ------------------------------------------------ integer conv (eq. 4) */

typedef struct {
    int N, H, W, Cin;           /* input NHWC */
    int Cout, kh, kw;           /* weights [Cout][kh][kw][Cin] */
    int stride_h, stride_w, pad_h, pad_w;
    int Ho, Wo;
} conv_geom;

static int conv_geometry(conv_geom *g)
{
    if (g->N <= 0 || g->H <= 0 || g->W <= 0 || g->Cin <= 0 || g->Cout <= 0 || g->kh <= 0 || g->kw <= 0) return 1;
    if (g->stride_h <= 0 || g->stride_w <= 0 || g->pad_h < 0 || g->pad_w < 0) return 1;
    const int eh = g->H + 2 * g->pad_h - g->kh, ew = g->W + 2 * g->pad_w - g->kw;
    if (eh < 0 || ew < 0) return 1;
    g->Ho = eh / g->stride_h + 1;
    g->Wo = ew / g->stride_w + 1;
    return 0;
}

/* accumulator of one output element; a tap that falls outside the image
 * contributes 0, i.e. the border is padded with z_x, the code of real 0 (Sec. 2.1) */
static int64_t conv_acc(const conv_geom *g, const uint8_t *x, int32_t z_x, const void *w, int bits, int64_t z_w, int n,
                        int ho, int wo, int co)
{
    int64_t acc = 0;
    for (int a = 0; a < g->kh; ++a)
        for (int b = 0; b < g->kw; ++b) {
            const int hi = ho * g->stride_h - g->pad_h + a;
            const int wi = wo * g->stride_w - g->pad_w + b;
            if (hi < 0 || hi >= g->H || wi < 0 || wi >= g->W) continue;
            const size_t xoff = (((size_t)n * g->H + hi) * g->W + wi) * g->Cin;
            const size_t woff = (((size_t)co * g->kh + a) * g->kw + b) * g->Cin;
            for (int ci = 0; ci < g->Cin; ++ci)
                acc += ((int64_t)x[xoff + ci] - z_x) * ((int64_t)weight_at(w, bits, woff + ci) - z_w);
        }
    return acc;
}

/* Full convolution, or (when `sample` != NULL) only the `n_sample` outputs whose
 * flat NHWC indices are listed; then y[i] receives output sample[i]. */
int oracle_qconv2d(const uint8_t *x, int N, int H, int W, int Cin, int32_t z_x, const void *w, int Cout, int kh, int kw,
                   int weight_bits, const int32_t *z_w, int stride_h, int stride_w, int pad_h, int pad_w,
                   const int32_t *bias, const int32_t *mult, const int32_t *shift, int32_t z_out, int32_t act_min,
                   int32_t act_max, uint8_t *y, const int64_t *sample, int64_t n_sample)
{
    conv_geom g = {N, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w, 0, 0};
    if (!x || !w || !mult || !shift || !y || conv_geometry(&g)) return ORACLE_EINVAL;
    if ((weight_bits != 8 && weight_bits != 4) || (weight_bits == 4 && (Cin & 1))) return ORACLE_EINVAL;
    if (z_x < 0 || z_x > 255 || bad_out_range(z_out, act_min, act_max)) return ORACLE_EINVAL;
    const int64_t total = (int64_t)N * g.Ho * g.Wo * Cout;
    const int64_t count = sample ? n_sample : total;
    int overflow = 0, bad = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow, bad)
    for (int64_t i = 0; i < count; ++i) {
        const int64_t flat = sample ? sample[i] : i;
        if (flat < 0 || flat >= total) {
            bad = 1;
            continue;
        }
        const int co = (int)(flat % Cout);
        const int64_t pix = flat / Cout;
        const int wo = (int)(pix % g.Wo);
        const int ho = (int)((pix / g.Wo) % g.Ho);
        const int n = (int)(pix / ((int64_t)g.Wo * g.Ho));
        int64_t acc = conv_acc(&g, x, z_x, w, weight_bits, z_w ? z_w[co] : 0, n, ho, wo, co);
        if (bias) acc += bias[co];
        if (acc > INT32_MAX || acc < INT32_MIN) overflow = 1;
        y[i] = finish_u8(acc, mult[co], shift[co], z_out, act_min, act_max);
    }
    if (bad) return ORACLE_EINVAL;
    return overflow ? ORACLE_EOVERFLOW : ORACLE_OK;
}

/* raw int64 accumulators (before bias and rescale) of the same convolution,
 * exposed so tests can pin the integer arithmetic separately from the rescale */
int oracle_qconv2d_acc(const uint8_t *x, int N, int H, int W, int Cin, int32_t z_x, const void *w, int Cout, int kh,
                       int kw, int weight_bits, const int32_t *z_w, int stride_h, int stride_w, int pad_h, int pad_w,
                       int64_t *acc_out)
{
    conv_geom g = {N, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w, 0, 0};
    if (!x || !w || !acc_out || conv_geometry(&g)) return ORACLE_EINVAL;
    if ((weight_bits != 8 && weight_bits != 4) || (weight_bits == 4 && (Cin & 1))) return ORACLE_EINVAL;
    for (int n = 0; n < N; ++n)
        for (int ho = 0; ho < g.Ho; ++ho)
            for (int wo = 0; wo < g.Wo; ++wo)
                for (int co = 0; co < Cout; ++co)
                    acc_out[((((size_t)n * g.Ho + ho) * g.Wo + wo) * Cout) + co] =
                        conv_acc(&g, x, z_x, w, weight_bits, z_w ? z_w[co] : 0, n, ho, wo, co);
    return ORACLE_OK;
}

/* depthwise: one kh x kw kernel per channel, weights [kh][kw][C] int8
 * (separable convolutions of the MobileNet family, Sec. 3 / Appendix A) */
int oracle_qdwconv2d(const uint8_t *x, int N, int H, int W, int C, int32_t z_x, const int8_t *w, int kh, int kw,
                     const int32_t *z_w, int stride_h, int stride_w, int pad_h, int pad_w, const int32_t *bias,
                     const int32_t *mult, const int32_t *shift, int32_t z_out, int32_t act_min, int32_t act_max,
                     uint8_t *y, const int64_t *sample, int64_t n_sample)
{
    conv_geom g = {N, H, W, C, C, kh, kw, stride_h, stride_w, pad_h, pad_w, 0, 0};
    if (!x || !w || !mult || !shift || !y || conv_geometry(&g)) return ORACLE_EINVAL;
    if (z_x < 0 || z_x > 255 || bad_out_range(z_out, act_min, act_max)) return ORACLE_EINVAL;
    const int64_t total = (int64_t)N * g.Ho * g.Wo * C;
    const int64_t count = sample ? n_sample : total;
    int overflow = 0, bad = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow, bad)
    for (int64_t i = 0; i < count; ++i) {
        const int64_t flat = sample ? sample[i] : i;
        if (flat < 0 || flat >= total) {
            bad = 1;
            continue;
        }
        const int c = (int)(flat % C);
        const int64_t pix = flat / C;
        const int wo = (int)(pix % g.Wo);
        const int ho = (int)((pix / g.Wo) % g.Ho);
        const int n = (int)(pix / ((int64_t)g.Wo * g.Ho));
        const int64_t zw = z_w ? z_w[c] : 0;
        int64_t acc = 0;
        for (int a = 0; a < kh; ++a)
            for (int b = 0; b < kw; ++b) {
                const int hi = ho * stride_h - pad_h + a;
                const int wi = wo * stride_w - pad_w + b;
                if (hi < 0 || hi >= H || wi < 0 || wi >= W) continue;
                const int64_t xv = (int64_t)x[(((size_t)n * H + hi) * W + wi) * C + c] - z_x;
                const int64_t wv = (int64_t)w[((size_t)a * kw + b) * C + c] - zw;
                acc += xv * wv;
            }
        if (bias) acc += bias[c];
        if (acc > INT32_MAX || acc < INT32_MIN) overflow = 1;
        y[i] = finish_u8(acc, mult[c], shift[c], z_out, act_min, act_max);
    }
    if (bad) return ORACLE_EINVAL;
    return overflow ? ORACLE_EOVERFLOW : ORACLE_OK;
}

/* ------------------------------------ element-wise add with rescale (Sec. 3.2.1) */

/* Both inputs are brought to a common scale before the addition and the sum is
 * rescaled to the output quantizer.  With L = left_shift head-room bits:
 *   ta = (a - z_a) * 2^L,  tb = (b - z_b) * 2^L
 *   u  = rescale(ta; mult_a, shift_a) + rescale(tb; mult_b, shift_b)
 *   y  = clamp(act_min, act_max, z_out + rescale(u; mult_o, shift_o))
 * The host chooses mult_a ~ s_a/(2 s_max), mult_b ~ s_b/(2 s_max),
 * mult_o ~ 2 s_max / (2^L s_out). */
int oracle_qadd(const uint8_t *a, int32_t z_a, int32_t mult_a, int32_t shift_a, const uint8_t *b, int32_t z_b,
                int32_t mult_b, int32_t shift_b, int32_t left_shift, int32_t mult_o, int32_t shift_o, int32_t z_out,
                int32_t act_min, int32_t act_max, uint8_t *y, size_t n)
{
    if ((n && (!a || !b || !y)) || left_shift < 0 || left_shift > 22) return ORACLE_EINVAL;
    if (z_a < 0 || z_a > 255 || z_b < 0 || z_b > 255 || bad_out_range(z_out, act_min, act_max)) return ORACLE_EINVAL;
    if (shift_a < -31 || shift_a > 31 || shift_b < -31 || shift_b > 31 || shift_o < -31 || shift_o > 31)
        return ORACLE_EINVAL;
#pragma omp parallel for schedule(static)
    for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i) {
        const int32_t ta = ((int32_t)a[i] - z_a) * (1 << left_shift);
        const int32_t tb = ((int32_t)b[i] - z_b) * (1 << left_shift);
        const int64_t u = (int64_t)oracle_rescale(ta, mult_a, shift_a) + (int64_t)oracle_rescale(tb, mult_b, shift_b);
        const int64_t r = (int64_t)oracle_rescale(sat32(u), mult_o, shift_o) + z_out;
        y[i] = (uint8_t)clamp_i64(act_min, act_max, r);
    }
    return ORACLE_OK;
}

/* parameters of oracle_qadd from the three real scales (L = 20) */
int oracle_qadd_params(double s_a, double s_b, double s_out, int32_t *left_shift, int32_t *mult_a, int32_t *shift_a,
                       int32_t *mult_b, int32_t *shift_b, int32_t *mult_o, int32_t *shift_o)
{
    if (!(s_a > 0.0) || !(s_b > 0.0) || !(s_out > 0.0)) return ORACLE_EINVAL;
    const int L = 20;
    const double twice_max = 2.0 * (s_a > s_b ? s_a : s_b);
    *left_shift = L;
    int rc = oracle_quantize_multiplier(s_a / twice_max, mult_a, shift_a);
    rc |= oracle_quantize_multiplier(s_b / twice_max, mult_b, shift_b);
    rc |= oracle_quantize_multiplier(twice_max / ((double)(1 << L) * s_out), mult_o, shift_o);
    return rc;
}
