/*
 * CPU oracle, second part: F x F binary convolution written as F*F parallel
 * shifted binary 1x1 convolutions, each with its own real scale.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE (see bcnn_oracle.c): only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it, and
 * it shares nothing with the library.
 *
 * What it follows (paper, Section 4.2.1): a binary convolution module adds a
 * learnable bias, takes the sign, applies a binary 1x1 convolution and then
 * batch norm (first paragraph); a module may hold P parallel branches, each with its own bias,
 * binary weights and batch-norm parameters, whose results are summed (Figure 2,
 * bottom), and the last paragraph builds an F x F binary convolution from
 * P = F*F such branches: branch (u,v) sees the real feature map shifted by
 * (u,v) and zero padded BEFORE its bias is added, so that
 *
 *   a_t[n][c][oh][ow] = a[n][c][oh*s-p+u][ow*s-p+v]   inside the image, else 0
 *   x_t               = sign(a_t + b_t[c])             (+1 for >= 0)
 *   y_t[n][oh][ow][o] = sum_c x_t[n][c][oh][ow] * w[o][c][u][v]
 *   z[n][oh][ow][o]   = sum_t ( g_t[o] * y_t + h_t[o] )
 *
 * with t = u*F + v, g/h the per-branch batch-norm scale and bias.  The module
 * of Figure 2 (bottom) itself, P parallel binary 1x1 branches on the unshifted
 * feature map, is the same sum with F = 1 and t = 0 .. P-1 (every branch reads
 * position (oh*s, ow*s); nothing is ever outside the image).  A padded
 * position therefore is the constant sign(b_t[c]) per branch and channel, not
 * a zero operand.  Readings where the paper is silent: the stride is applied
 * by evaluating every branch at the output positions only; branches are
 * summed in the order t = 0 .. F*F-1.
 *
 * Two evaluations are offered:
 *   oracle_branches_real : the steps above, literally, from the real tensor,
 *                          sums in double.
 *   oracle_branches_pm1  : the same on already binarised operands (one tensor
 *                          per branch or one shared by all), with an explicit
 *                          pad value per (branch, channel) from {-1, 0, +1};
 *                          0 is the variant in which a padded tap contributes
 *                          nothing.  z is produced twice: in double (the
 *                          definition) and in float as the chain
 *                            z = h[o];  z = fmaf(g_t[o], (float)y_t, z), t = 0..P-1
 *                          which is the precision and order in which the bit
 *                          (z >= 0) of the fused variant is decided.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

int oracle_out_dim(int in, int k, int stride, int pad);

/* Bias, then sign (Section 4.2.1, first paragraph).  x: [outer][C][inner]
 * float, bias: [C] float, s: same shape as x, int8.  The sum is rounded to
 * float before the comparison; NaN gives -1. */
void oracle_sign_bias_f32(const float *x, const float *bias, int64_t outer, int64_t C,
                          int64_t inner, int8_t *s)
{
    for (int64_t a = 0; a < outer; ++a)
        for (int64_t c = 0; c < C; ++c)
            for (int64_t i = 0; i < inner; ++i) {
                const size_t at = (size_t)((a * C + c) * inner + i);
                volatile float v = x[at] + bias[c];
                s[at] = (v >= 0.0f) ? (int8_t)1 : (int8_t)-1;
            }
}

/*
 * Literal evaluation from the real tensor.  a: [N][C][H][W] float;
 * b: [P][C] float;  w: [O][C][F][F] int8 +-1;  g, h: [P][O] float;
 * z: [N][Ho][Wo][O] double.  P = F*F.  Returns 0, or -1 for an empty output.
 */
int oracle_branches_real(const float *a, const float *b, const int8_t *w,
                         const float *g, const float *h,
                         int N, int C, int H, int W, int O, int F, int stride, int pad,
                         double *z)
{
    const int Ho = oracle_out_dim(H, F, stride, pad);
    const int Wo = oracle_out_dim(W, F, stride, pad);
    if (N < 1 || C < 1 || O < 1 || Ho < 1 || Wo < 1)
        return -1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int oh = 0; oh < Ho; ++oh)
            for (int ow = 0; ow < Wo; ++ow)
                for (int o = 0; o < O; ++o) {
                    double sum = 0.0;
                    for (int u = 0; u < F; ++u)
                        for (int v = 0; v < F; ++v) {
                            const int t = u * F + v;
                            const int ih = oh * stride - pad + u;
                            const int iw = ow * stride - pad + v;
                            const int inside = ih >= 0 && ih < H && iw >= 0 && iw < W;
                            int32_t y = 0;
                            for (int c = 0; c < C; ++c) {
                                const float shifted =
                                    inside ? a[(((size_t)n * C + c) * H + ih) * W + iw] : 0.0f;
                                volatile float biased = shifted + b[(size_t)t * C + c];
                                const int32_t xs = (biased >= 0.0f) ? 1 : -1;
                                y += xs * (int32_t)w[(((size_t)o * C + c) * F + u) * F + v];
                            }
                            sum += (double)g[(size_t)t * O + o] * (double)y + (double)h[(size_t)t * O + o];
                        }
                    z[(((size_t)n * Ho + oh) * Wo + ow) * O + o] = sum;
                }
    return 0;
}

/*
 * On binarised operands.  P is the number of branches: F*F for the shifted
 * construction (branch t = u*F + v reads the map shifted by (u, v)), any
 * P >= 1 when F = 1 (parallel branches, no shift); anything else returns -3.
 * xb: [B][N][C][H][W] int8 +-1 with B = P (one tensor
 * per branch) or B = 1 (shared != 0: every branch reads the same tensor);
 * padv: [P][C] int8 from {-1, 0, +1}, the operand a tap outside the image
 * stands for;  w: [O][C][P] int8 +-1 (for F > 1 this is [O][C][F][F]);
 * g: [P][O] float;  h: [O] float or
 * NULL (= 0), the sum of the branches' biases;  outputs, each may be NULL:
 * z64 [N][Ho][Wo][O] double (exact products, double sums), z32 the float
 * fmaf chain described at the top, y_taps [N][Ho][Wo][O][P] int32 the
 * per-branch integer sums.
 */
int oracle_branches_pm1(const int8_t *xb, int shared, const int8_t *padv, const int8_t *w,
                        const float *g, const float *h,
                        int N, int C, int H, int W, int O, int F, int P, int stride, int pad,
                        double *z64, float *z32, int32_t *y_taps)
{
    const int Ho = oracle_out_dim(H, F, stride, pad);
    const int Wo = oracle_out_dim(W, F, stride, pad);
    if (N < 1 || C < 1 || O < 1 || Ho < 1 || Wo < 1)
        return -1;
    if (P < 1 || (F > 1 && P != F * F))
        return -3;
    const size_t branch_elems = (size_t)N * C * H * W;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int oh = 0; oh < Ho; ++oh)
            for (int ow = 0; ow < Wo; ++ow)
                for (int o = 0; o < O; ++o) {
                    const size_t at = (((size_t)n * Ho + oh) * Wo + ow) * O + o;
                    double sum64 = h ? (double)h[o] : 0.0;
                    float sum32 = h ? h[o] : 0.0f;
                    for (int t = 0; t < P; ++t) {
                        const int u = (F > 1) ? t / F : 0;
                        const int v = (F > 1) ? t % F : 0;
                        const int ih = oh * stride - pad + u;
                        const int iw = ow * stride - pad + v;
                        const int inside = ih >= 0 && ih < H && iw >= 0 && iw < W;
                        const int8_t *xt = xb + (shared ? 0 : (size_t)t * branch_elems);
                        int32_t y = 0;
                        for (int c = 0; c < C; ++c) {
                            const int32_t xv = inside
                                ? (int32_t)xt[(((size_t)n * C + c) * H + ih) * W + iw]
                                : (int32_t)padv[(size_t)t * C + c];
                            y += xv * (int32_t)w[((size_t)o * C + c) * P + t];
                        }
                        if (y_taps)
                            y_taps[at * P + t] = y;
                        sum64 += (double)g[(size_t)t * O + o] * (double)y;
                        sum32 = fmaf(g[(size_t)t * O + o], (float)y, sum32);
                    }
                    if (z64)
                        z64[at] = sum64;
                    if (z32)
                        z32[at] = sum32;
                }
    return 0;
}

/*
 * What follows the binary convolution inside a convolution module (paper,
 * Section 4.2.1, first paragraph): batch norm as a per-channel scale and bias,
 * addition of the module's real identity path, PReLU with a learnable slope
 * per channel.  y: [rows][O] int32 sums;  gamma, beta: [O];  identity:
 * [rows][O] float or NULL (no identity path);  alpha: [O] or NULL (no
 * activation).  Outputs, each may be NULL: r64 in double from the plain
 * formula, r32 in float in this order of operations, one rounding each:
 *   t = fmaf(gamma[o], (float)y, beta[o]);  t = t + identity;
 *   r = (t >= 0) ? t : alpha[o] * t
 * (a NaN t takes the alpha branch).  The binarisation for the next module is
 * oracle_sign_bias_f32 on the stored r.
 */
void oracle_module_epilogue(const int32_t *y, const float *gamma, const float *beta,
                            const float *identity, const float *alpha,
                            int64_t rows, int O, double *r64, float *r32)
{
    for (int64_t m = 0; m < rows; ++m)
        for (int o = 0; o < O; ++o) {
            const size_t at = (size_t)m * O + o;
            if (r64) {
                double t = (double)gamma[o] * (double)y[at] + (double)beta[o];
                if (identity)
                    t += (double)identity[at];
                r64[at] = (t >= 0.0 || !alpha) ? t : (double)alpha[o] * t;
            }
            if (r32) {
                volatile float t = fmaf(gamma[o], (float)y[at], beta[o]);
                if (identity)
                    t = t + identity[at];
                if (!(t >= 0.0f) && alpha) {
                    volatile float a = alpha[o] * t;
                    r32[at] = a;
                } else {
                    r32[at] = t;
                }
            }
        }
}

/*
 * The same tail for a module whose binary part is a sum of parallel branches
 * (Figure 2, bottom): the branches' scaled sum z (with the batch-norm biases
 * already in it) takes the place of the batch-norm output; identity addition
 * and PReLU follow as above.  z64 / z32: [rows][O], either may be NULL
 * together with its output; identity [rows][O] float or NULL; alpha [O] or
 * NULL.  Float path, one rounding per step:  t = z + identity;
 * r = (t >= 0) ? t : alpha[o] * t.
 */
void oracle_module_tail(const double *z64, const float *z32, const float *identity,
                        const float *alpha, int64_t rows, int O, double *r64, float *r32)
{
    for (int64_t m = 0; m < rows; ++m)
        for (int o = 0; o < O; ++o) {
            const size_t at = (size_t)m * O + o;
            if (z64 && r64) {
                double t = z64[at];
                if (identity)
                    t += (double)identity[at];
                r64[at] = (t >= 0.0 || !alpha) ? t : (double)alpha[o] * t;
            }
            if (z32 && r32) {
                volatile float t = z32[at];
                if (identity)
                    t = t + identity[at];
                if (!(t >= 0.0f) && alpha) {
                    volatile float a = alpha[o] * t;
                    r32[at] = a;
                } else {
                    r32[at] = t;
                }
            }
        }
}

/*
 * Storage rounding of the real stream.  A module writes its real output in
 * the stream's type and everything behind it (the next module's bias + sign,
 * the identity addition of the module after) reads the value as stored
 * (Section 4.2.1, first paragraph: the bias is added to the module's real
 * input; the paper fixes no storage type, so the reading is: the input is
 * what memory holds).  Two 16-bit types:
 *   binary16 : 1 sign, 5 exponent bits (bias 15), 10 fraction bits
 *   bfloat16 : 1 sign, 8 exponent bits (bias 127), 7 fraction bits
 * The conversion is the IEEE 754 one: round to nearest, ties to the even
 * fraction; results at or beyond largest finite + half a step are infinity;
 * below the smallest normal number the step stays that of the smallest
 * normal exponent (gradual underflow, no flush); a NaN stays a NaN (quiet,
 * sign kept, payload dropped).  It is written out from that definition: take
 * the exponent e of |x| (not below the smallest normal one), express |x| in
 * units of 2^(e - fraction bits), round that count to an integer.
 * nearbyint() rounds ties to even in the default rounding mode, which is the
 * only one this library runs in; the division by a power of two is exact.
 */
static uint16_t store_16bit(float x, int ebits, int fbits, float *back)
{
    const int bias = (1 << (ebits - 1)) - 1;
    const int emin = 1 - bias, emax = bias;
    const uint16_t sign = signbit(x) ? (uint16_t)(1u << (ebits + fbits)) : 0;
    const uint16_t all_ones_exp = (uint16_t)(((1u << ebits) - 1u) << fbits);
    if (isnan(x)) {
        *back = signbit(x) ? -NAN : NAN;
        return (uint16_t)(sign | all_ones_exp | (1u << (fbits - 1)));
    }
    const double a = fabs((double)x);
    if (a == 0.0) {
        *back = signbit(x) ? -0.0f : 0.0f;
        return sign;
    }
    if (isinf(x)) {
        *back = x;
        return (uint16_t)(sign | all_ones_exp);
    }
    int ex;
    (void)frexp(a, &ex);            /* a = m * 2^ex with 0.5 <= m < 1, so 2^(ex-1) <= a < 2^ex */
    int e = ex - 1;
    if (e < emin)
        e = emin;
    double unit = ldexp(1.0, e - fbits);
    double count = nearbyint(a / unit);             /* 0 .. 2^(fbits+1) */
    if (count == ldexp(1.0, fbits + 1)) {           /* rounded up into the next exponent */
        e += 1;
        unit = ldexp(1.0, e - fbits);
        count = ldexp(1.0, fbits);
    }
    if (e > emax) {
        *back = signbit(x) ? -INFINITY : INFINITY;
        return (uint16_t)(sign | all_ones_exp);
    }
    const double v = count * unit;                  /* exact */
    *back = (float)(signbit(x) ? -v : v);           /* exact: every such value is a float */
    const unsigned n = (unsigned)count;
    if (n < (1u << fbits))                          /* subnormal (or zero): exponent field 0 */
        return (uint16_t)(sign | n);
    return (uint16_t)(sign | ((unsigned)(e + bias) << fbits) | (n - (1u << fbits)));
}

/* x: [count] float -> code: [count] the 16-bit patterns, back: [count] the
 * stored values read back as float (either output may be NULL). */
void oracle_store_f16(const float *x, int64_t count, uint16_t *code, float *back)
{
    for (int64_t i = 0; i < count; ++i) {
        float b;
        const uint16_t c = store_16bit(x[i], 5, 10, &b);
        if (code) code[i] = c;
        if (back) back[i] = b;
    }
}

void oracle_store_bf16(const float *x, int64_t count, uint16_t *code, float *back)
{
    for (int64_t i = 0; i < count; ++i) {
        float b;
        const uint16_t c = store_16bit(x[i], 8, 7, &b);
        if (code) code[i] = c;
        if (back) back[i] = b;
    }
}

/* The value of a bfloat16 pattern: sign, exponent field E, fraction F give
 * (-1)^s * 2^(E-127) * (1 + F/128), E = 0: (-1)^s * 2^-126 * F/128,
 * E = 255: infinity (F = 0) or NaN. */
void oracle_load_bf16(const uint16_t *code, int64_t count, float *value)
{
    for (int64_t i = 0; i < count; ++i) {
        const int s = code[i] >> 15, E = (code[i] >> 7) & 0xFF, F = code[i] & 0x7F;
        double v;
        if (E == 255)
            v = F ? (double)NAN : (double)INFINITY;
        else if (E == 0)
            v = ldexp((double)F / 128.0, -126);
        else
            v = ldexp(1.0 + (double)F / 128.0, E - 127);
        value[i] = (float)(s ? -v : v);
    }
}
