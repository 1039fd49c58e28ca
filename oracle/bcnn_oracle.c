/*
 * CPU oracle for the binary (+-1 x +-1) CNN-style 2D convolution hot path.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It exists so that the HIP
 * kernels can be checked against something that is obviously right.  Only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it; the
 * library itself never does, and this file shares nothing with it (no header,
 * no packed-word helper, no popcount).
 *
 * What it computes is the plain definition, nothing else:
 *
 *   - The operator (paper, Section 1, "CNN style 2D convolution": a 3D input
 *     tensor and a 4D weight tensor give a 3D output tensor, and the operator
 *     lowers to a matrix-matrix product): cross-correlation, no kernel flip,
 *       y[n][oh][ow][o] = sum_{c,u,v} X~[n][c][oh*s-p+u][ow*s-p+v] * w[o][c][u][v]
 *     with every operand in {-1,+1} (Section 4.2.1: a feature is present (+1)
 *     or absent (-1), a weight positive (+1) or negative (-1)).  A leading
 *     batch index n is added; images are independent.
 *   - Padding: the paper pads in the real domain before bias and sign
 *     (Section 4.2.1, last paragraph), so a padded position is a fixed +-1
 *     after the sign, never a zero operand.  The convention taken here is
 *     X~ = -1 outside the image, for every channel.
 *   - sign(v) = +1 for v >= 0, else -1 (the paper only says "sign"); NaN
 *     compares false and therefore gives -1.
 *   - Epilogue: batch-norm scale/bias and the next module's bias-then-sign
 *     (Section 4.2.1, first paragraph), without the real identity path,
 *     collapse to one integer threshold per output channel:
 *     bit = (y >= thr[o]).
 *   - Packing: 32 consecutive channels to one 32-bit word, channel 32*j+i is
 *     bit i of word j (bit 1 <=> +1), unused high bits of the last word are 0.
 *     Bit-level storage is the point of binarisation (Section 2.4: memory and
 *     data movement scale with the number of bits).
 *
 * Arithmetic is int8 operands, int32 sums, seven nested loops.  No blocking,
 * no bit tricks.  OpenMP only splits the outermost (n, oh) iterations.
 *
 * Every function here is pinned by tests/test_oracle_pins.py against things
 * other than itself: hand-worked examples (tests/golden/), a brute-force
 * float evaluation of the textbook double sum on an explicitly padded tensor,
 * a library convolution and an integer matrix product, closed forms and
 * parity/range invariants.
 */
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Output extent of a strided, padded window sweep: floor((in + 2p - k)/s) + 1.
 * (The paper's Table 1 only shows exact halvings; floor is the reading.) */
int oracle_out_dim(int in, int k, int stride, int pad)
{
    int span = in + 2 * pad - k;
    if (span < 0 || stride < 1)
        return 0;
    return span / stride + 1;
}

/* sign of real values -> +-1 (Section 4.2.1: sign binarises activations). */
void oracle_sign_f32(const float *x, int64_t count, int8_t *s)
{
    for (int64_t i = 0; i < count; ++i)
        s[i] = (x[i] >= 0.0f) ? (int8_t)1 : (int8_t)-1;
}

/*
 * The operator.  x: [N][C][H][W] int8 in {-1,+1};  w: [O][C][KH][KW] int8 in
 * {-1,+1};  y: [N][Ho][Wo][O] int32 (row-major M x O matrix with
 * M = N*Ho*Wo, the matrix-product view of Section 1).  Returns 0, or -1 if
 * the output would be empty.
 */
int oracle_conv2d_pm1(const int8_t *x, const int8_t *w,
                      int N, int C, int H, int W, int O, int KH, int KW,
                      int stride, int pad, int32_t *y)
{
    const int Ho = oracle_out_dim(H, KH, stride, pad);
    const int Wo = oracle_out_dim(W, KW, stride, pad);
    if (N < 1 || C < 1 || O < 1 || Ho < 1 || Wo < 1)
        return -1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int oh = 0; oh < Ho; ++oh)
            for (int ow = 0; ow < Wo; ++ow)
                for (int o = 0; o < O; ++o) {
                    int32_t acc = 0;
                    for (int c = 0; c < C; ++c)
                        for (int u = 0; u < KH; ++u)
                            for (int v = 0; v < KW; ++v) {
                                const int ih = oh * stride - pad + u;
                                const int iw = ow * stride - pad + v;
                                int32_t xv = -1; /* outside the image */
                                if (ih >= 0 && ih < H && iw >= 0 && iw < W)
                                    xv = x[(((size_t)n * C + c) * H + ih) * W + iw];
                                acc += xv * (int32_t)w[(((size_t)o * C + c) * KH + u) * KW + v];
                            }
                    y[(((size_t)n * Ho + oh) * Wo + ow) * O + o] = acc;
                }
    return 0;
}

/* The same sum for a list of single outputs: idx holds count quadruples
 * (n, oh, ow, o); out[i] receives that one element.  For spot checks at sizes
 * where the full tensor would take too long. */
int oracle_conv2d_pm1_at(const int8_t *x, const int8_t *w,
                         int N, int C, int H, int W, int O, int KH, int KW,
                         int stride, int pad,
                         const int32_t *idx, int64_t count, int32_t *out)
{
    const int Ho = oracle_out_dim(H, KH, stride, pad);
    const int Wo = oracle_out_dim(W, KW, stride, pad);
    if (N < 1 || C < 1 || O < 1 || Ho < 1 || Wo < 1)
        return -1;
    for (int64_t i = 0; i < count; ++i) {
        const int n = idx[4 * i + 0], oh = idx[4 * i + 1];
        const int ow = idx[4 * i + 2], o = idx[4 * i + 3];
        if (n < 0 || n >= N || oh < 0 || oh >= Ho || ow < 0 || ow >= Wo || o < 0 || o >= O)
            return -2;
    }
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t i = 0; i < count; ++i) {
        const int n = idx[4 * i + 0], oh = idx[4 * i + 1];
        const int ow = idx[4 * i + 2], o = idx[4 * i + 3];
        int32_t acc = 0;
        for (int c = 0; c < C; ++c)
            for (int u = 0; u < KH; ++u)
                for (int v = 0; v < KW; ++v) {
                    const int ih = oh * stride - pad + u;
                    const int iw = ow * stride - pad + v;
                    int32_t xv = -1;
                    if (ih >= 0 && ih < H && iw >= 0 && iw < W)
                        xv = x[(((size_t)n * C + c) * H + ih) * W + iw];
                    acc += xv * (int32_t)w[(((size_t)o * C + c) * KH + u) * KW + v];
                }
        out[i] = acc;
    }
    return 0;
}

/* Epilogue decision: s = +1 where y >= thr[channel], else -1.
 * y: [rows][O] int32, thr: [O] int32, s: [rows][O] int8. */
void oracle_threshold_sign(const int32_t *y, const int32_t *thr,
                           int64_t rows, int O, int8_t *s)
{
    for (int64_t r = 0; r < rows; ++r)
        for (int o = 0; o < O; ++o)
            s[r * O + o] = (y[r * O + o] >= thr[o]) ? (int8_t)1 : (int8_t)-1;
}

/* Channel packing.  s: [outer][C][inner] int8 in {-1,+1} (anything > 0 counts
 * as +1);  dst: [outer][inner][ceil(C/32)] uint32, bit i of word j is channel
 * 32*j+i, tail bits 0. */
void oracle_pack_channels(const int8_t *s, int64_t outer, int64_t C, int64_t inner,
                          uint32_t *dst)
{
    const int64_t Cw = (C + 31) / 32;
    for (int64_t a = 0; a < outer; ++a)
        for (int64_t i = 0; i < inner; ++i)
            for (int64_t j = 0; j < Cw; ++j) {
                uint32_t word = 0;
                for (int64_t b = 0; b < 32; ++b) {
                    const int64_t c = 32 * j + b;
                    if (c < C && s[(a * C + c) * inner + i] > 0)
                        word |= (uint32_t)1 << b;
                }
                dst[(a * inner + i) * Cw + j] = word;
            }
}

/* Inverse of the above: every channel < C becomes +-1. */
void oracle_unpack_channels(const uint32_t *src, int64_t outer, int64_t C, int64_t inner,
                            int8_t *s)
{
    const int64_t Cw = (C + 31) / 32;
    for (int64_t a = 0; a < outer; ++a)
        for (int64_t c = 0; c < C; ++c)
            for (int64_t i = 0; i < inner; ++i) {
                const uint32_t word = src[(a * inner + i) * Cw + c / 32];
                s[(a * C + c) * inner + i] = ((word >> (c % 32)) & 1u) ? (int8_t)1 : (int8_t)-1;
            }
}
