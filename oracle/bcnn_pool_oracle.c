/*
 * CPU oracle, third part: the average pooling that stands in front of the
 * binary 1x1 convolution module on the identity path of a down-sampling block.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE (see bcnn_oracle.c): only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it, and
 * it shares nothing with the library.
 *
 * What it follows (paper, Section 4.2.3): where a block down-samples by a
 * factor S, its identity path becomes S x S average pooling with stride S
 * followed by a binary 1x1 convolution module.  That module (Section 4.2.1,
 * first paragraph) adds its bias to the pooled real map, takes the sign and
 * feeds the binary convolution, and it adds the pooled real map itself as its
 * identity.  So the pooling has two consumers, the real pooled map and its
 * bias-sign bits; the bits are oracle_sign_bias_f32 (bcnn_branches_oracle.c)
 * applied to the pooled map as stored.
 *
 * Readings where the paper is silent: windows do not overlap and are not
 * padded; rows and columns that do not fill a whole window are dropped
 * (Ho = floor(H / S)); the mean is the plain sum over the window divided by
 * S*S.  The float evaluation adds the window's values in raster order (row of
 * the window outer, column inner), one rounding per addition, then divides by
 * (float)(S*S) with one rounding.
 */
#include <stddef.h>
#include <stdint.h>

/*
 * a: [N][H][W][C] float (channel last, the layout of the real stream between
 * modules);  outputs, each may be NULL: p64 [N][H/S][W/S][C] double (double
 * sums), p32 the float chain described above.  Returns 0, -1 for an empty
 * output, -2 for S < 1.
 */
int oracle_avgpool_nhwc(const float *a, int N, int H, int W, int C, int S, double *p64, float *p32)
{
    if (S < 1)
        return -2;
    const int Ho = H / S, Wo = W / S;
    if (N < 1 || C < 1 || Ho < 1 || Wo < 1)
        return -1;
    const float count32 = (float)(S * S);
    const double count64 = (double)(S * S);
    for (int n = 0; n < N; ++n)
        for (int oh = 0; oh < Ho; ++oh)
            for (int ow = 0; ow < Wo; ++ow)
                for (int c = 0; c < C; ++c) {
                    double sum64 = 0.0;
                    volatile float sum32 = 0.0f;
                    for (int u = 0; u < S; ++u)
                        for (int v = 0; v < S; ++v) {
                            const float x = a[(((size_t)n * H + (size_t)(oh * S + u)) * W + (size_t)(ow * S + v)) * C + c];
                            sum64 += (double)x;
                            if (u == 0 && v == 0)
                                sum32 = x;             /* the chain starts from the first value, not from +0 */
                            else
                                sum32 = sum32 + x;
                        }
                    const size_t at = (((size_t)n * Ho + oh) * Wo + ow) * C + c;
                    if (p64)
                        p64[at] = sum64 / count64;
                    if (p32) {
                        volatile float q = sum32 / count32;
                        p32[at] = q;
                    }
                }
    return 0;
}
