/*
 * bcnn.h - C ABI of the binary-convolution hot path for AMD MI355X (gfx950).
 *
 * The operation is the CNN-style 2D convolution of the BCNN paper (Section 1:
 * a 3D input tensor and a 4D weight tensor give a 3D output tensor, and the
 * operator lowers to a matrix-matrix product) with both operands binary
 * (Section 4.2.1: inputs and weights are +1 or -1).  A leading batch index is
 * added; images are independent.
 *
 * Conventions shared by every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates, frees or keeps them and uses no hidden workspace.
 *   - Calls are asynchronous: kernels are enqueued on `hip_stream` (a
 *     hipStream_t passed as void*, NULL = the default stream) and the call
 *     returns without synchronising.  Outputs are valid once the stream has
 *     reached that point.
 *   - Return value: BCNN_OK (0) or a negative bcnn_status.  Arguments are
 *     checked on the host before anything is launched; a call that returns an
 *     error has launched nothing.  Pointers are checked for NULL and for
 *     4-byte alignment only; whether they really are device memory of the
 *     required size is the caller's responsibility.
 *   - Bit convention: bit 1 <=> +1, bit 0 <=> -1.  32 consecutive channels
 *     form one little-endian uint32, channel 32*j+i is bit i of word j, and
 *     the unused high bits of the last word of a channel vector are 0 in
 *     every packed tensor (inputs must obey this, outputs do).
 *   - Packed activations: [n][h][w][ceil(c/32)] uint32.
 *     Packed weights:     [c_out][kh][kw][ceil(c_in/32)] uint32.
 *   - Padding: a position outside the image counts as -1 in every channel
 *     (all-zero packed words).  The paper pads real values before bias and
 *     sign (Section 4.2.1, last paragraph), so a padded operand is a fixed
 *     +-1, never 0; -1 is the convention fixed here.
 *   - Output extent: floor((in + 2*pad - k) / stride) + 1.
 *   - Supported: kh = kw in {1, 3}; stride in {1, 2}; pad in {0, 1} with
 *     pad <= (kh-1)/2; every extent >= 1; n*h_out*w_out*c_out and
 *     n*h*w*ceil(c_in/32) below 2^31.  Anything else returns
 *     BCNN_ERR_UNSUPPORTED.
 */
#ifndef BCNN_H
#define BCNN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BCNN_OK = 0,
    BCNN_ERR_INVALID_ARG = -1, /* NULL pointer, non-positive extent, aliasing in/out */
    BCNN_ERR_UNSUPPORTED = -2, /* filter size, stride, padding or size outside the list above */
    BCNN_ERR_ALIGNMENT = -3,   /* a pointer is not 4-byte aligned */
    BCNN_ERR_DEVICE = -4       /* the HIP runtime refused the launch */
} bcnn_status;

/* BCNN_BF16: bfloat16 (1 sign, 8 exponent, 7 fraction bits), rounded to nearest even when stored */
typedef enum { BCNN_F32 = 0, BCNN_F16 = 1, BCNN_I8 = 2, BCNN_BF16 = 3 } bcnn_dtype;

/* Which arithmetic the convolution runs on.  All variants give identical
 * results; AUTO picks the fastest one measured for the shape. */
typedef enum {
    BCNN_VARIANT_AUTO = 0,
    BCNN_VARIANT_VALU = 1,     /* xor + popcount on the vector ALUs */
    BCNN_VARIANT_MFMA_I8 = 2,  /* +-1 expanded to int8, matrix cores */
    BCNN_VARIANT_MFMA_FP4 = 3, /* +-1 expanded to 4-bit floats, matrix cores; tile chosen by shape */
    BCNN_VARIANT_MFMA_FP4_T4 = 4, /* the same with 2 x 4 blocks of 32 x 32 per wave forced */
    BCNN_VARIANT_MFMA_FP4_T7 = 5, /* the same with 2 x 7 blocks forced (fused output only) */
    /* position-major tiles forced: a block of 32 rows is one output position in 32 consecutive
     * images, tiles are sorted by which filter taps fall outside the image and do not walk those.
     * Fused output, 3 x 3 filter, c_in a multiple of 256 and n a multiple of 32 only, and no
     * output row or column whose window misses the image on both sides.
     * P6: interior tiles of 2 x 6 blocks per wave, edge tiles of 2 x 7; P7: 2 x 7 throughout;
     * P5: workgroups of two waves (one block column), interior tiles of 2 x 5 blocks, edge 2 x 8;
     * P68: two waves, interior 2 x 6, edge 2 x 8 */
    BCNN_VARIANT_MFMA_FP4_P6 = 6,
    BCNN_VARIANT_MFMA_FP4_P7 = 7,
    BCNN_VARIANT_MFMA_FP4_P5 = 8,
    BCNN_VARIANT_MFMA_FP4_P68 = 9
} bcnn_variant;

typedef struct {
    int32_t n, c_in, h, w; /* input  [n][c_in][h][w] (logical) */
    int32_t c_out, kh, kw; /* weights [c_out][c_in][kh][kw] (logical) */
    int32_t stride, pad;
} bcnn_conv_desc;

/*
 * Sign-binarise and pack along the channel axis (Section 4.2.1: sign turns
 * activations, and implicitly weights, into +-1; Section 2.4: storage and
 * data movement scale with the number of bits).
 *   src : device, contiguous [outer][channels][inner] of `dtype`.
 *         NCHW activations: outer = n, inner = h*w.  OIHW weights: outer =
 *         c_out, inner = kh*kw.  Channel-last data: inner = 1.
 *   dst : device, [outer][inner][ceil(channels/32)] uint32.
 *   bit = (value >= 0); so +0.0 and -0.0 give 1, NaN gives 0.
 * Errors: INVALID_ARG for NULL or non-positive sizes, UNSUPPORTED for an
 * unknown dtype or more than 2^31-1 output words, ALIGNMENT if dst is not
 * 4-byte aligned or src not aligned to its element size.
 */
int bcnn_pack(const void *src, bcnn_dtype dtype, int64_t outer, int64_t channels, int64_t inner,
              uint32_t *dst, void *hip_stream);

/*
 * The same with a learnable per-channel bias added before the sign (Section
 * 4.2.1, first paragraph: bias, then sign, in front of every binary
 * convolution):  bit = (float(value) + bias[channel] >= 0), the sum rounded to
 * float32 (its sign is that of the exact sum; NaN gives 0).
 *   bias : device, float32 [channels].  NULL is INVALID_ARG.
 * Everything else as bcnn_pack.
 */
int bcnn_pack_bias(const void *src, bcnn_dtype dtype, int64_t outer, int64_t channels, int64_t inner,
                   const float *bias, uint32_t *dst, void *hip_stream);

/*
 * bcnn_pack_bias on a source whose channels are replicated by bookkeeping
 * (Section 4.2.2: a building block that widens the network sees every real
 * channel `replication` times; the real map is not copied): the packed
 * tensor has replication * src_channels channels, channel c is
 *   bit = (float(src[.][c mod src_channels][.]) + bias[c] >= 0).
 *   src  : device, contiguous [outer][src_channels][inner] of `dtype`
 *   bias : device, float32 [replication * src_channels]
 *   dst  : device, [outer][inner][ceil(replication * src_channels / 32)]
 * replication = 1 is bcnn_pack_bias.
 */
int bcnn_pack_bias_replicated(const void *src, bcnn_dtype dtype, int64_t outer, int64_t src_channels,
                              int64_t inner, int32_t replication, const float *bias, uint32_t *dst,
                              void *hip_stream);

/*
 * S x S average pooling with stride S of the channel-last real stream, fused
 * with the bias + sign + pack of the binary 1x1 convolution module behind it
 * (Section 4.2.3: identity path of a block that down-samples by S; Section
 * 4.2.1, first paragraph: bias, then sign).  One pass writes both consumers of
 * the pooled map:
 *   pooled[n][oh][ow][c]   = (sum over the window, raster order, float32,
 *                             one rounding per addition) / float(S*S), stored
 *                             in the stream's type (half: round to nearest even)
 *   x_packed[n][oh][ow][.] : bit c = (float(pooled as stored) + bias[c] >= 0)
 * Windows are not padded; rows and columns that do not fill a window are
 * dropped (h_out = h / S, w_out = w / S, rounded down).
 *   src        : device, [n][h][w][channels] of real_dtype (BCNN_F32, BCNN_F16 or BCNN_BF16)
 *   bias       : device, float32 [channels], or NULL for no bias
 *   pooled     : device, [n][h_out][w_out][channels] of real_dtype, or NULL
 *   x_packed   : device, [n][h_out][w_out][ceil(channels/32)], tail bits 0, or NULL
 * Errors: INVALID_ARG for NULL src, both outputs NULL, non-positive sizes, an
 * empty pooled map or an output that is the input; UNSUPPORTED for another
 * dtype, S > 8 or more than 2^31-1 output words * 8; ALIGNMENT for pointers
 * not aligned to their element size.  Rows of 4-element-aligned tensors with
 * channels a multiple of 4 take the fast path.
 */
int bcnn_avgpool_bias_sign_pack(const void *src, bcnn_dtype real_dtype, int32_t n, int32_t h, int32_t w,
                                int32_t channels, int32_t s, const float *bias, void *pooled,
                                uint32_t *x_packed, void *hip_stream);

/*
 * Binary convolution, integer sums (Section 1 operator, Section 4.2.1
 * operands):
 *   y[n][oh][ow][o] = sum_{u,v,c} X~[n][oh*s-p+u][ow*s-p+v][c] * W[o][u][v][c]
 * with X~ = -1 outside the image.  Evaluated as K - 2*popcount(x xor w) over
 * packed words, K = c_in*kh*kw.
 *   x_packed : device, packed activations  [n][h][w][ceil(c_in/32)]
 *   w_packed : device, packed weights      [c_out][kh][kw][ceil(c_in/32)]
 *   y        : device, int32 [n][h_out][w_out][c_out] (the row-major M x c_out
 *              matrix of the matrix-product view, M = n*h_out*w_out)
 */
int bcnn_conv2d_binary(const bcnn_conv_desc *desc, const uint32_t *x_packed,
                       const uint32_t *w_packed, int32_t *y, void *hip_stream);

/*
 * Binary convolution with the fused epilogue: the per-channel scale and bias
 * of batch norm followed by the next module's bias and sign (Section 4.2.1,
 * first paragraph; without the real identity path) reduce to one integer
 * threshold per output channel.  The sums never leave the chip:
 *   bit[n][oh][ow][o] = (y[n][oh][ow][o] >= thr[o])
 *   thr      : device, int32 [c_out]
 *   y_packed : device, packed activations [n][h_out][w_out][ceil(c_out/32)],
 *              directly usable as the next layer's x_packed.  Must not alias
 *              x_packed.
 */
int bcnn_conv2d_binary_sign_pack(const bcnn_conv_desc *desc, const uint32_t *x_packed,
                                 const uint32_t *w_packed, const int32_t *thr,
                                 uint32_t *y_packed, void *hip_stream);

/*
 * The two calls above with the arithmetic variant chosen by the caller, for
 * measuring one variant against another.  thr == NULL: `out` is int32 sums;
 * thr != NULL: `out` is packed bits.  A variant that does not cover the shape
 * returns BCNN_ERR_UNSUPPORTED.
 */
int bcnn_conv2d_binary_variant(const bcnn_conv_desc *desc, const uint32_t *x_packed,
                               const uint32_t *w_packed, const int32_t *thr, void *out,
                               int variant, void *hip_stream);

/*
 * Binary convolution followed by the real-valued part of a convolution module
 * (Section 4.2.1, first paragraph: batch norm as a per-channel scale and bias,
 * addition of the module's real identity path, PReLU), and the binarisation
 * the next module starts with (its bias, then sign).  Per output element, in
 * float32 and in this order, one rounding per step:
 *   t = fma(bn_scale[o], float(y), bn_bias[o])      y: the integer sum of
 *   t = t + identity[m][o]                          bcnn_conv2d_binary
 *   r = t >= 0 ? t : prelu_slope[o] * t
 *   r is rounded to real_dtype and stored;  bit = (r_stored + next_bias[o] >= 0)
 * All arrays are device memory.  identity == NULL: no identity path;
 * prelu_slope == NULL: no activation; next_bias == NULL: 0.  identity and r
 * are [n*h_out*w_out][c_out] of real_dtype (BCNN_F32, BCNN_F16 or BCNN_BF16), i.e. the
 * real stream in channel-last order; r may be the same buffer as identity
 * (the stream is updated in place).  identity_channels (0 = c_out): when the
 * block widens the network by replicating channels (Section 4.2.2), the
 * identity stream keeps its identity_channels channels, [m][identity_channels],
 * and output channel o adds identity channel o mod identity_channels; r then
 * has to be a different buffer.
 *   r             : device, real output, or NULL to skip it
 *   x_next_packed : device, packed [n][h_out][w_out][ceil(c_out/32)], or NULL
 *                   to skip it; at least one of the two outputs is required
 *   variant       : BCNN_VARIANT_AUTO, _VALU or _MFMA_FP4; others UNSUPPORTED
 */
typedef struct {
    const float *bn_scale;    /* [c_out] */
    const float *bn_bias;     /* [c_out] */
    const void *identity;     /* [m][c_out] of real_dtype, or NULL */
    const float *prelu_slope; /* [c_out], or NULL */
    const float *next_bias;   /* [c_out], or NULL */
    int32_t real_dtype;       /* BCNN_F32, BCNN_F16 or BCNN_BF16 (the branch call's tail: F32 or F16) */
    int32_t identity_channels; /* channels of the identity stream; 0 means c_out */
} bcnn_module_epilogue;

int bcnn_conv2d_binary_module(const bcnn_conv_desc *desc, const uint32_t *x_packed,
                              const uint32_t *w_packed, const bcnn_module_epilogue *ep, void *r,
                              uint32_t *x_next_packed, int variant, void *hip_stream);

/*
 * The epilogue alone (same decision as the fused call), for sums that are
 * already in memory:  y int32 [rows][c_out], thr int32 [c_out] ->
 * y_packed [rows][ceil(c_out/32)].
 */
int bcnn_threshold_sign_pack(const int32_t *y, const int32_t *thr, int64_t rows, int64_t c_out,
                             uint32_t *y_packed, void *hip_stream);

/*
 * Parallel binary 1x1 branches, each with its own real scale, summed (the
 * module with P parallel branches of Figure 2, bottom), and the F x F binary
 * convolution built from F*F such branches on shifted copies of the feature
 * map (Section 4.2.1, last paragraph):
 *   y_t[n][oh][ow][o] = sum_c X_t[n][oh*s-p+u][ow*s-p+v][c] * W[o][t][c]
 *   z[n][oh][ow][o]   = bias[o] + sum_t scale[t][o] * y_t[n][oh][ow][o]
 * evaluated in float32 as z = bias[o], then z = fma(scale[t][o], float(y_t), z)
 * for t = 0, 1, ... in this order (y_t is an exact integer).
 *   branches        : number of branches.  kh = kw = 3: must be 9, branch
 *                     t = u*kw + v reads the map shifted by (u, v).
 *                     kh = kw = 1: any count from 1 to 1024, no shift (u = v = 0).
 *   x_packed        : device, packed activations.  Branch t reads the tensor at
 *                     x_packed + t * x_branch_stride (in uint32 words), each
 *                     [n][h][w][ceil(c_in/32)]: one binarisation per branch
 *                     (its own bias before the sign, bcnn_pack_bias).
 *                     x_branch_stride = 0: every branch reads the same tensor.
 *   w_packed        : device, packed weights [c_out][branches][ceil(c_in/32)]
 *                     (for 3x3 this is the layout [c_out][kh][kw][..] of the
 *                     other calls)
 *   pad_mode        : BCNN_PAD_WORDS - a position outside the image stands for
 *                     the packed words pad_words[t][ceil(c_in/32)] (device; the
 *                     paper fills with 0 before the branch's bias, so the operand
 *                     is sign(bias_t[c]) per channel; tail bits 0); pad_words =
 *                     NULL means -1 in every channel.
 *                     BCNN_PAD_ZERO - a tap outside the image contributes
 *                     nothing to y_t (pad_words is ignored).
 *   scale           : device, float32 [branches][c_out], finite
 *   bias            : device, float32 [c_out], or NULL for 0 (the sum of the
 *                     branches' batch-norm biases, and whatever the caller
 *                     folds in)
 *   z               : device, float32 [n][h_out][w_out][c_out]
 *   z_packed        : device, packed [n][h_out][w_out][ceil(c_out/32)],
 *                     bit = (z >= 0); must not alias x_packed.
 *   variant         : BCNN_VARIANT_AUTO, _VALU or _MFMA_FP4 (the matrix-core
 *                     kernel needs c_in a multiple of 256; UNSUPPORTED otherwise);
 *                     all variants give identical results
 * Same shape limits and errors as bcnn_conv2d_binary; additionally
 * INVALID_ARG for an unknown pad_mode, a branch count that does not fit the
 * filter, or a non-zero x_branch_stride smaller than one tensor.
 */
typedef enum { BCNN_PAD_WORDS = 0, BCNN_PAD_ZERO = 1 } bcnn_pad_mode;

int bcnn_conv2d_binary_branches(const bcnn_conv_desc *desc, int32_t branches,
                                const uint32_t *x_packed, int64_t x_branch_stride, const uint32_t *w_packed,
                                const uint32_t *pad_words, int pad_mode, const float *scale,
                                const float *bias, float *z, int variant, void *hip_stream);

int bcnn_conv2d_binary_branches_sign_pack(const bcnn_conv_desc *desc, int32_t branches,
                                          const uint32_t *x_packed, int64_t x_branch_stride, const uint32_t *w_packed,
                                          const uint32_t *pad_words, int pad_mode, const float *scale,
                                          const float *bias, uint32_t *z_packed, int variant,
                                          void *hip_stream);

/*
 * The module with parallel branches (Figure 2, bottom; with kh = kw = 3 the
 * F x F construction of Section 4.2.1's last paragraph inside a module): the
 * branch sum z of bcnn_conv2d_binary_branches takes the place of the
 * batch-norm output and continues, in float32 and one rounding per step, as
 *   t = z + identity[m][o];  r = t >= 0 ? t : prelu_slope[o] * t
 *   r is rounded to real_dtype and stored;  bit = (r_stored + next_bias[o] >= 0)
 * Arguments as in bcnn_conv2d_binary_branches and bcnn_conv2d_binary_module;
 * ep->bn_scale and ep->bn_bias must be NULL here (scale[branches][c_out] and
 * bias[c_out] are the branches' batch norms).  c_out below 32 is UNSUPPORTED.
 */
int bcnn_conv2d_binary_branches_module(const bcnn_conv_desc *desc, int32_t branches,
                                       const uint32_t *x_packed, int64_t x_branch_stride,
                                       const uint32_t *w_packed, const uint32_t *pad_words, int pad_mode,
                                       const float *scale, const float *bias,
                                       const bcnn_module_epilogue *ep, void *r, uint32_t *x_next_packed,
                                       int variant, void *hip_stream);

/* floor((in + 2*pad - k)/stride) + 1, or 0 if the window does not fit. Host only. */
int bcnn_out_dim(int32_t in, int32_t k, int32_t stride, int32_t pad);

/* Static, NUL-terminated description of a bcnn_status value. Host only. */
const char *bcnn_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* BCNN_H */
