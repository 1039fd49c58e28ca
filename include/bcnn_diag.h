/*
 * libbcnn measurement helpers (C ABI).  Not part of the method of the BCNN
 * paper and not needed to use the library: bench.py and the profiling runs
 * call them to get denominators (what the vector ALUs, the matrix cores and
 * HBM sustain on this chip) and a kernel of known size to calibrate memory
 * counters against.  Same conventions as bcnn.h: device pointers owned by the
 * caller, asynchronous on the given hipStream_t (NULL = default stream), one
 * kernel launch per call, negative bcnn_status on error before any launch.
 */
#ifndef BCNN_DIAG_H
#define BCNN_DIAG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* dst[i] = src[i] for `words` 32-bit words (4-byte aligned, words >= 1). */
int bcnn_diag_copy_u32(const uint32_t *src, uint32_t *dst, int64_t words, void *hip_stream);

/* Store only: fills dst (16-byte aligned, `words` a positive multiple of 4) with a fixed pattern using
 * 16-byte non-temporal stores.  blocks = 0 launches one workgroup per 16 KB, otherwise `blocks`
 * workgroups that stride over the buffer. */
int bcnn_diag_store_u32(uint32_t *dst, int64_t words, int32_t blocks, void *hip_stream);

/* Read only: streams src (16-byte aligned, `words` a positive multiple of 4) with 16-byte non-temporal
 * loads and writes one word per lane to sink (blocks * 256 words; with blocks = 0 the launch has
 * ceil(words / 8192) workgroups and sink must hold 256 words for each). */
int bcnn_diag_read_u32(const uint32_t *src, int64_t words, uint32_t *sink, int32_t blocks, void *hip_stream);

/* Every lane runs `iters` rounds of 64 independent xor + popcount-accumulate pairs on registers and
 * writes one word to sink[global thread id]; sink holds blocks*256 words.  Times the vector ALUs'
 * xor/popcount issue rate with no memory traffic. */
int bcnn_diag_valu_peak(uint32_t *sink, int32_t blocks, int32_t iters, void *hip_stream);

/* Every wave issues `iters` rounds of 8 independent 32x32x64 fp4 matrix instructions on random +-1
 * operands held in registers and writes one float to sink[global thread id] (blocks*256 floats).
 * Times the rate the matrix cores sustain on this kind of data. */
int bcnn_diag_mfma_fp4_peak(float *sink, int32_t blocks, int32_t iters, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* BCNN_DIAG_H */
