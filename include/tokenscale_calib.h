/*
 * tokenscale_calib.h -- measurement aids of the MI355X mixed paged-attention library.
 *
 * Nothing here is a step of the attention pass.  These launches of known traffic / known
 * arithmetic exist so that hardware-counter readings and kernel rates of the pass can be scaled
 * against them on the same GPU: a streaming copy and a streaming read for the HBM counters, a
 * stream of back-to-back matrix instructions for what the matrix cores sustain on given data.
 * Return value 0 = success, -1 = invalid argument (checked before anything is launched),
 * otherwise the HIP error code of the launch.  All are asynchronous on `stream` (a hipStream_t
 * passed as void*, NULL = default stream) and work on the calling thread's current device.
 */
#ifndef TOKENSCALE_CALIB_H
#define TOKENSCALE_CALIB_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* A plain streaming copy (dst[i] = src[i]) and a
 * streaming read (sum into a 4-byte result) of `bytes` bytes (multiple of 16) of DEV memory,
 * launched on `stream`.  They let a profile be scaled against a kernel of known traffic. */
int ts_calib_copy(void *stream, const void *src, void *dst, int64_t bytes);
int ts_calib_read(void *stream, const void *src, void *result4, int64_t bytes);

/* Calibration helper for the matrix cores: one resident workgroup per CU issues `iters` x 16
 * bf16 32x32x16 MFMAs per wave (8 waves, two per SIMD) back to back, A operands read from LDS as in
 * the prefill kernel; softmax != 0 adds that kernel's vector work per MFMA (multiply-add,
 * exponential, add, half a pack).  operands: DEV, 131072 bytes of bf16 values of the caller's
 * choosing (the rate the chip sustains depends on how many bits toggle: the clock it holds under
 * this load is set by its power limit); result4: DEV, 4 bytes; iters: 1..200000; *flops (HOST) is
 * set to the floating-point operations of the launch.  Asynchronous on `stream`. */
int ts_calib_mfma(void *stream, const void *operands, void *result4, int iters, int softmax, int64_t *flops);

#ifdef __cplusplus
}
#endif
#endif /* TOKENSCALE_CALIB_H */
