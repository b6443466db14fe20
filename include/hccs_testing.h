/*
 * hccs_testing.h -- entry points of libhccs.so that exist for TESTS AND BENCHMARKS ONLY.
 *
 * None of them is part of the method's path: two expose single stages of the row kernels so
 * that exhaustive checks can reach the GPU arithmetic directly, one a piece of host logic that
 * picks a kernel, one is a plain copy kernel
 * (reference point for streaming rates and for scaling hardware byte counters), one is a
 * float32 exact-exponential softmax with the same memory traffic (comparison only).
 * Conventions as in hccs.h.
 */
#ifndef HCCS_TESTING_H
#define HCCS_TESTING_H

#include "hccs.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Comparison kernel for benchmarks only (never parity-checked): exact-exponential
 * float32 softmax of the same int8 logits, out = rint(255 * softmax(scale_h * x)),
 * same traffic (1 byte in, 1 byte out per element).  scale_host: H floats.
 * Requires Lk a multiple of 16, Lk <= 16384, 16-byte aligned pointers. */
HCCS_API int hccs_exp_softmax_i8_f32(const int8_t *logits_dev, uint8_t *probs_dev, int32_t B, int32_t H,
                            int32_t Lq, int32_t Lk, const float *scale_host, void *hip_stream);

/* Test hook: runs the kernels' reciprocal routine, rho = floor(255*2^15 / Z),
 * over an array.  z_dev, rho_dev: count uint32 values on the device, every
 * Z in [256, 255*2^15] (the range the admissibility band guarantees).  Lets
 * the exhaustive check of Eq. (8) reach the GPU code. */
HCCS_API int hccs_reciprocal_u8(const uint32_t *z_dev, uint32_t *rho_dev, int64_t count, void *hip_stream);

/* Test hook: the kernels' normalise stage alone.  bsdz_dev: count quadruples (B, S, Dmax, Z) of
 * int32 on the device (16-byte aligned), each with 0 <= S*Dmax <= B <= Z and 256 <= Z <= 255*2^15,
 * which is what a row under either band produces.  out_dev: count*256 bytes, entry i holding
 * ((B - S*min(delta, Dmax)) * floor(255*2^15 / Z)) >> 15 for delta = 0..255.  Lets a sweep over the
 * constants reach the exact-float arithmetic of the 8-bit path directly. */
HCCS_API int hccs_normalise_table_u8(const int32_t *bsdz_dev, uint8_t *out_dev, int64_t count, void *hip_stream);

/* Test hook, host only (no GPU work): the bound the fused kernels use to decide whether the
 * probabilities of a table may enter the signed matrix unit as they are.  For each of the H
 * heads of params_host ((B, S, Dmax) triples, as for hccs_attention_i8), bound_host[h] receives
 * the largest probability a row of n keys can produce under the 8-bit output path: that of a
 * row with one key at the maximum and every other key beyond the window (Eq. (3), (5), (8)).
 * Returns HCCS_E_NULL, HCCS_E_SHAPE (H outside 1..HCCS_MAX_HEADS, n < 1) or HCCS_OK; the
 * parameters are not checked against a band. */
HCCS_API int hccs_largest_probability_u8(const int32_t *params_host, int32_t H, int32_t n, int32_t *bound_host);

/* Plain device-to-device copy kernel (uint4 per lane), used to scale hardware
 * byte counters and as the streaming reference point in benchmarks.
 * bytes must be a multiple of 16; pointers 16-byte aligned. */
HCCS_API int hccs_copy_bytes(const void *src_dev, void *dst_dev, int64_t bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* HCCS_TESTING_H */
