/*
 * hccs.h -- C ABI of the gfx950 implementation of the Head-Calibrated
 * Clipped-Linear Softmax (HCCS), "Taming the Exponential: A Fast Softmax
 * Surrogate for Integer-Native Edge Inference".
 *
 * Conventions for every entry point
 *   - Pointers named *_dev are device (HBM) addresses owned by the caller;
 *     pointers named *_host are host addresses, read during the call only.
 *   - Tensors are dense, row-major, innermost dimension contiguous.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL =
 *     the default stream) and the call returns after the enqueue; nothing is
 *     synchronised, nothing is allocated or freed, there is no global state.
 *   - Per-head constants travel by value in the kernel arguments, so the host
 *     table may be freed as soon as the call returns.
 *   - All checks run on the host before anything is launched.  A call that
 *     returns any status other than HCCS_OK or HCCS_E_HIP has launched nothing
 *     and has not touched its outputs.  HCCS_E_HIP is what the runtime answered
 *     to one of the call's own launches (an error left over from an earlier,
 *     unrelated runtime call is not reported here); an entry point that enqueues
 *     several kernels (hccs_calibrate_grid) may then have enqueued the earlier
 *     ones, and its outputs are undefined.
 *   - Return value: HCCS_OK (0) or a negative hccs_status.
 *   - Sizes: B*H*Lq (the number of rows) must stay below 2^31.
 *
 * Entry points that exist for tests and benchmarks only (the reciprocal and
 * normalise stages on their own, a copy kernel, a float32 comparison softmax)
 * are declared in hccs_testing.h.
 */
#ifndef HCCS_H
#define HCCS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HCCS_API __attribute__((visibility("default")))

/* Per-head calibrated constants theta_h = (B_h, S_h, Dmax_h) of Sec. III-A / III-C:
 * score s = B - S * min(max_j x_j - x, Dmax)   (Eq. (2), (3)). */
typedef struct {
    int32_t B;        /* intercept, 1..32767                       */
    int32_t S;        /* slope, 0..127 (an int8 MAC operand)       */
    int32_t Dmax;     /* clamp on the distance to the row maximum, 0..127 */
    int32_t reserved; /* ignored                                   */
} hccs_head_params;

/* Fixed-point rescale of the fused block's int32 Q.K^T accumulator to an
 * int8 logit:  x = clamp((acc * mult + 2^(shift-1)) >> shift, -128, 127)
 * with a flooring shift (round half up).  1 <= mult <= 4096, 1 <= shift <= 24.
 * The paper starts from int8 logits and does not define this step. */
typedef struct {
    int32_t mult;
    int32_t shift;
} hccs_requant;

typedef enum {
    HCCS_OK = 0,
    HCCS_E_NULL = -1,        /* a required pointer is NULL                               */
    HCCS_E_SHAPE = -2,       /* a dimension is out of the supported range                */
    HCCS_E_ALIGN = -3,       /* a device pointer is not aligned as documented            */
    HCCS_E_SCALE = -4,       /* unsupported output scale / reciprocal kind / band value  */
    HCCS_E_PARAM_RANGE = -5, /* Dmax, S or B outside its range, or B - S*Dmax < 0        */
    HCCS_E_PARAM_FLOOR = -6, /* n*(B - S*Dmax) < 256: the row sum could drop below 256   */
    HCCS_E_PARAM_CEIL = -7,  /* n*B above the band's ceiling                             */
    HCCS_E_HIP = -8,         /* the HIP runtime refused the launch                       */
    HCCS_E_REQUANT = -9,     /* mult or shift outside its range                          */
    HCCS_E_SCRATCH = -10     /* more work memory needed than the static buffer holds     */
} hccs_status;

/* Admissibility bands (Sec. IV-C "Integer Range Constraints", Eq. (11)).
 * Both require 0 <= Dmax <= 127, 0 <= S <= 127, 1 <= B <= 32767,
 * B - S*Dmax >= 0 and n*(B - S*Dmax) >= 256 (so Z >= 256 and the shifted
 * reciprocal of Eq. (8) fits 15 bits).
 * HCCS_BAND_STRICT adds n*B <= 32767 (Z <= 32767, needed by the 16-bit path).
 * HCCS_BAND_U8 replaces that by n*B <= 255*2^15 (reciprocal of Eq. (8) >= 1),
 * which is all the 8-bit path needs. */
#define HCCS_BAND_U8 0
#define HCCS_BAND_STRICT 1

#define HCCS_MAX_HEADS 64        /* table entries carried in the kernel arguments */
#define HCCS_MAX_ROW_LENGTH 65536

/* Reciprocal kinds for hccs_calibrated_softmax_i8_ex. */
#define HCCS_RECIP_EXACT 0       /* floor division, Eq. (6) / Eq. (8)           */
#define HCCS_RECIP_CLB 1         /* leading-bit approximation, Eq. (9)          */

/* Checks H table entries against a band for rows of length n (Sec. IV-C).
 * table_host: H entries.  first_bad_head (may be NULL) receives the index of
 * the first entry that fails, or -1.  Pure host function, no GPU needed.
 * Returns HCCS_OK or the status naming the violated constraint. */
HCCS_API int hccs_validate_params(const hccs_head_params *table_host, int32_t H, int32_t n, int32_t band,
                         int32_t *first_bad_head);

/* HCCS over every row of an int8 logit tensor, 8-bit output (Alg. 1 with the
 * "int8 output path" of Sec. III-B: rho = floor(255*2^15 / Z), p = (s*rho) >> 15).
 *   logits_dev  [B,H,Lq,Lk] int8; a row is the Lk keys of one (b,h,q); row r
 *               uses the constants of head (r / Lq) mod H (Sec. IV-D).
 *   probs_dev   same shape, uint8 in [0,255]; may be the same buffer as
 *               logits_dev (in place) but must not partially overlap it.
 *   B,H,Lq      >= 0 for B and Lq (an empty tensor is a no-op), 1 <= H <= HCCS_MAX_HEADS,
 *               B*H*Lq < 2^31.
 *   Lk          1..HCCS_MAX_ROW_LENGTH.  Any length and any tensor address run on the same
 *               vectorised kernels (rows up to 16384 elements in one wave's registers, longer
 *               ones in one block's); fastest when both tensors begin on a 16-byte boundary
 *               and Lk is a multiple of 16 (every vector aligned), otherwise rows are read
 *               and written with 16-byte accesses wherever they lie.
 *   table_host  H entries, validated against `band` with n = Lk.
 *   out_scale_T must be 255.
 * Errors: NULL pointers, bad shapes, out_scale_T != 255, inadmissible table. */
HCCS_API int hccs_calibrated_softmax_i8(const int8_t *logits_dev, uint8_t *probs_dev, int32_t B, int32_t H,
                               int32_t Lq, int32_t Lk, const hccs_head_params *table_host,
                               int32_t out_scale_T, int32_t band, void *hip_stream);

/* The other output modes of the same row operation.
 *   out_scale_T = 255:   out_dev is uint8  [B,H,Lq,Lk], as above.
 *   out_scale_T = 32767: out_dev is uint16 [B,H,Lq,Lk] (2-byte aligned; every vector is aligned
 *                        when both tensors are 16-byte aligned and Lk is a multiple of 8):
 *                        Alg. 1 as printed, rho = floor(32767 / Z), p = s * rho (Eq. (6), (7)).  Needs Z <= 32767, so the table is validated against
 *                        HCCS_BAND_STRICT whatever `band` says.  No in-place use.
 *   reciprocal = HCCS_RECIP_EXACT: floor division.
 *   reciprocal = HCCS_RECIP_CLB:   leading-bit approximation of Sec. III-B, Eq. (9):
 *                        k = floor(log2 Z), rho = floor(255*2^15 / 2^k) resp. floor(32767 / 2^k).
 *                        The over-estimate (< 2x) can pass T; the result saturates at T (the
 *                        paper leaves that case open).
 * Everything else as hccs_calibrated_softmax_i8. */
HCCS_API int hccs_calibrated_softmax_i8_ex(const int8_t *logits_dev, void *out_dev, int32_t B, int32_t H,
                                           int32_t Lq, int32_t Lk, const hccs_head_params *table_host,
                                           int32_t out_scale_T, int32_t reciprocal, int32_t band,
                                           void *hip_stream);

/* Fused int8 attention block for one tensor set:
 *   A = Q.K^T (int32)  ->  x = requant_h(A) (int8)  ->  P = HCCS_u8(x) row-wise, n = L
 *   ->  O = P.V (int32).  Logits and probabilities never reach HBM.
 *   q_dev,k_dev,v_dev [B,H,L,d] int8, 16-byte aligned; o_dev [B,H,L,d] int32, 16-byte aligned.
 *   Same as hccs_attention_i8_ex with Lq = Lk = L.
 *   table_host H entries validated against `band` with n = L; requant_host H entries.
 * The block is motivated, not defined, by the paper (Sec. I, Sec. II); the
 * rescale rule is the one documented at hccs_requant. */
HCCS_API int hccs_attention_i8(const int8_t *q_dev, const int8_t *k_dev, const int8_t *v_dev, int32_t *o_dev,
                               int32_t B, int32_t H, int32_t L, int32_t d,
                               const hccs_head_params *table_host, const hccs_requant *requant_host,
                               int32_t out_scale_T, int32_t band, void *hip_stream);

/* The same block with separate query and key lengths:
 *   q_dev [B,H,Lq,d], k_dev and v_dev [B,H,Lk,d] int8, o_dev [B,H,Lq,d] int32, all 16-byte aligned.
 *   d = 64 or 128; 1 <= Lk <= HCCS_MAX_ROW_LENGTH; Lq >= 0 (0 is a no-op);
 *   B*H*Lq < 2^31.  The row length of HCCS, and of the band check, is n = Lk.
 * Blocks with d = 64 and up to 896 keys keep a query tile's logits in registers and K, V in LDS
 * (beyond 448 keys only with more than 64 queries); every other shape streams K and V through
 * LDS in chunks.  Up to 4096 keys at d = 64 and 2048 at d = 128 a query tile's logits stay in
 * registers as bytes (Q.K^T once, two passes); beyond that Q.K^T is recomputed three times
 * (maximum, sum, output), because the floors of HCCS do not allow partial results to be
 * rescaled.  All are bit-exact to the same definition. */
HCCS_API int hccs_attention_i8_ex(const int8_t *q_dev, const int8_t *k_dev, const int8_t *v_dev, int32_t *o_dev,
                                  int32_t B, int32_t H, int32_t Lq, int32_t Lk, int32_t d,
                                  const hccs_head_params *table_host, const hccs_requant *requant_host,
                                  int32_t out_scale_T, int32_t band, void *hip_stream);

/* Offline calibration by grid search (Sec. III-C, Eq. (10)).  For every head h and candidate c,
 *   objective[h*n_candidates + c] = mean over the rows of head h of
 *       KL( softmax(alpha_h * x) || phat / sum(phat) ),  phat the 16-bit HCCS output of the row
 *   (the paper minimises the divergence "in the int16 space"), in double precision;
 *   +infinity for candidates outside HCCS_BAND_STRICT for n = Lk.
 *   best[h] = first index of the minimum, -1 if no candidate is admissible.
 * alpha_host: H positive dequantisation scales (real logit = alpha_h * int8 logit; the paper does
 * not name this scale, it is an input).  candidates_dev: n_candidates (1..65535) entries ON THE
 * DEVICE.  objective_dev: H*n_candidates doubles, best_dev: H int32, both on the device.
 * workspace_dev: at least hccs_calibrate_workspace_bytes(...) bytes of device memory, 8-byte
 * aligned, contents undefined on entry and exit.  B >= 1, Lq >= 1, any Lk.
 * Sums are taken in a fixed order: two calls with equal inputs give equal bits. */
HCCS_API int64_t hccs_calibrate_workspace_bytes(int32_t B, int32_t H, int32_t Lq, int32_t Lk);
HCCS_API int hccs_calibrate_grid(const int8_t *logits_dev, int32_t B, int32_t H, int32_t Lq, int32_t Lk,
                                 const double *alpha_host, const hccs_head_params *candidates_dev,
                                 int32_t n_candidates, double *objective_dev, int32_t *best_dev,
                                 void *workspace_dev, int64_t workspace_bytes, void *hip_stream);

/* hccs_calibrate_grid for callers that cannot allocate device memory or bring a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * inputs, outputs, arithmetic and bits as hccs_calibrate_grid; the work memory is a buffer of
 * HCCS_STATIC_SCRATCH_BYTES that lives inside the library (one per GPU the library runs on, held
 * until the process ends).  The call allocates and frees nothing.  A problem whose
 * hccs_calibrate_workspace_bytes(...) exceeds HCCS_STATIC_SCRATCH_BYTES returns HCCS_E_SCRATCH and
 * launches nothing (the limit covers 64 batches of [8 heads, 128 queries], the calibration set of
 * Sec. V-A).  Every call on a GPU uses that GPU's one buffer: calls that overlap in time on one
 * GPU (different streams, or different host threads) race on it and must be serialised by the
 * caller; calls on one stream are ordered by the stream.  Nothing in the buffer has to survive
 * from one call to the next, and nothing in it has to start at zero. */
#define HCCS_STATIC_SCRATCH_BYTES (36 * 1024 * 1024)
HCCS_API int hccs_calibrate_grid_static(const int8_t *logits_dev, int32_t B, int32_t H, int32_t Lq, int32_t Lk,
                                        const double *alpha_host, const hccs_head_params *candidates_dev,
                                        int32_t n_candidates, double *objective_dev, int32_t *best_dev,
                                        void *hip_stream);

/* Static description of a status code. */
HCCS_API const char *hccs_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* HCCS_H */
