/*
 * HCCS reference oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, scalar, deliberately slow CPU statement of the Head-Calibrated
 * Clipped-Linear Softmax, written from the paper's definitions.  Only the test
 * suite, the smoke check and the benchmark's CPU-baseline leg may call it; the
 * GPU library never does, and the two share no code, headers, tables or
 * helpers.  Every intermediate is held in 64-bit integers and every range the
 * paper states is re-checked as it is produced, so a violated bound is an
 * error return, never a silent wrap.
 *
 * Functions and the passage each follows:
 *   hccs_oracle_check_params   Sec. IV-C (integer range constraints), Eq. (11)
 *   hccs_oracle_row_u8         Alg. 1 with the "int8 output path" paragraph of
 *                              Sec. III-B (Eq. (8), R = 15) in place of its
 *                              reciprocal / scaling steps
 *   hccs_oracle_row_i16        Alg. 1 as printed (Eq. (6), (7), T = 32767)
 *   hccs_oracle_row_clb_*      Sec. III-B "leading-bit detection", Eq. (9)
 *   hccs_oracle_softmax_*      Sec. IV-D: rows are independent, the head of a
 *                              row selects its parameters
 *   hccs_oracle_calibrate      Sec. III-C, Eq. (10): mean KL(softmax || HCCS) per head and
 *                              candidate, in the 16-bit output space; arg-min per head
 *   hccs_oracle_attention_i8   int8 Q.K^T -> per-head requantisation -> HCCS
 *                              -> P.V ; the paper only motivates this block
 *                              (Sec. I, Sec. II), the requantisation rule is
 *                              this repository's own definition (see below).
 *
 * Pins (tests, CPU only): hand-worked rows under tests/golden/, the exact
 * rational sandwich for the two-step normalisation, invariants (range,
 * monotonicity, sum bounds), closed forms for flat / one-hot rows, brute
 * force over every int8 row of length 2 against an independent big-integer
 * Python version, and an exhaustive check of the reciprocal; the same cases also run
 * through a build of this file with the address and undefined-behaviour sanitizers
 * (sanitize_driver.c).
 * The fused block has no definition in the paper: its composition is pinned
 * to the row function and to library matrix products, its requantisation to
 * exact rational rounding.  Parity for the fused block is therefore pinned to
 * this repository's reading only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_E_ARG -1          /* null pointer, non-positive size            */
#define ORACLE_E_PARAM_RANGE -5  /* D, S, B outside their ranges, or B-S*D < 0 */
#define ORACLE_E_PARAM_FLOOR -6  /* n*(B-S*D) < 256                            */
#define ORACLE_E_PARAM_CEIL -7   /* upper limit on n*B violated                */
#define ORACLE_E_INTERNAL -100   /* a bound the paper states did not hold      */

#define INV_SHIFT 15             /* R of Eq. (8)                               */
#define OUT_SHIFT 0              /* the paper names it, gives no value; 0 makes
                                    the result fill [0,255] and sum to ~255   */

/* Sec. IV-C.  band 1: every listed constraint (the band of Eq. (11)).
 * band 0: the constraints the 8-bit output path needs -- the same list with
 * the int16-path limit n*B <= 32767 replaced by n*B <= 255*2^15, which is what
 * keeps the reciprocal of Eq. (8) at least 1.  n <= 65536 keeps Z in 31 bits. */
int hccs_oracle_check_params(int64_t B, int64_t S, int64_t D, int64_t n, int band)
{
    if (n < 1 || n > 65536) return ORACLE_E_ARG;
    if (D < 0 || D > 127) return ORACLE_E_PARAM_RANGE;      /* delta fits int8        */
    if (S < 0 || S > 127) return ORACLE_E_PARAM_RANGE;      /* int8 MAC operand       */
    if (B < 1 || B > 32767) return ORACLE_E_PARAM_RANGE;    /* int16 score storage    */
    if (B - S * D < 0) return ORACLE_E_PARAM_RANGE;         /* Eq. (4)                */
    if (n * (B - S * D) < 256) return ORACLE_E_PARAM_FLOOR; /* Z >= 256               */
    if (band == 1) {
        if (n * B > 32767) return ORACLE_E_PARAM_CEIL;      /* Z <= 32767             */
    } else {
        if (n * B > ((int64_t)255 << INV_SHIFT)) return ORACLE_E_PARAM_CEIL;
    }
    return ORACLE_OK;
}

/* Steps shared by every output mode: row maximum, clamped unsigned distance
 * (Eq. (2)), clipped-linear score (Eq. (3)), row sum (Eq. (5)).
 * s must hold n entries.  Returns Z through *Z_out. */
static int scores_and_sum(const int8_t *x, int64_t n, int64_t B, int64_t S, int64_t D,
                          int64_t *s, int64_t *Z_out)
{
    int64_t m = x[0];
    for (int64_t i = 1; i < n; ++i)
        if (x[i] > m) m = x[i];
    int64_t Z = 0;
    for (int64_t i = 0; i < n; ++i) {
        int64_t delta = m - (int64_t)x[i];
        if (delta > D) delta = D;
        if (delta < 0 || delta > 127) return ORACLE_E_INTERNAL;
        int64_t si = B - S * delta;
        if (si < 0 || si > 32767) return ORACLE_E_INTERNAL;
        s[i] = si;
        Z += si;
    }
    *Z_out = Z;
    return ORACLE_OK;
}

/* One row, 8-bit output: rho = floor(255*2^15 / Z), p_i = (s_i*rho) >> 15. */
int hccs_oracle_row_u8(const int8_t *x, int64_t n, int64_t B, int64_t S, int64_t D,
                       uint8_t *p, int64_t *Z_out, int64_t *rho_out)
{
    if (!x || !p || n < 1) return ORACLE_E_ARG;
    int64_t *s = (int64_t *)malloc((size_t)n * sizeof(int64_t));
    if (!s) return ORACLE_E_ARG;
    int64_t Z;
    int rc = scores_and_sum(x, n, B, S, D, s, &Z);
    if (rc == ORACLE_OK && Z < 256) rc = ORACLE_E_INTERNAL;
    if (rc == ORACLE_OK) {
        int64_t rho = (((int64_t)255) << INV_SHIFT) / Z;
        if (rho < 1 || rho > 32767) rc = ORACLE_E_INTERNAL;
        for (int64_t i = 0; rc == ORACLE_OK && i < n; ++i) {
            int64_t pi = (s[i] * rho) >> (INV_SHIFT + OUT_SHIFT);
            if (pi < 0 || pi > 255) rc = ORACLE_E_INTERNAL;
            p[i] = (uint8_t)pi;
        }
        if (Z_out) *Z_out = Z;
        if (rho_out) *rho_out = rho;
    }
    free(s);
    return rc;
}

/* One row, 16-bit output exactly as Alg. 1 prints it: rho = floor(32767 / Z),
 * p_i = s_i * rho.  Needs the strict band (Z <= 32767). */
int hccs_oracle_row_i16(const int8_t *x, int64_t n, int64_t B, int64_t S, int64_t D,
                        uint16_t *p, int64_t *Z_out, int64_t *rho_out)
{
    if (!x || !p || n < 1) return ORACLE_E_ARG;
    int64_t *s = (int64_t *)malloc((size_t)n * sizeof(int64_t));
    if (!s) return ORACLE_E_ARG;
    int64_t Z;
    int rc = scores_and_sum(x, n, B, S, D, s, &Z);
    if (rc == ORACLE_OK && (Z < 1 || Z > 32767)) rc = ORACLE_E_INTERNAL;
    if (rc == ORACLE_OK) {
        int64_t rho = 32767 / Z;
        if (rho < 1) rc = ORACLE_E_INTERNAL;
        for (int64_t i = 0; rc == ORACLE_OK && i < n; ++i) {
            int64_t pi = s[i] * rho;
            if (pi < 0 || pi > 32767) rc = ORACLE_E_INTERNAL;
            p[i] = (uint16_t)pi;
        }
        if (Z_out) *Z_out = Z;
        if (rho_out) *rho_out = rho;
    }
    free(s);
    return rc;
}

/* k = floor(log2 Z) by counting halvings. */
static int floor_log2(int64_t Z)
{
    int k = 0;
    while (Z > 1) { Z >>= 1; ++k; }
    return k;
}

/* Leading-bit reciprocal, Eq. (9), 8-bit output.  The paper gives rho ~ T/2^k
 * for the generic scale; carried to the shifted reciprocal of Eq. (8) that is
 * rho = floor(255*2^15 / 2^k).  Because 2^k <= Z the product can exceed the
 * 8-bit range by up to 2x; the paper does not say what then happens, this
 * repository saturates at 255.  rho itself is kept in 64 bits here. */
int hccs_oracle_row_clb_u8(const int8_t *x, int64_t n, int64_t B, int64_t S, int64_t D,
                           uint8_t *p, int64_t *Z_out, int64_t *rho_out)
{
    if (!x || !p || n < 1) return ORACLE_E_ARG;
    int64_t *s = (int64_t *)malloc((size_t)n * sizeof(int64_t));
    if (!s) return ORACLE_E_ARG;
    int64_t Z;
    int rc = scores_and_sum(x, n, B, S, D, s, &Z);
    if (rc == ORACLE_OK && Z < 256) rc = ORACLE_E_INTERNAL;
    if (rc == ORACLE_OK) {
        int k = floor_log2(Z);
        int64_t rho = (((int64_t)255) << INV_SHIFT) / ((int64_t)1 << k);
        for (int64_t i = 0; i < n; ++i) {
            int64_t pi = (s[i] * rho) >> (INV_SHIFT + OUT_SHIFT);
            if (pi < 0) rc = ORACLE_E_INTERNAL;
            if (pi > 255) pi = 255;
            p[i] = (uint8_t)pi;
        }
        if (Z_out) *Z_out = Z;
        if (rho_out) *rho_out = rho;
    }
    free(s);
    return rc;
}

/* Leading-bit reciprocal, Eq. (9), 16-bit output: rho = floor(32767 / 2^k),
 * p_i = s_i*rho, saturated at 32767 (same unstated-overflow reading). */
int hccs_oracle_row_clb_i16(const int8_t *x, int64_t n, int64_t B, int64_t S, int64_t D,
                            uint16_t *p, int64_t *Z_out, int64_t *rho_out)
{
    if (!x || !p || n < 1) return ORACLE_E_ARG;
    int64_t *s = (int64_t *)malloc((size_t)n * sizeof(int64_t));
    if (!s) return ORACLE_E_ARG;
    int64_t Z;
    int rc = scores_and_sum(x, n, B, S, D, s, &Z);
    if (rc == ORACLE_OK && (Z < 1 || Z > 32767)) rc = ORACLE_E_INTERNAL;
    if (rc == ORACLE_OK) {
        int k = floor_log2(Z);
        int64_t rho = 32767 / ((int64_t)1 << k);
        for (int64_t i = 0; i < n; ++i) {
            int64_t pi = s[i] * rho;
            if (pi < 0) rc = ORACLE_E_INTERNAL;
            if (pi > 32767) pi = 32767;
            p[i] = (uint16_t)pi;
        }
        if (Z_out) *Z_out = Z;
        if (rho_out) *rho_out = rho;
    }
    free(s);
    return rc;
}

/* Whole tensor [Bt,H,Lq,Lk]: row r belongs to head (r / Lq) mod H (Sec. IV-D:
 * each row is processed on its own, with its head's constants).
 * table holds H triples (B, S, Dmax).  mode: 0 = u8 exact, 1 = i16 exact,
 * 2 = u8 leading-bit, 3 = i16 leading-bit.  out is uint8 for even modes and
 * uint16 for odd ones.  threads > 1 spreads whole rows over that many OpenMP
 * threads; the arithmetic of a row is unchanged. */
int hccs_oracle_softmax(const int8_t *logits, void *out, int64_t Bt, int64_t H, int64_t Lq,
                        int64_t Lk, const int32_t *table, int band, int mode, int threads)
{
    if (!logits || !out || !table) return ORACLE_E_ARG;
    if (Bt < 0 || H < 1 || Lq < 0 || Lk < 1 || mode < 0 || mode > 3) return ORACLE_E_ARG;
    if ((mode & 1) && band != 1) return ORACLE_E_ARG;
    for (int64_t h = 0; h < H; ++h) {
        int rc = hccs_oracle_check_params(table[3 * h], table[3 * h + 1], table[3 * h + 2], Lk, band);
        if (rc != ORACLE_OK) return rc;
    }
    const int64_t rows = Bt * H * Lq;
    int status = ORACLE_OK;
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const int64_t h = (r / Lq) % H;
        const int64_t B = table[3 * h], S = table[3 * h + 1], D = table[3 * h + 2];
        const int8_t *x = logits + r * Lk;
        int rc;
        if (mode == 0) rc = hccs_oracle_row_u8(x, Lk, B, S, D, (uint8_t *)out + r * Lk, 0, 0);
        else if (mode == 1) rc = hccs_oracle_row_i16(x, Lk, B, S, D, (uint16_t *)out + r * Lk, 0, 0);
        else if (mode == 2) rc = hccs_oracle_row_clb_u8(x, Lk, B, S, D, (uint8_t *)out + r * Lk, 0, 0);
        else rc = hccs_oracle_row_clb_i16(x, Lk, B, S, D, (uint16_t *)out + r * Lk, 0, 0);
        if (rc != ORACLE_OK) {
#pragma omp critical
            status = rc;
        }
    }
    return status;
}

/* Fused block: Q [Bt,H,Lq,d], K and V [Bt,H,Lk,d] int8 -> O [Bt,H,Lq,d] int32.
 * Per (b,h):
 *   A[i][j] = sum_t Q[i][t]*K[j][t]                      (no 1/sqrt(d): any such
 *                                                         factor lives in mult/shift)
 *   x[i][j] = clamp((A[i][j]*mult_h + 2^(shift_h-1)) >> shift_h, -128, 127)
 *             with a flooring (arithmetic) shift: round half up
 *   p[i][.] = HCCS 8-bit row of x[i][.] with n = Lk and head h's constants
 *   O[i][t] = sum_j p[i][j]*V[j][t]
 * requant holds H pairs (mult, shift), 1 <= mult <= 4096, 1 <= shift <= 24 (the largest
 * product, 2^18 * 2^12 for 64 products of 6-bit magnitudes, still fits 32 bits; here it
 * is held in 64).
 * This requantisation rule is this repository's definition, not the paper's. */
int hccs_oracle_attention_i8(const int8_t *q, const int8_t *k, const int8_t *v, int32_t *o,
                             int64_t Bt, int64_t H, int64_t Lq, int64_t Lk, int64_t d,
                             const int32_t *table, const int32_t *requant, int band, int threads)
{
    if (!q || !k || !v || !o || !table || !requant) return ORACLE_E_ARG;
    if (Bt < 0 || H < 1 || Lq < 0 || Lk < 1 || d < 1) return ORACLE_E_ARG;
    for (int64_t h = 0; h < H; ++h) {
        int rc = hccs_oracle_check_params(table[3 * h], table[3 * h + 1], table[3 * h + 2], Lk, band);
        if (rc != ORACLE_OK) return rc;
        if (requant[2 * h] < 1 || requant[2 * h] > 4096) return ORACLE_E_ARG;
        if (requant[2 * h + 1] < 1 || requant[2 * h + 1] > 24) return ORACLE_E_ARG;
    }
    int status = ORACLE_OK;
    if (threads < 1) threads = 1;
    const int64_t blocks = Bt * H;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t bh = 0; bh < blocks; ++bh) {
        const int64_t h = bh % H;
        const int64_t B = table[3 * h], S = table[3 * h + 1], D = table[3 * h + 2];
        const int64_t mult = requant[2 * h], shift = requant[2 * h + 1];
        const int8_t *Q = q + bh * Lq * d, *K = k + bh * Lk * d, *V = v + bh * Lk * d;
        int32_t *O = o + bh * Lq * d;
        int8_t *x = (int8_t *)malloc((size_t)Lk);
        uint8_t *p = (uint8_t *)malloc((size_t)Lk);
        for (int64_t i = 0; i < Lq; ++i) {
            for (int64_t j = 0; j < Lk; ++j) {
                int64_t acc = 0;
                for (int64_t t = 0; t < d; ++t) acc += (int64_t)Q[i * d + t] * (int64_t)K[j * d + t];
                int64_t prod = acc * mult + ((int64_t)1 << (shift - 1));
                /* floor division by 2^shift, written without relying on how the
                 * compiler shifts negative numbers */
                int64_t two = (int64_t)1 << shift;
                int64_t y = prod / two;
                if (prod % two != 0 && prod < 0) y -= 1;
                if (y < -128) y = -128;
                if (y > 127) y = 127;
                x[j] = (int8_t)y;
            }
            int rc = hccs_oracle_row_u8(x, Lk, B, S, D, p, 0, 0);
            if (rc != ORACLE_OK) {
#pragma omp critical
                status = rc;
            }
            for (int64_t t = 0; t < d; ++t) {
                int64_t acc = 0;
                for (int64_t j = 0; j < Lk; ++j) acc += (int64_t)p[j] * (int64_t)V[j * d + t];
                if (acc > INT32_MAX || acc < INT32_MIN) {
#pragma omp critical
                    status = ORACLE_E_INTERNAL;
                }
                O[i * d + t] = (int32_t)acc;
            }
        }
        free(x);
        free(p);
    }
    return status;
}

/* The int8 logits the fused block feeds to HCCS, exposed so that a test can
 * look at the middle of the pipeline: x [Bt,H,Lq,Lk]. */
int hccs_oracle_requant_logits(const int8_t *q, const int8_t *k, int8_t *x, int64_t Bt, int64_t H,
                               int64_t Lq, int64_t Lk, int64_t d, const int32_t *requant)
{
    if (!q || !k || !x || !requant) return ORACLE_E_ARG;
    for (int64_t bh = 0; bh < Bt * H; ++bh) {
        const int64_t h = bh % H;
        const int64_t mult = requant[2 * h], shift = requant[2 * h + 1];
        if (mult < 1 || mult > 4096 || shift < 1 || shift > 24) return ORACLE_E_ARG;
        const int8_t *Q = q + bh * Lq * d, *K = k + bh * Lk * d;
        for (int64_t i = 0; i < Lq; ++i)
            for (int64_t j = 0; j < Lk; ++j) {
                int64_t acc = 0;
                for (int64_t t = 0; t < d; ++t) acc += (int64_t)Q[i * d + t] * (int64_t)K[j * d + t];
                int64_t prod = acc * mult + ((int64_t)1 << (shift - 1));
                int64_t two = (int64_t)1 << shift;
                int64_t y = prod / two;
                if (prod % two != 0 && prod < 0) y -= 1;
                if (y < -128) y = -128;
                if (y > 127) y = 127;
                x[(bh * Lq + i) * Lk + j] = (int8_t)y;
            }
    }
    return ORACLE_OK;
}

/* rho of Eq. (8) for an array of row sums: used by the exhaustive check that
 * rho*Z <= 255*2^15 < (rho+1)*Z for every admissible Z. */
int hccs_oracle_reciprocal_u8(const int64_t *Z, int64_t *rho, int64_t count)
{
    if (!Z || !rho) return ORACLE_E_ARG;
    for (int64_t i = 0; i < count; ++i) {
        if (Z[i] < 1) return ORACLE_E_ARG;
        rho[i] = (((int64_t)255) << INV_SHIFT) / Z[i];
    }
    return ORACLE_OK;
}

/* Offline calibration objective, Sec. III-C Eq. (10), evaluated by brute force.
 * For head h and candidate c = (B, S, Dmax):
 *   J[h][c] = mean over the rows r of head h of  KL( softmax(alpha_h * x_r) || q_r ),
 *   q_r[i]  = phat_r[i] / sum_j phat_r[j],  phat_r the 16-bit HCCS output of row r
 *             (Alg. 1 as printed: the paper asks for the divergence "in the int16 space").
 * alpha_h turns an int8 logit into a real one (the paper does not name the dequantisation
 * scale; it is an input here).  The softmax and the divergence are in double precision,
 * KL = sum_i P_i (log P_i - log q_i), terms with P_i = 0 contribute nothing.
 * Candidates that are not admissible under the strict band (Sec. IV-C) get +infinity.
 * objective: H*nc doubles; best[h] = the first index attaining the minimum, or -1 if no
 * candidate is admissible. */
int hccs_oracle_calibrate(const int8_t *logits, int64_t Bt, int64_t H, int64_t Lq, int64_t Lk,
                          const double *alpha, const int32_t *cand, int64_t nc, double *objective,
                          int32_t *best, int threads)
{
    if (!logits || !alpha || !cand || !objective || !best) return ORACLE_E_ARG;
    if (Bt < 1 || H < 1 || Lq < 1 || Lk < 1 || nc < 1) return ORACLE_E_ARG;
    int status = ORACLE_OK;
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(dynamic, 1)
    for (int64_t hc = 0; hc < H * nc; ++hc) {
        const int64_t h = hc / nc, c = hc % nc;
        const int64_t B = cand[3 * c], S = cand[3 * c + 1], D = cand[3 * c + 2];
        if (hccs_oracle_check_params(B, S, D, Lk, 1) != ORACLE_OK) {
            objective[hc] = INFINITY;
            continue;
        }
        double *P = (double *)malloc((size_t)Lk * sizeof(double));
        uint16_t *ph = (uint16_t *)malloc((size_t)Lk * sizeof(uint16_t));
        double total = 0.0;
        for (int64_t b = 0; b < Bt; ++b)
            for (int64_t qi = 0; qi < Lq; ++qi) {
                const int8_t *x = logits + (((b * H + h) * Lq) + qi) * Lk;
                int64_t m = x[0];
                for (int64_t i = 1; i < Lk; ++i)
                    if (x[i] > m) m = x[i];
                double den = 0.0;
                for (int64_t i = 0; i < Lk; ++i) {
                    P[i] = exp(alpha[h] * (double)((int64_t)x[i] - m));
                    den += P[i];
                }
                int rc = hccs_oracle_row_i16(x, Lk, B, S, D, ph, 0, 0);
                if (rc != ORACLE_OK) {
#pragma omp critical
                    status = rc;
                    continue;
                }
                int64_t sum = 0;
                for (int64_t i = 0; i < Lk; ++i) sum += ph[i];
                double kl = 0.0;
                for (int64_t i = 0; i < Lk; ++i) {
                    const double p = P[i] / den;
                    if (p > 0.0) kl += p * (log(p) - log((double)ph[i] / (double)sum));
                }
                total += kl;
            }
        objective[hc] = total / (double)(Bt * Lq);
        free(P);
        free(ph);
    }
    for (int64_t h = 0; h < H; ++h) {
        best[h] = -1;
        for (int64_t c = 0; c < nc; ++c)
            if (isfinite(objective[h * nc + c]) && (best[h] < 0 || objective[h * nc + c] < objective[h * nc + best[h]]))
                best[h] = (int32_t)c;
    }
    return status;
}
