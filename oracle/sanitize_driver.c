/*
 * Command-line front end of the HCCS oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Linked with hccs_oracle.c into one executable that the test suite builds with
 * -fsanitize=address,undefined, so that the oracle's own memory accesses and integer
 * arithmetic are checked by the sanitizers while it computes the pinned cases.  This file
 * holds no arithmetic of the method: it reads a request, calls one oracle function on
 * heap buffers of exactly the documented sizes (so an access one element past an end is
 * caught), and writes the result.
 *
 *   sanitize_driver request.bin reply.bin
 *
 * request: 12 int64 {op, Bt, H, Lq, Lk, d, band, mode, threads, nc, 0, 0}, then the
 * operation's arrays in the order listed at each case below.
 * reply: int64 status, then the operation's outputs.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int hccs_oracle_check_params(int64_t B, int64_t S, int64_t D, int64_t n, int band);
int hccs_oracle_row_u8(const int8_t *, int64_t, int64_t, int64_t, int64_t, uint8_t *, int64_t *, int64_t *);
int hccs_oracle_row_i16(const int8_t *, int64_t, int64_t, int64_t, int64_t, uint16_t *, int64_t *, int64_t *);
int hccs_oracle_row_clb_u8(const int8_t *, int64_t, int64_t, int64_t, int64_t, uint8_t *, int64_t *, int64_t *);
int hccs_oracle_row_clb_i16(const int8_t *, int64_t, int64_t, int64_t, int64_t, uint16_t *, int64_t *, int64_t *);
int hccs_oracle_softmax(const int8_t *, void *, int64_t, int64_t, int64_t, int64_t, const int32_t *, int, int, int);
int hccs_oracle_attention_i8(const int8_t *, const int8_t *, const int8_t *, int32_t *, int64_t, int64_t, int64_t,
                             int64_t, int64_t, const int32_t *, const int32_t *, int, int);
int hccs_oracle_requant_logits(const int8_t *, const int8_t *, int8_t *, int64_t, int64_t, int64_t, int64_t, int64_t,
                               const int32_t *);
int hccs_oracle_reciprocal_u8(const int64_t *, int64_t *, int64_t);
int hccs_oracle_calibrate(const int8_t *, int64_t, int64_t, int64_t, int64_t, const double *, const int32_t *,
                          int64_t, double *, int32_t *, int);

static FILE *in, *out;

static void *get(size_t bytes)
{
    void *p = malloc(bytes ? bytes : 1);
    if (!p || (bytes && fread(p, 1, bytes, in) != bytes)) {
        fprintf(stderr, "sanitize_driver: short request\n");
        exit(2);
    }
    return p;
}

static void put(const void *p, size_t bytes)
{
    if (bytes && fwrite(p, 1, bytes, out) != bytes) exit(2);
}

int main(int argc, char **argv)
{
    if (argc != 3) return 2;
    in = fopen(argv[1], "rb");
    out = fopen(argv[2], "wb");
    if (!in || !out) return 2;
    int64_t *h = (int64_t *)get(12 * sizeof(int64_t));
    const int64_t op = h[0], Bt = h[1], H = h[2], Lq = h[3], Lk = h[4], d = h[5], nc = h[9];
    const int band = (int)h[6], mode = (int)h[7], threads = (int)h[8];
    int64_t rc = 0;
    switch (op) {
        case 1: {   /* softmax: table int32[3H], logits int8[Bt*H*Lq*Lk] -> out (1 or 2 bytes each) */
            const size_t count = (size_t)(Bt * H * Lq * Lk), width = (mode & 1) ? 2 : 1;
            int32_t *table = (int32_t *)get((size_t)H * 3 * 4);
            int8_t *x = (int8_t *)get(count);
            void *p = calloc(count ? count : 1, width);
            rc = hccs_oracle_softmax(x, p, Bt, H, Lq, Lk, table, band, mode, threads);
            put(&rc, 8), put(p, count * width);
            free(table), free(x), free(p);
            break;
        }
        case 2: {   /* attention: table, requant int32[2H], q int8[Bt*H*Lq*d], k, v int8[Bt*H*Lk*d] -> o int32 */
            const size_t nq = (size_t)(Bt * H * Lq * d), nk = (size_t)(Bt * H * Lk * d);
            int32_t *table = (int32_t *)get((size_t)H * 3 * 4), *rq = (int32_t *)get((size_t)H * 2 * 4);
            int8_t *q = (int8_t *)get(nq), *k = (int8_t *)get(nk), *v = (int8_t *)get(nk);
            int32_t *o = (int32_t *)calloc(nq ? nq : 1, 4);
            rc = hccs_oracle_attention_i8(q, k, v, o, Bt, H, Lq, Lk, d, table, rq, band, threads);
            put(&rc, 8), put(o, nq * 4);
            free(table), free(rq), free(q), free(k), free(v), free(o);
            break;
        }
        case 3: {   /* requantised logits: requant, q, k -> x int8[Bt*H*Lq*Lk] */
            const size_t nq = (size_t)(Bt * H * Lq * d), nk = (size_t)(Bt * H * Lk * d);
            const size_t nx = (size_t)(Bt * H * Lq * Lk);
            int32_t *rq = (int32_t *)get((size_t)H * 2 * 4);
            int8_t *q = (int8_t *)get(nq), *k = (int8_t *)get(nk);
            int8_t *x = (int8_t *)calloc(nx ? nx : 1, 1);
            rc = hccs_oracle_requant_logits(q, k, x, Bt, H, Lq, Lk, d, rq);
            put(&rc, 8), put(x, nx);
            free(rq), free(q), free(k), free(x);
            break;
        }
        case 4: {   /* reciprocal: Z int64[nc] -> rho int64[nc] */
            int64_t *Z = (int64_t *)get((size_t)nc * 8), *rho = (int64_t *)calloc((size_t)(nc ? nc : 1), 8);
            rc = hccs_oracle_reciprocal_u8(Z, rho, nc);
            put(&rc, 8), put(rho, (size_t)nc * 8);
            free(Z), free(rho);
            break;
        }
        case 5: {   /* calibration: alpha double[H], candidates int32[3nc], logits -> objective double[H*nc], best int32[H] */
            const size_t count = (size_t)(Bt * H * Lq * Lk);
            double *alpha = (double *)get((size_t)H * 8);
            int32_t *cand = (int32_t *)get((size_t)nc * 3 * 4);
            int8_t *x = (int8_t *)get(count);
            double *obj = (double *)calloc((size_t)(H * nc), 8);
            int32_t *best = (int32_t *)calloc((size_t)H, 4);
            rc = hccs_oracle_calibrate(x, Bt, H, Lq, Lk, alpha, cand, nc, obj, best, threads);
            put(&rc, 8), put(obj, (size_t)(H * nc) * 8), put(best, (size_t)H * 4);
            free(alpha), free(cand), free(x), free(obj), free(best);
            break;
        }
        case 6: {   /* one row of length Lk: params int32[3], x int8[Lk] -> Z, rho (int64), p */
            int32_t *t = (int32_t *)get(3 * 4);
            int8_t *x = (int8_t *)get((size_t)Lk);
            const size_t width = (mode & 1) ? 2 : 1;
            void *p = calloc((size_t)(Lk ? Lk : 1), width);
            int64_t Z = 0, rho = 0;
            if (mode == 0) rc = hccs_oracle_row_u8(x, Lk, t[0], t[1], t[2], (uint8_t *)p, &Z, &rho);
            else if (mode == 1) rc = hccs_oracle_row_i16(x, Lk, t[0], t[1], t[2], (uint16_t *)p, &Z, &rho);
            else if (mode == 2) rc = hccs_oracle_row_clb_u8(x, Lk, t[0], t[1], t[2], (uint8_t *)p, &Z, &rho);
            else rc = hccs_oracle_row_clb_i16(x, Lk, t[0], t[1], t[2], (uint16_t *)p, &Z, &rho);
            put(&rc, 8), put(&Z, 8), put(&rho, 8), put(p, (size_t)Lk * width);
            free(t), free(x), free(p);
            break;
        }
        case 7:     /* admissibility of (B, S, D) = (Bt, H, Lq) for rows of length Lk */
            rc = hccs_oracle_check_params(Bt, H, Lq, Lk, band);
            put(&rc, 8);
            break;
        default: return 2;
    }
    free(h);
    fclose(in);
    return fclose(out) == 0 ? 0 : 2;
}
