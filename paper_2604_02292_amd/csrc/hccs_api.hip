// C ABI of the library (see include/hccs.h and include/hccs_testing.h): argument checks, the
// admissibility test of Sec. IV-C, and hand-off to the kernel launchers.  Host code only.
#include <hip/hip_runtime.h>

#include "hccs_device.h"
#include "../../include/hccs_testing.h"

namespace hccs {
hipError_t launch_softmax(const int8_t *x, void *out, int64_t Bt, int H, int Lq, int Lk, const HeadTable &tab,
                          int mode, bool vector_ok, hipStream_t st);
hipError_t launch_reciprocal(const uint32_t *z, uint32_t *rho, int64_t count, hipStream_t st);
hipError_t launch_copy(const void *src, void *dst, int64_t bytes, hipStream_t st);
hipError_t launch_normalise_table(const int32_t *bsdz, uint8_t *out, int64_t count, hipStream_t st);
bool attention_is_resident(int Lq, int Lk);   // head size 64
hipError_t launch_attention(const int8_t *q, const int8_t *k, const int8_t *v, int32_t *o, int64_t Bt, int H, int Lq, int L,
                            int d, const HeadTable &tab, const RequantTable &rq, hipStream_t st);
hipError_t launch_attention_stream(const int8_t *q, const int8_t *k, const int8_t *v, int32_t *o, int64_t Bt, int H,
                                   int Lq, int Lk, int d, const HeadTable &tab, const RequantTable &rq,
                                   hipStream_t st);
int64_t calibrate_workspace_bytes(int64_t Bt, int64_t H, int64_t Lq);
hipError_t launch_calibrate(const int8_t *logits, int Bt, int H, int Lq, int Lk, const double *alpha,
                            const hccs_head_params *cand, int nc, double *objective, int32_t *best, void *workspace,
                            hipStream_t st);
hipError_t static_scratch(void **ptr);
hipError_t launch_exp_softmax(const int8_t *x, uint8_t *p, int64_t Bt, int H, int Lq, int Lk, const float *scale,
                              hipStream_t st);
}  // namespace hccs

namespace {

// One head against one band, Sec. IV-C.  64-bit products: n*B can pass 2^31.
int check_head(const hccs_head_params &hp, int64_t n, int band)
{
    const int64_t B = hp.B, S = hp.S, D = hp.Dmax;
    if (D < 0 || D > 127) return HCCS_E_PARAM_RANGE;
    if (S < 0 || S > 127) return HCCS_E_PARAM_RANGE;
    if (B < 1 || B > 32767) return HCCS_E_PARAM_RANGE;
    if (B - S * D < 0) return HCCS_E_PARAM_RANGE;
    if (n * (B - S * D) < 256) return HCCS_E_PARAM_FLOOR;
    const int64_t ceiling = (band == HCCS_BAND_STRICT) ? 32767 : (int64_t)hccs::kRecipNumerator;
    if (n * B > ceiling) return HCCS_E_PARAM_CEIL;
    return HCCS_OK;
}

bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

// rows = B*H*Lq must stay below 2^31: row and block numbers are 32-bit in the kernels
bool rows_fit(int64_t B, int64_t H, int64_t Lq) { return B * H * Lq < ((int64_t)1 << 31); }

int fill_table(const hccs_head_params *table_host, int H, hccs::HeadTable &out)
{
    for (int h = 0; h < H; ++h) out.e[h] = make_int4(table_host[h].B, table_host[h].S, table_host[h].Dmax, 0);
    for (int h = H; h < HCCS_MAX_HEADS; ++h) out.e[h] = make_int4(0, 0, 0, 0);
    return HCCS_OK;
}

}  // namespace

extern "C" {

int hccs_validate_params(const hccs_head_params *table_host, int32_t H, int32_t n, int32_t band,
                         int32_t *first_bad_head)
{
    if (first_bad_head) *first_bad_head = -1;
    if (!table_host) return HCCS_E_NULL;
    if (H < 1 || n < 1 || n > HCCS_MAX_ROW_LENGTH) return HCCS_E_SHAPE;
    if (band != HCCS_BAND_U8 && band != HCCS_BAND_STRICT) return HCCS_E_SCALE;
    for (int h = 0; h < H; ++h) {
        const int rc = check_head(table_host[h], n, band);
        if (rc != HCCS_OK) {
            if (first_bad_head) *first_bad_head = h;
            return rc;
        }
    }
    return HCCS_OK;
}

int hccs_calibrated_softmax_i8_ex(const int8_t *logits_dev, void *out_dev, int32_t B, int32_t H, int32_t Lq,
                                  int32_t Lk, const hccs_head_params *table_host, int32_t out_scale_T,
                                  int32_t reciprocal, int32_t band, void *hip_stream)
{
    if (!table_host) return HCCS_E_NULL;
    if (B < 0 || H < 1 || H > HCCS_MAX_HEADS || Lq < 0 || Lk < 1 || Lk > HCCS_MAX_ROW_LENGTH || !rows_fit(B, H, Lq))
        return HCCS_E_SHAPE;
    if (out_scale_T != 255 && out_scale_T != 32767) return HCCS_E_SCALE;
    if (reciprocal != HCCS_RECIP_EXACT && reciprocal != HCCS_RECIP_CLB) return HCCS_E_SCALE;
    if (band != HCCS_BAND_U8 && band != HCCS_BAND_STRICT) return HCCS_E_SCALE;
    const bool wide = (out_scale_T == 32767);
    // the 16-bit path needs Z <= 32767 whatever band the caller named (Sec. IV-C, last item)
    const int rc = hccs_validate_params(table_host, H, Lk, wide ? HCCS_BAND_STRICT : band, nullptr);
    if (rc != HCCS_OK) return rc;
    if (B == 0 || Lq == 0) return HCCS_OK;
    if (!logits_dev || !out_dev) return HCCS_E_NULL;
    const uint64_t in_bytes = (uint64_t)B * H * Lq * Lk, out_bytes = in_bytes * (wide ? 2 : 1);
    const uintptr_t a = (uintptr_t)logits_dev, b = (uintptr_t)out_dev;
    const bool same = (a == b) && !wide;                       // in place: 8-bit modes only
    if (!same && a < b + out_bytes && b < a + in_bytes) return HCCS_E_ALIGN;   // overlapping buffers
    if (wide && (b & 1u)) return HCCS_E_ALIGN;
    hccs::HeadTable tab;
    fill_table(table_host, H, tab);
    const int mode = (wide ? 1 : 0) | (reciprocal == HCCS_RECIP_CLB ? 2 : 0);
    const bool vector_ok = aligned16(logits_dev) && aligned16(out_dev);
    const hipError_t e =
        hccs::launch_softmax(logits_dev, out_dev, B, H, Lq, Lk, tab, mode, vector_ok, (hipStream_t)hip_stream);
    return e == hipSuccess ? HCCS_OK : HCCS_E_HIP;
}

int hccs_calibrated_softmax_i8(const int8_t *logits_dev, uint8_t *probs_dev, int32_t B, int32_t H, int32_t Lq,
                               int32_t Lk, const hccs_head_params *table_host, int32_t out_scale_T, int32_t band,
                               void *hip_stream)
{
    if (out_scale_T != 255) return HCCS_E_SCALE;
    return hccs_calibrated_softmax_i8_ex(logits_dev, probs_dev, B, H, Lq, Lk, table_host, 255, HCCS_RECIP_EXACT,
                                         band, hip_stream);
}

int hccs_attention_i8_ex(const int8_t *q_dev, const int8_t *k_dev, const int8_t *v_dev, int32_t *o_dev, int32_t B,
                         int32_t H, int32_t Lq, int32_t Lk, int32_t d, const hccs_head_params *table_host,
                         const hccs_requant *requant_host, int32_t out_scale_T, int32_t band, void *hip_stream)
{
    if (!table_host || !requant_host) return HCCS_E_NULL;
    if (B < 0 || H < 1 || H > HCCS_MAX_HEADS) return HCCS_E_SHAPE;
    if ((d != 64 && d != 128) || Lq < 0 || Lk < 1 || Lk > HCCS_MAX_ROW_LENGTH) return HCCS_E_SHAPE;
    if (!rows_fit(B, H, Lq > 0 ? Lq : 1)) return HCCS_E_SHAPE;
    if (out_scale_T != 255) return HCCS_E_SCALE;
    const int rc = hccs_validate_params(table_host, H, Lk, band, nullptr);
    if (rc != HCCS_OK) return rc;
    for (int h = 0; h < H; ++h) {
        if (requant_host[h].mult < 1 || requant_host[h].mult > 4096) return HCCS_E_REQUANT;
        if (requant_host[h].shift < 1 || requant_host[h].shift > 24) return HCCS_E_REQUANT;
    }
    if (B == 0 || Lq == 0) return HCCS_OK;
    if (!q_dev || !k_dev || !v_dev || !o_dev) return HCCS_E_NULL;
    if (!aligned16(q_dev) || !aligned16(k_dev) || !aligned16(v_dev) || !aligned16(o_dev)) return HCCS_E_ALIGN;
    hccs::HeadTable tab;
    fill_table(table_host, H, tab);
    hccs::RequantTable rq;
    for (int h = 0; h < HCCS_MAX_HEADS; ++h)
        rq.e[h] = h < H ? make_int4(requant_host[h].mult, requant_host[h].shift, 0, 0) : make_int4(1, 1, 0, 0);
    // Blocks whose keys fit LDS go to the resident kernels, everything else streams
    const bool resident = d == 64 && hccs::attention_is_resident(Lq, Lk);
    const hipError_t e =
        resident ? hccs::launch_attention(q_dev, k_dev, v_dev, o_dev, B, H, Lq, Lk, d, tab, rq, (hipStream_t)hip_stream)
                 : hccs::launch_attention_stream(q_dev, k_dev, v_dev, o_dev, B, H, Lq, Lk, d, tab, rq,
                                                 (hipStream_t)hip_stream);
    return e == hipSuccess ? HCCS_OK : HCCS_E_HIP;
}

int hccs_attention_i8(const int8_t *q_dev, const int8_t *k_dev, const int8_t *v_dev, int32_t *o_dev, int32_t B,
                      int32_t H, int32_t L, int32_t d, const hccs_head_params *table_host,
                      const hccs_requant *requant_host, int32_t out_scale_T, int32_t band, void *hip_stream)
{
    return hccs_attention_i8_ex(q_dev, k_dev, v_dev, o_dev, B, H, L, L, d, table_host, requant_host, out_scale_T,
                                band, hip_stream);
}

int64_t hccs_calibrate_workspace_bytes(int32_t B, int32_t H, int32_t Lq, int32_t Lk)
{
    if (B < 1 || H < 1 || H > HCCS_MAX_HEADS || Lq < 1 || Lk < 1 || Lk > HCCS_MAX_ROW_LENGTH || !rows_fit(B, H, Lq))
        return HCCS_E_SHAPE;
    return hccs::calibrate_workspace_bytes(B, H, Lq);
}

int hccs_calibrate_grid(const int8_t *logits_dev, int32_t B, int32_t H, int32_t Lq, int32_t Lk,
                        const double *alpha_host, const hccs_head_params *candidates_dev, int32_t n_candidates,
                        double *objective_dev, int32_t *best_dev, void *workspace_dev, int64_t workspace_bytes,
                        void *hip_stream)
{
    if (!alpha_host) return HCCS_E_NULL;
    const int64_t need = hccs_calibrate_workspace_bytes(B, H, Lq, Lk);
    if (need < 0) return HCCS_E_SHAPE;
    if (n_candidates < 1 || n_candidates > 65535) return HCCS_E_SHAPE;
    for (int h = 0; h < H; ++h)
        if (!(alpha_host[h] > 0.0) || !(alpha_host[h] < 1e6)) return HCCS_E_SCALE;
    if (!logits_dev || !candidates_dev || !objective_dev || !best_dev || !workspace_dev) return HCCS_E_NULL;
    if (workspace_bytes < need) return HCCS_E_SHAPE;
    if (((uintptr_t)workspace_dev & 7u) || ((uintptr_t)objective_dev & 7u) || ((uintptr_t)best_dev & 3u) ||
        ((uintptr_t)candidates_dev & 3u))
        return HCCS_E_ALIGN;
    const hipError_t e = hccs::launch_calibrate(logits_dev, B, H, Lq, Lk, alpha_host, candidates_dev, n_candidates,
                                                objective_dev, best_dev, workspace_dev, (hipStream_t)hip_stream);
    return e == hipSuccess ? HCCS_OK : HCCS_E_HIP;
}

int hccs_calibrate_grid_static(const int8_t *logits_dev, int32_t B, int32_t H, int32_t Lq, int32_t Lk,
                               const double *alpha_host, const hccs_head_params *candidates_dev, int32_t n_candidates,
                               double *objective_dev, int32_t *best_dev, void *hip_stream)
{
    const int64_t need = hccs_calibrate_workspace_bytes(B, H, Lq, Lk);
    if (need < 0) return HCCS_E_SHAPE;
    if (need > (int64_t)HCCS_STATIC_SCRATCH_BYTES) return HCCS_E_SCRATCH;
    void *scratch_dev = nullptr;
    if (hccs::static_scratch(&scratch_dev) != hipSuccess) return HCCS_E_HIP;
    return hccs_calibrate_grid(logits_dev, B, H, Lq, Lk, alpha_host, candidates_dev, n_candidates, objective_dev,
                               best_dev, scratch_dev, (int64_t)HCCS_STATIC_SCRATCH_BYTES, hip_stream);
}

int hccs_exp_softmax_i8_f32(const int8_t *logits_dev, uint8_t *probs_dev, int32_t B, int32_t H, int32_t Lq,
                            int32_t Lk, const float *scale_host, void *hip_stream)
{
    if (!scale_host) return HCCS_E_NULL;
    if (B < 0 || H < 1 || H > HCCS_MAX_HEADS || Lq < 0 || Lk < 16 || Lk > 16384 || Lk % 16 != 0 || !rows_fit(B, H, Lq))
        return HCCS_E_SHAPE;
    if (B == 0 || Lq == 0) return HCCS_OK;
    if (!logits_dev || !probs_dev) return HCCS_E_NULL;
    if (!aligned16(logits_dev) || !aligned16(probs_dev)) return HCCS_E_ALIGN;
    const hipError_t e =
        hccs::launch_exp_softmax(logits_dev, probs_dev, B, H, Lq, Lk, scale_host, (hipStream_t)hip_stream);
    return e == hipSuccess ? HCCS_OK : HCCS_E_HIP;
}

int hccs_reciprocal_u8(const uint32_t *z_dev, uint32_t *rho_dev, int64_t count, void *hip_stream)
{
    if (count < 0) return HCCS_E_SHAPE;
    if (count == 0) return HCCS_OK;
    if (!z_dev || !rho_dev) return HCCS_E_NULL;
    const hipError_t e = hccs::launch_reciprocal(z_dev, rho_dev, count, (hipStream_t)hip_stream);
    return e == hipSuccess ? HCCS_OK : HCCS_E_HIP;
}

int hccs_normalise_table_u8(const int32_t *bsdz_dev, uint8_t *out_dev, int64_t count, void *hip_stream)
{
    if (count < 0 || count > 0x7fffffff) return HCCS_E_SHAPE;
    if (count == 0) return HCCS_OK;
    if (!bsdz_dev || !out_dev) return HCCS_E_NULL;
    if (!aligned16(bsdz_dev) || ((uintptr_t)out_dev & 3u)) return HCCS_E_ALIGN;
    const hipError_t e = hccs::launch_normalise_table(bsdz_dev, out_dev, count, (hipStream_t)hip_stream);
    return e == hipSuccess ? HCCS_OK : HCCS_E_HIP;
}

int hccs_largest_probability_u8(const int32_t *params_host, int32_t H, int32_t n, int32_t *bound_host)
{
    if (!params_host || !bound_host) return HCCS_E_NULL;
    if (H < 1 || H > HCCS_MAX_HEADS || n < 1) return HCCS_E_SHAPE;
    for (int h = 0; h < H; ++h)
        bound_host[h] = (int32_t)hccs::largest_probability(params_host[3 * h], params_host[3 * h + 1],
                                                           params_host[3 * h + 2], n);
    return HCCS_OK;
}

int hccs_copy_bytes(const void *src_dev, void *dst_dev, int64_t bytes, void *hip_stream)
{
    if (bytes < 0 || bytes % 16 != 0) return HCCS_E_SHAPE;
    if (bytes == 0) return HCCS_OK;
    if (!src_dev || !dst_dev) return HCCS_E_NULL;
    if (!aligned16(src_dev) || !aligned16(dst_dev)) return HCCS_E_ALIGN;
    const hipError_t e = hccs::launch_copy(src_dev, dst_dev, bytes, (hipStream_t)hip_stream);
    return e == hipSuccess ? HCCS_OK : HCCS_E_HIP;
}

const char *hccs_status_string(int status)
{
    switch (status) {
        case HCCS_OK: return "ok";
        case HCCS_E_NULL: return "a required pointer is NULL";
        case HCCS_E_SHAPE: return "a dimension is outside the supported range";
        case HCCS_E_ALIGN: return "a device pointer is misaligned or buffers partially overlap";
        case HCCS_E_SCALE: return "unsupported output scale, reciprocal kind or band";
        case HCCS_E_PARAM_RANGE: return "head constants out of range (Dmax, S, B, or B - S*Dmax < 0)";
        case HCCS_E_PARAM_FLOOR: return "n*(B - S*Dmax) < 256: row sum could fall below 256";
        case HCCS_E_PARAM_CEIL: return "n*B exceeds the ceiling of the chosen band";
        case HCCS_E_HIP: return "the HIP runtime reported an error at launch";
        case HCCS_E_REQUANT: return "requantisation multiplier or shift out of range";
        case HCCS_E_SCRATCH: return "the problem needs more work memory than the library's static buffer holds";
        default: return "unknown status";
    }
}

}  // extern "C"
