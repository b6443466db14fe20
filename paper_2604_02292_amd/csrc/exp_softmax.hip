// Comparison kernel, benchmarks only: exact-exponential float32 softmax of int8
// logits, out = rint(255 * softmax(scale_h * x)), written with the same lane-group
// layout and the same 1 byte in / 1 byte out traffic as the HCCS kernel so that
// the two differ in arithmetic only.  Not part of the method, never parity-checked.
#include "hccs_device.h"

namespace hccs {

struct ScaleTable {
    float e[HCCS_MAX_HEADS];
};

template <int G, int V>
__global__ __launch_bounds__(256) void exp_softmax_kernel(const int8_t *__restrict__ logits,
                                                          uint8_t *__restrict__ probs, int Lq, int n16,
                                                          BlockPlace place, ScaleTable scale)
{
    constexpr int kRowsPerWave = 64 / G;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % G, grp = lane / G;
    uint32_t tile, head, slab_no;   // the same linear launch as the HCCS kernel
    place.locate(tile, head, slab_no);
    const float c = scale.e[head] * 1.44269504088896f;   // exp(s*x) = exp2(s*log2(e)*x)
    const int n = n16 * 16;
    const size_t slab = (size_t)slab_no * (size_t)Lq;
    const int row = ((int)tile * 4 + wave) * kRowsPerWave + grp;
    const bool live = row < Lq;
    const int8_t *src = logits + (slab + row) * (size_t)n;
    uint8_t *dst = probs + (slab + row) * (size_t)n;

    u32x4 d[V];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int vi = v * G + sub;
        d[v] = (live && vi < n16) ? load_stream(src + vi * 16) : (u32x4){kPadWord, kPadWord, kPadWord, kPadWord};
    }
    ByteMax bm;
    bm.init(d[0][0]);
    bm.add(d[0][1]);
    bm.add(d[0][2]);
    bm.add(d[0][3]);
#pragma unroll
    for (int v = 1; v < V; ++v) {
#pragma unroll
        for (int cidx = 0; cidx < 4; ++cidx) bm.add(d[v][cidx]);
    }
    const int m = group_max<G>(bm.result());
    const float fm = (float)m;

    float sum = 0.f;
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const bool ok = (v * G + sub) < n16;
#pragma unroll
        for (int cidx = 0; cidx < 4; ++cidx)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const float x = (float)(int8_t)(d[v][cidx] >> (8 * b));
                const float e = __builtin_amdgcn_exp2f((x - fm) * c);
                sum += ok ? e : 0.f;
            }
    }
    // float all-reduce over the lane group, same pairing as the integer helpers
    sum += __builtin_bit_cast(float, dpp<0xB1>(__builtin_bit_cast(int, sum)));
    sum += __builtin_bit_cast(float, dpp<0x4E>(__builtin_bit_cast(int, sum)));
    if constexpr (G >= 8) sum += __builtin_bit_cast(float, dpp<0x141>(__builtin_bit_cast(int, sum)));
    if constexpr (G >= 16) sum += __builtin_bit_cast(float, dpp<0x140>(__builtin_bit_cast(int, sum)));
    if constexpr (G >= 32) sum += __builtin_bit_cast(float, xor16(__builtin_bit_cast(int, sum)));
    if constexpr (G >= 64) sum += __builtin_bit_cast(float, xor32(__builtin_bit_cast(int, sum)));
    const float inv = 255.0f * __builtin_amdgcn_rcpf(sum);

#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int vi = v * G + sub;
#pragma unroll
        for (int cidx = 0; cidx < 4; ++cidx) {
            uint32_t out = 0;
            const uint32_t word = d[v][cidx];
            out = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_exp2f(((float)(int8_t)(word)-fm) * c) * inv, 0, out);
            out = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_exp2f(((float)(int8_t)(word >> 8) - fm) * c) * inv, 1, out);
            out = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_exp2f(((float)(int8_t)(word >> 16) - fm) * c) * inv, 2, out);
            out = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_exp2f(((float)(int8_t)(word >> 24) - fm) * c) * inv, 3, out);
            d[v][cidx] = out;
        }
        if (live && vi < n16) store_stream(dst + vi * 16, d[v]);
    }
}

template <int G, int V>
static hipError_t launch_exp(const int8_t *x, uint8_t *p, int64_t Bt, int H, int Lq, int n16, const ScaleTable &sc,
                             hipStream_t st)
{
    constexpr int kRowsPerBlock = 4 * (64 / G);
    dim3 grid;
    const BlockPlace place = place_blocks((Lq + kRowsPerBlock - 1) / kRowsPerBlock, H, Bt, grid);
    return launch(exp_softmax_kernel<G, V>, grid, dim3(256), st, x, p, Lq, n16, place, sc);
}

hipError_t launch_exp_softmax(const int8_t *x, uint8_t *p, int64_t Bt, int H, int Lq, int Lk, const float *scale,
                              hipStream_t st)
{
    ScaleTable sc;
    for (int h = 0; h < HCCS_MAX_HEADS; ++h) sc.e[h] = h < H ? scale[h] : 0.f;
    const int n16 = Lk / 16;
    if (n16 <= 4) return launch_exp<4, 1>(x, p, Bt, H, Lq, n16, sc, st);
    if (n16 <= 8) return launch_exp<8, 1>(x, p, Bt, H, Lq, n16, sc, st);
    if (n16 <= 16) return launch_exp<16, 1>(x, p, Bt, H, Lq, n16, sc, st);
    if (n16 <= 32) return launch_exp<16, 2>(x, p, Bt, H, Lq, n16, sc, st);
    if (n16 <= 64) return launch_exp<64, 1>(x, p, Bt, H, Lq, n16, sc, st);
    if (n16 <= 128) return launch_exp<64, 2>(x, p, Bt, H, Lq, n16, sc, st);
    if (n16 <= 256) return launch_exp<64, 4>(x, p, Bt, H, Lq, n16, sc, st);
    if (n16 <= 512) return launch_exp<64, 8>(x, p, Bt, H, Lq, n16, sc, st);
    return launch_exp<64, 16>(x, p, Bt, H, Lq, n16, sc, st);
}

}  // namespace hccs
