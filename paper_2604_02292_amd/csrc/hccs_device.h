// Device-side building blocks shared by the HCCS kernels (gfx950, wave64).
//
// Everything the method computes is integer arithmetic (Alg. 1; Eq. (2), (3),
// (5), (8)); the few float instructions used below are exact on the operand
// ranges the admissibility band guarantees, and each such use says why.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>
#include <utility>

#include "../../include/hccs.h"

namespace hccs {

constexpr uint32_t kRecipNumerator = 255u << 15;  // numerator of Eq. (8), R = 15

// Per-head constants carried by value in the kernel arguments, one int4 per
// head: (B, S, Dmax, unused).  A block works on rows of one head, so the entry
// is fetched with scalar loads.
struct HeadTable {
    int4 e[HCCS_MAX_HEADS];
};

// Rescale rule of the fused block per head: (mult, shift, accumulator saturation bounds lo, hi).
struct RequantTable {
    int4 e[HCCS_MAX_HEADS];
};

// 16 bytes of a row, as the hardware moves them (global_load/store_dwordx4).
// The loads and stores are marked non-temporal: every byte is touched once.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u32x4 load_stream(const void *p) { return __builtin_nontemporal_load((const u32x4 *)p); }
__device__ __forceinline__ void store_stream(void *p, u32x4 v) { __builtin_nontemporal_store(v, (u32x4 *)p); }
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x2 load_stream8(const void *p) { return __builtin_nontemporal_load((const u32x2 *)p); }
constexpr uint32_t kPadWord = 0x80808080u;   // four logits of -128

// ---- cross-lane movement -------------------------------------------------
// DPP controls: quad_perm[1,0,3,2] = 0xB1, quad_perm[2,3,0,1] = 0x4E,
// row_half_mirror = 0x141 (lane i <-> 7-i inside each 8), row_mirror = 0x140
// (i <-> 15-i inside each 16).  Applied in that order they pair every lane with
// one from the other half of a growing group, which is all an all-reduce of a
// commutative operation needs.
template <int CTRL>
__device__ __forceinline__ int dpp(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}

__device__ __forceinline__ int xor16(int v) { return __builtin_amdgcn_ds_swizzle(v, 0x401F); }
__device__ __forceinline__ int xor32(int v) { return __shfl_xor(v, 32); }

// All-reduce over aligned groups of G lanes (G a power of two, 4..64).
template <int G>
__device__ __forceinline__ int group_max(int v)
{
    v = max(v, dpp<0xB1>(v));
    v = max(v, dpp<0x4E>(v));
    if constexpr (G >= 8) v = max(v, dpp<0x141>(v));
    if constexpr (G >= 16) v = max(v, dpp<0x140>(v));
    if constexpr (G >= 32) v = max(v, xor16(v));
    if constexpr (G >= 64) v = max(v, xor32(v));
    return v;
}

template <int G>
__device__ __forceinline__ int group_sum(int v)
{
    v += dpp<0xB1>(v);
    v += dpp<0x4E>(v);
    if constexpr (G >= 8) v += dpp<0x141>(v);
    if constexpr (G >= 16) v += dpp<0x140>(v);
    if constexpr (G >= 32) v += xor16(v);
    if constexpr (G >= 64) v += xor32(v);
    return v;
}

// ---- exact integer division ------------------------------------------------
// floor(N / Z) for 1 <= Z <= N < 2^24 with a quotient below 2^16.  N and Z are
// exact in float, the hardware reciprocal is good to 1 ulp, so the truncated float
// quotient is within one of the true one; the remainder test repairs it in
// either direction, which makes the result the exact floor.
__device__ __forceinline__ uint32_t floor_div(uint32_t N, uint32_t Z)
{
    float qf = (float)N * __builtin_amdgcn_rcpf((float)Z);
    uint32_t q = (uint32_t)qf;
    int32_t rem = (int32_t)N - (int32_t)__umul24(q, Z);
    if (rem < 0) {
        q -= 1;
        rem += (int32_t)Z;
    }
    if (rem >= (int32_t)Z) q += 1;
    return q;
}

// The reciprocal of Eq. (8): rho = floor(255*2^15 / Z), 256 <= Z <= 255*2^15, so rho <= 32640.
__device__ __forceinline__ uint32_t reciprocal_u8(uint32_t Z) { return floor_div(kRecipNumerator, Z); }

// Output modes: scale T (Sec. III-B) x reciprocal kind.
enum : int {
    kModeU8 = 0,      // T = 255,   rho = floor(255*2^15 / Z), p = (s*rho) >> 15      Eq. (8)
    kModeI16 = 1,     // T = 32767, rho = floor(32767 / Z),    p = s*rho              Eq. (6), (7)
    kModeClbU8 = 2,   // T = 255,   rho = floor(255*2^15 / 2^k), k = floor(log2 Z), p saturated at 255   Eq. (9)
    kModeClbI16 = 3   // T = 32767, rho = floor(32767 / 2^k),  p saturated at 32767                      Eq. (9)
};

// rho for a mode.  Leading-bit modes replace the division by a shift taken from the
// position of the highest set bit of Z.
template <int MODE>
__device__ __forceinline__ uint32_t reciprocal_for_mode(uint32_t Z)
{
    if constexpr (MODE == kModeU8) return reciprocal_u8(Z);
    if constexpr (MODE == kModeI16) return floor_div(32767u, Z);
    const int k = 31 - __builtin_clz(Z);
    if constexpr (MODE == kModeClbU8) return kRecipNumerator >> k;
    return 32767u >> k;
}

// Scalar form of the last step for one score (used by the byte kernel and the
// leading-bit 8-bit path): s*rho stays below 2^24 in every mode.
template <int MODE>
__device__ __forceinline__ uint32_t scale_score(uint32_t s, uint32_t rho)
{
    const uint32_t prod = __umul24(s, rho);
    if constexpr (MODE == kModeU8) return prod >> 15;
    if constexpr (MODE == kModeI16) return prod;
    if constexpr (MODE == kModeClbU8) return min(prod >> 15, 255u);
    return min(prod, 32767u);
}

// ---- per-row constants of the normalise stage -----------------------------
// With delta the unclamped distance to the row maximum and pmin the output of a
// fully clamped element, the 8-bit output (Eq. (8)) of an element inside the
// window is
//     p = floor((B - S*delta) * rho / 2^15)
//       = pmin + floor(((B*rho - pmin*2^15) - (S*rho)*delta) / 2^15).
// B <= Z (the maximum itself scores B), so B*rho <= 255*2^15 < 2^23, S*rho <
// 2^23, and the bracket is an integer below 2^23 for delta <= Dmax: one float
// fma evaluates it exactly.  The pack instruction v_cvt_pk_u8_f32 rounds to
// nearest-even and saturates at 0 and 255, so the constant term carries
// -(1/2 - 2^-16): the fraction is a multiple of 2^-15, hence the shifted value
// never sits on a tie and rounds to the floor.  For delta > Dmax the bracket is
// below 2^15, the shifted value is below 1/2 and packs to 0, i.e. p = pmin:
// the clamp of Eq. (2) costs no instruction.
struct RowAffine {
    float slope;      // -(S*rho) / 2^15
    float offset;     // (2*(B*rho - pmin*2^15) - 32767) / 2^16
    uint32_t pmin4;   // pmin in each byte
};

__device__ __forceinline__ RowAffine row_affine(uint32_t Z, int B, int S, int D)
{
    const uint32_t rho = reciprocal_u8(Z);
    const uint32_t a = __umul24((uint32_t)S, rho);
    const uint32_t pmin = __umul24((uint32_t)(B - S * D), rho) >> 15;
    const uint32_t b0 = __umul24((uint32_t)B, rho) - (pmin << 15);
    RowAffine r;
    r.slope = -(float)a * 0x1p-15f;
    r.offset = (float)((int32_t)(2u * b0) - 32767) * 0x1p-16f;
    r.pmin4 = pmin * 0x01010101u;
    return r;
}

// Four distances (one per byte) -> four output bytes.
__device__ __forceinline__ uint32_t normalise4(uint32_t delta4, const RowAffine &r)
{
    uint32_t out = 0;
    out = __builtin_amdgcn_cvt_pk_u8_f32(fmaf((float)(delta4 & 0xffu), r.slope, r.offset), 0, out);
    out = __builtin_amdgcn_cvt_pk_u8_f32(fmaf((float)((delta4 >> 8) & 0xffu), r.slope, r.offset), 1, out);
    out = __builtin_amdgcn_cvt_pk_u8_f32(fmaf((float)((delta4 >> 16) & 0xffu), r.slope, r.offset), 2, out);
    out = __builtin_amdgcn_cvt_pk_u8_f32(fmaf((float)(delta4 >> 24), r.slope, r.offset), 3, out);
    return out + r.pmin4;  // p <= 255 in every byte, so no carry crosses bytes
}

// ---- byte-parallel helpers -------------------------------------------------
typedef short short2_t __attribute__((ext_vector_type(2)));

// Running signed maximum of the bytes of a dword stream, two 16-bit lanes at a
// time.  A signed 16-bit compare is decided by the high byte (the low byte only
// breaks ties), so feeding raw dwords tracks the odd bytes and feeding dwords
// shifted left by 8 tracks the even bytes; the result is read from the high
// bytes only.
struct ByteMax {
    short2_t odd, even;
    __device__ __forceinline__ void init(uint32_t v)
    {
        odd = __builtin_bit_cast(short2_t, v);
        even = __builtin_bit_cast(short2_t, v << 8);
    }
    __device__ __forceinline__ void add(uint32_t v)
    {
        odd = __builtin_elementwise_max(odd, __builtin_bit_cast(short2_t, v));
        even = __builtin_elementwise_max(even, __builtin_bit_cast(short2_t, v << 8));
    }
    // maximum as a signed value in [-128,127]
    __device__ __forceinline__ int result() const
    {
        short2_t m = __builtin_elementwise_max(odd, even);
        int hi = (int)m.y >> 8, lo = (int)m.x >> 8;
        return max(hi, lo);
    }
};

// Distances of four int8 logits to the row maximum, one per byte, unclamped.
// With the offset-binary form u = x + 128 the complement y = 255 - u is
// x ^ 0x7f, and delta = (m+128) - u = y - (127 - m); every byte of y is at
// least 127 - m, so one 32-bit subtraction does all four with no borrow.
__device__ __forceinline__ uint32_t distance4(uint32_t x4, uint32_t neg_base4)
{
    return (x4 ^ 0x7f7f7f7fu) + neg_base4;   // neg_base4 = -(127 - m) * 0x01010101
}

// ---- 16-bit packed arithmetic (two elements per instruction) -------------------
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));

// bytes (b0,b1) or (b2,b3) of a dword, zero-extended to two 16-bit lanes
__device__ __forceinline__ ushort2_t bytes_lo_pair(uint32_t w)
{
    return __builtin_bit_cast(ushort2_t, __builtin_amdgcn_perm(0u, w, 0x0c010c00u));
}
__device__ __forceinline__ ushort2_t bytes_hi_pair(uint32_t w)
{
    return __builtin_bit_cast(ushort2_t, __builtin_amdgcn_perm(0u, w, 0x0c030c02u));
}

// Scores of two elements from their unclamped distances: s = B - S*min(delta, Dmax)
// (Eq. (2), (3)); s <= 32767, arithmetic modulo 2^16.
__device__ __forceinline__ ushort2_t scores2(ushort2_t delta, unsigned short D, unsigned short negS,
                                             unsigned short B)
{
    const ushort2_t d2 = {D, D}, s2 = {negS, negS}, b2 = {B, B};
    return __builtin_elementwise_min(delta, d2) * s2 + b2;
}

// Division of a number below 2^31 by a fixed divisor: floor(x / d) = (x * magic) >> (31 + l)
// with l = ceil(log2 d) and magic = floor(2^(31+l) / d) + 1 < 2^32 (round-up method for 31-bit
// dividends).
struct FastDiv {
    uint32_t divisor, magic, shift;
    __device__ __forceinline__ uint32_t quotient(uint32_t x) const
    {
        return (uint32_t)(((uint64_t)x * magic) >> 31) >> shift;
    }
};
inline FastDiv make_fast_div(uint32_t d)
{
    uint32_t l = 0;
    while (((uint64_t)1 << l) < d) ++l;
    FastDiv f;
    f.divisor = d, f.shift = l;
    f.magic = (uint32_t)((((uint64_t)1 << (31 + l)) / d) + 1);
    return f;
}

// Where a block works: tile inside a (batch, head) slab, head, slab number.  The grid is
// one-dimensional (tiles*H*B blocks; the entry points keep the row count, hence the block
// count, below 2^31) and the block number is taken apart by multiply-shift divisions.
struct BlockPlace {
    FastDiv by_tiles, by_H;
    // neighbours: workgroups go to the 8 dies round-robin; of every 64 consecutive blocks each die then takes 8
    // consecutive ones (the blocks behind the last full 64 keep their numbers).  For rows that are no whole
    // number of 128-byte lines, where consecutive blocks meet inside lines that the die's L2 can then put
    // together: 2-7 % faster ([4,16,2048,4000] 173 against 180 us, 6000 bytes 257 against 262, 12000 bytes 248
    // against 266, 50000 bytes 266 against 274); rows of whole lines lose 5-6 % with it ([4,16,4096,4096] 349 against 328 us).
    uint32_t neighbours;
    __device__ __forceinline__ void locate(uint32_t &tile, uint32_t &head, uint32_t &slab) const
    {
        uint32_t block = blockIdx.x;
        if (neighbours && block < (gridDim.x & ~63u)) block = (block & ~63u) + (block & 7u) * 8u + ((block >> 3) & 7u);
        slab = by_tiles.quotient(block);
        tile = block - slab * by_tiles.divisor;
        head = slab - by_H.quotient(slab) * by_H.divisor;
    }
};
// grid and block placement for `tiles` blocks per slab (tiles*H*Bt < 2^31)
inline BlockPlace place_blocks(int64_t tiles, int H, int64_t Bt, dim3 &grid, bool neighbours = false)
{
    BlockPlace bp;
    bp.by_tiles = make_fast_div((uint32_t)tiles), bp.by_H = make_fast_div((uint32_t)H);
    bp.neighbours = neighbours ? 1u : 0u;
    grid = dim3((uint32_t)(tiles * H * Bt));
    return bp;
}

// Launches `kernel` and returns the status of this launch alone (an error left behind by an
// earlier, unrelated runtime call is neither reported nor cleared here).
template <typename... Params, typename... Args, size_t... I>
inline hipError_t launch_impl(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t st,
                              std::index_sequence<I...>, Args &&...args)
{
    std::tuple<Params...> held(static_cast<Params>(std::forward<Args>(args))...);
    void *ptrs[] = {(void *)&std::get<I>(held)...};
    return hipLaunchKernel((const void *)kernel, grid, block, ptrs, lds_bytes, st);
}
template <typename... Params, typename... Args>
inline hipError_t launch(void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t st, Args &&...args)
{
    static_assert(sizeof...(Params) == sizeof...(Args), "one argument per kernel parameter");
    return launch_impl(kernel, grid, block, 0, st, std::index_sequence_for<Params...>{}, std::forward<Args>(args)...);
}
// The same with `lds_bytes` of LDS per block that the kernel does not touch: fewer blocks fit a compute unit at once.
template <typename... Params, typename... Args>
inline hipError_t launch_fewer(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t st,
                               Args &&...args)
{
    static_assert(sizeof...(Params) == sizeof...(Args), "one argument per kernel parameter");
    return launch_impl(kernel, grid, block, lds_bytes, st, std::index_sequence_for<Params...>{}, std::forward<Args>(args)...);
}

// P <= 127 for every row the table allows: the largest probability of a row is that of its maximum,
// (B*rho) >> 15, and rho = floor(255*2^15 / Z) is largest for the smallest row sum a head can have,
// Z = B + (n-1)*(B - S*Dmax) (one element at the maximum, all others clamped).
inline int64_t largest_probability(int64_t B, int64_t S, int64_t D, int64_t n)
{
    const int64_t zmin = B + (n - 1) * (B - S * D);
    const int64_t rho = (int64_t)kRecipNumerator / (zmin > 0 ? zmin : 1);
    return (B * rho) >> 15;
}
inline bool probabilities_fit_signed(const HeadTable &tab, int H, int n)
{
    for (int h = 0; h < H; ++h)
        if (largest_probability(tab.e[h].x, tab.e[h].y, tab.e[h].z, n) > 127) return false;
    return true;
}

}  // namespace hccs
