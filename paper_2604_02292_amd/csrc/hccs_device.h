// Device-side building blocks shared by the HCCS kernels (gfx950, wave64).
//
// Everything the method computes is integer arithmetic (Alg. 1; Eq. (2), (3),
// (5), (8)); the few float instructions used below are exact on the operand
// ranges the admissibility band guarantees, and each such use says why.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/hccs.h"

namespace hccs {

constexpr uint32_t kRecipNumerator = 255u << 15;  // numerator of Eq. (8), R = 15

// Per-head constants carried by value in the kernel arguments, one int4 per
// head: (B, S, Dmax, unused).  A block works on rows of one head, so the entry
// is fetched with scalar loads.
struct HeadTable {
    int4 e[HCCS_MAX_HEADS];
};

struct RequantTable {
    int2 e[HCCS_MAX_HEADS];
};

// 16 bytes of a row, as the hardware moves them (global_load/store_dwordx4).
// The loads and stores are marked non-temporal: every byte is touched once.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u32x4 load_stream(const void *p)
{
    return __builtin_nontemporal_load((const u32x4 *)p);
}
__device__ __forceinline__ void store_stream(void *p, u32x4 v)
{
    __builtin_nontemporal_store(v, (u32x4 *)p);
}
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

// ---- the reciprocal of Eq. (8) -------------------------------------------
// rho = floor(255*2^15 / Z) for 256 <= Z <= 255*2^15.  Numerator and Z are below
// 2^24, so both are exact in float; the hardware reciprocal is good to 1 ulp and
// the quotient is at most 32640, so the truncated float quotient is within one
// of the true one.  The remainder test repairs it in either direction, which
// makes the result the exact floor.
__device__ __forceinline__ uint32_t reciprocal_u8(uint32_t Z)
{
    float qf = (float)kRecipNumerator * __builtin_amdgcn_rcpf((float)Z);
    uint32_t q = (uint32_t)qf;
    int32_t rem = (int32_t)kRecipNumerator - (int32_t)__umul24(q, Z);
    if (rem < 0) {
        q -= 1;
        rem += (int32_t)Z;
    }
    if (rem >= (int32_t)Z) q += 1;
    return q;
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

}  // namespace hccs
