// Pieces shared by the two fused-attention kernels (resident and streaming).
#pragma once
#include "hccs_device.h"

namespace hccs {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef v2i __attribute__((address_space(3))) lds_v2i;   // operand type of the transposing LDS read

// min(max(x, lo), hi); the compiler selects v_med3_i32 for it
__device__ __forceinline__ int clamp_i32(int x, int lo, int hi) { return min(max(x, lo), hi); }

// D = S0.u16 * S1.u16 + S2.u32 on the low (lo) or high (hi) half of the first source.
__device__ __forceinline__ uint32_t mad_u32_u16_lo(uint32_t a, uint32_t b, uint32_t c)
{
    uint32_t d;
    asm("v_mad_u32_u16 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}
__device__ __forceinline__ uint32_t mad_u32_u16_hi(uint32_t a, uint32_t b, uint32_t c)
{
    uint32_t d;
    asm("v_mad_u32_u16 %0, %1, %2, %3 op_sel:[1,0,0,0]" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

// Two signed 16-bit values -> two unsigned bytes, saturated to [0,255], in the low half.
__device__ __forceinline__ uint32_t sat_pk_u8_i16(uint32_t v)
{
    uint32_t d;
    asm("v_sat_pk_u8_i16 %0, %1" : "=v"(d) : "v"(v));
    return d;
}

// the value the lane next door (lane ^ 1) holds: DPP quad_perm [1,0,3,2]
__device__ __forceinline__ int neighbour_lane(int x) { return __builtin_amdgcn_mov_dpp(x, 0xB1, 0xF, 0xF, true); }

// Stores the 16 rows of a query tile after a transposed second contraction.  As the contraction
// leaves them, the four lanes (g = 0..3) of a query hold 64 consecutive bytes of its row per
// accumulator, and a store of one accumulator would write half a 128-byte line of 16 rows: memory
// takes such halves at little more than half the rate of whole lines (measured 3.5 against 5.9
// TB/s).  So neighbouring queries (lanes qi, qi ^ 1) first trade accumulators: the even lane keeps
// chunk `pair` of both rows, the odd lane chunk `pair + 1`, and each store instruction then writes
// whole lines of 8 rows.  tile_base: the tile's first row; row_ints: row pitch in 32-bit words;
// rows: how many of the 16 rows exist.  NCH (even): accumulators per lane, 16 columns each.
template <int NCH>
__device__ __forceinline__ void store_rows_whole_lines(int32_t *tile_base, int row_ints, int rows, int lane,
                                                       const v4i (&oacc)[NCH])
{
    static_assert(NCH % 2 == 0, "chunks are traded in pairs");
    const int qi = lane & 15, g = lane >> 4;
    const bool odd = qi & 1;
    const int upper_row = qi & ~1;
    int32_t *dst = tile_base + (size_t)upper_row * row_ints + 16 * (qi & 1) + 4 * g;
#pragma unroll
    for (int pair = 0; pair < NCH; pair += 2) {
        v4i upper, lower;   // rows 2p and 2p + 1 of the lane pair
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int theirs_lo = neighbour_lane(oacc[pair][c]), theirs_hi = neighbour_lane(oacc[pair + 1][c]);
            upper[c] = odd ? theirs_hi : oacc[pair][c];
            lower[c] = odd ? oacc[pair + 1][c] : theirs_lo;
        }
        if (upper_row < rows) __builtin_nontemporal_store(upper, (v4i *)(dst + 16 * pair));
        if (upper_row + 1 < rows) __builtin_nontemporal_store(lower, (v4i *)(dst + row_ints + 16 * pair));
    }
}

constexpr int kKStride = 80;   // bytes per K row in LDS: 64 + 16 of padding against bank conflicts

// How the int32 accumulator becomes a 16-bit logit (before the int8 saturation):
enum : int {
    kRescaleHigh16 = 0,   // every head's rule was rewritten to shift 16: the logit is the high half
    kRescaleShift = 1,    // multiply-add, arithmetic shift, saturating pack
    kRescalePreclamp = 2  // as kRescaleShift, with the accumulator saturated first
};


// Rescale of four accumulators of one key tile to two 16-bit logit pairs (before the int8
// saturation): keys r = 0,1 in the first pair, r = 2,3 in the second.
template <int RQ>
__device__ __forceinline__ void rescale_tile(const v4i &acc, int mult, int shift, int round_c, int lim_lo,
                                             int lim_hi, short2_t &p01, short2_t &p23)
{
    int y[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        int a = acc[r];
        if constexpr (RQ == kRescalePreclamp) a = clamp_i32(a, lim_lo, lim_hi);
        y[r] = __mul24(a, mult) + round_c;
    }
    if constexpr (RQ == kRescaleHigh16) {
        // shift is 16 and |acc*mult + 2^15| < 2^31: the logit is the signed high half
        p01 = __builtin_bit_cast(short2_t, __builtin_amdgcn_perm((uint32_t)y[1], (uint32_t)y[0], 0x07060302u));
        p23 = __builtin_bit_cast(short2_t, __builtin_amdgcn_perm((uint32_t)y[3], (uint32_t)y[2], 0x07060302u));
    } else {
        p01 = __builtin_amdgcn_cvt_pk_i16(y[0] >> shift, y[1] >> shift);   // saturating 32 -> 16
        p23 = __builtin_amdgcn_cvt_pk_i16(y[2] >> shift, y[3] >> shift);
    }
}

// 16-bit lane masks of the keys kbase + {0,1} and kbase + {2,3} that exist (key < Lk): all ones
// except in the last, partial key tile.
__device__ __forceinline__ void key_pair_masks(int kbase, int Lk, uint32_t &m01, uint32_t &m23)
{
    m01 = (kbase < Lk ? 0x0000ffffu : 0u) | (kbase + 1 < Lk ? 0xffff0000u : 0u);
    m23 = (kbase + 2 < Lk ? 0x0000ffffu : 0u) | (kbase + 3 < Lk ? 0xffff0000u : 0u);
}
__device__ __forceinline__ short2_t mask_pair(short2_t p, uint32_t mask, uint32_t fill)
{
    return __builtin_bit_cast(short2_t, (__builtin_bit_cast(uint32_t, p) & mask) | (fill & ~mask));
}

// Four scores (two 16-bit pairs) -> four bytes P - 128: byte 2 of s*(2*rho) + 0x800000 is
// ((s*rho) >> 15) + 128 modulo 256.
__device__ __forceinline__ uint32_t probabilities_minus_128(uint32_t s01, uint32_t s23, uint32_t rho2)
{
    const uint32_t bias = 0x800000u;
    const uint32_t e0 = mad_u32_u16_lo(s01, rho2, bias), e1 = mad_u32_u16_hi(s01, rho2, bias);
    const uint32_t e2 = mad_u32_u16_lo(s23, rho2, bias), e3 = mad_u32_u16_hi(s23, rho2, bias);
    const uint32_t h01 = __builtin_amdgcn_perm(e1, e0, 0x00000602u);
    const uint32_t h23 = __builtin_amdgcn_perm(e3, e2, 0x00000602u);
    return __builtin_amdgcn_perm(h23, h01, 0x05040100u);
}

// Four scores (two 16-bit pairs) -> four bytes P: byte 2 of s*(2*rho) is (s*rho) >> 15.
__device__ __forceinline__ uint32_t probabilities_plain(uint32_t s01, uint32_t s23, uint32_t rho2)
{
    const uint32_t e0 = mad_u32_u16_lo(s01, rho2, 0u), e1 = mad_u32_u16_hi(s01, rho2, 0u);
    const uint32_t e2 = mad_u32_u16_lo(s23, rho2, 0u), e3 = mad_u32_u16_hi(s23, rho2, 0u);
    const uint32_t h01 = __builtin_amdgcn_perm(e1, e0, 0x00000602u);
    const uint32_t h23 = __builtin_amdgcn_perm(e3, e2, 0x00000602u);
    return __builtin_amdgcn_perm(h23, h01, 0x05040100u);
}

// The matrix unit multiplies signed bytes, so it reads a probability above 127 as P - 256.  A row has at most one
// such probability (its probabilities sum to at most 255), and only if its largest one, (B*rho) >> 15, exceeds 127;
// top_tile (wave-uniform) says that some row of the tile can.  Then, if any lane holds such a byte among the four
// registers p (64 keys of its query), p becomes the top bits as bytes of 64 and the call returns true: the caller
// feeds them four more times into the same accumulators, P.V = (P - 256*b).V + 4*(64*b).V.
template <bool PS>
__device__ __forceinline__ bool top_bits_as_64s(bool top_tile, v4i &p)
{
    if constexpr (PS) return false;
    if (!top_tile) return false;
    if (__builtin_amdgcn_ballot_w64(((p[0] | p[1] | p[2] | p[3]) & (int)0x80808080) != 0) == 0) return false;
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) p[tt] = (int)(((uint32_t)p[tt] & 0x80808080u) >> 1);
    return true;
}

// 4x4 byte transpose: r[k] holds 4 columns of key k; w[c] receives the 4 keys of column c.
__device__ __forceinline__ void transpose4x4(const uint32_t (&r)[4], uint32_t (&w)[4])
{
    const uint32_t a_lo = __builtin_amdgcn_perm(r[1], r[0], 0x05010400u);
    const uint32_t a_hi = __builtin_amdgcn_perm(r[1], r[0], 0x07030602u);
    const uint32_t b_lo = __builtin_amdgcn_perm(r[3], r[2], 0x05010400u);
    const uint32_t b_hi = __builtin_amdgcn_perm(r[3], r[2], 0x07030602u);
    w[0] = __builtin_amdgcn_perm(b_lo, a_lo, 0x05040100u);
    w[1] = __builtin_amdgcn_perm(b_lo, a_lo, 0x07060302u);
    w[2] = __builtin_amdgcn_perm(b_hi, a_hi, 0x05040100u);
    w[3] = __builtin_amdgcn_perm(b_hi, a_hi, 0x07060302u);
}

// Workgroups are handed to the chip's 8 accelerator dies round-robin in linear order, and each
// die has its own L2.  This maps a block's linear number so that consecutive logical numbers
// (the query tiles of one (batch, head), which all stream the same K and V) run on one die:
// die x = linear % 8 gets the logical range [start_x, start_x + count_x).
constexpr uint32_t kDies = 8;
__device__ __forceinline__ uint32_t die_major_block(uint32_t linear, uint32_t total)
{
    const uint32_t die = linear % kDies, slot = linear / kDies;
    const uint32_t per = total / kDies, extra = total % kDies;
    return die * per + min(die, extra) + slot;
}

// Saturation bounds for the accumulator of one head (kRescalePreclamp): the smallest a whose
// rescaled value is already >= 127 and the largest a whose rescaled value is already <= -128.
// Clamping the accumulator to [lo, hi] therefore changes no logit, and hi*mult + 2^(shift-1)
// <= 127*2^shift + mult - 1 and lo*mult + 2^(shift-1) >= -127*2^shift - mult stay inside 32 bits
// for every mult <= 4096 and shift <= 24.  Both are also held within the accumulator's own range
// (the 24-bit multiply needs |a| < 2^23).
inline void preclamp_limits(int64_t mult, int64_t shift, int64_t acc_bound, int &lo, int &hi)
{
    const int64_t half = (int64_t)1 << (shift - 1), top = (int64_t)127 << shift;
    const int64_t hi64 = (top - half + mult - 1) / mult;                 // ceil((127*2^shift - half) / mult)
    const int64_t lo64 = -((top + half + 1 + mult - 1) / mult);          // floor((-127*2^shift - half - 1) / mult)
    hi = (int)(hi64 < acc_bound ? hi64 : acc_bound);
    lo = (int)(lo64 > -acc_bound ? lo64 : -acc_bound);
}

// Picks the cheapest exact rescale form for a set of heads (|acc| <= acc_bound) and rewrites
// the table for it: every rule as (mult << (16-shift), 16) if that keeps acc*mult + 2^15 (plus
// `headroom`, for a kernel that adds an offset to the rounding constant) in 32 bits, else
// multiply-add and shift, with the accumulator saturated first if needed (entries z, w of the
// rewritten table: the bounds of preclamp_limits).
inline int choose_rescale(const RequantTable &in, int H, int64_t acc_bound, RequantTable &out, int64_t headroom = 0)
{
    out = in;
    bool high16 = true, preclamp = false;
    for (int h = 0; h < H; ++h) {
        const int64_t mult = in.e[h].x, shift = in.e[h].y;
        if (shift > 16 || (acc_bound * (mult << (16 - shift)) + (1 << 15) + headroom) > 0x7fffffffll) high16 = false;
        if (acc_bound * mult + ((int64_t)1 << (shift - 1)) > 0x7fffffffll) preclamp = true;
    }
    for (int h = 0; h < H; ++h) {
        if (high16) out.e[h].x = in.e[h].x << (16 - in.e[h].y), out.e[h].y = 16;
        preclamp_limits(in.e[h].x, in.e[h].y, acc_bound, out.e[h].z, out.e[h].w);
    }
    return high16 ? kRescaleHigh16 : (preclamp ? kRescalePreclamp : kRescaleShift);
}

}  // namespace hccs
