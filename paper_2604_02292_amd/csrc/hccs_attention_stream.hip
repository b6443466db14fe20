// Fused int8 attention block for shapes the resident kernel does not take: any number of
// queries, any key length, head size 64 or 128.  K and V stream through LDS in chunks (64 keys
// in the three-pass kernel, 128 in the two-pass one), so neither the logits of a row nor K and V
// have to fit anywhere.  HCCS needs the row maximum before the clamped sum and the sum before
// the first output, and its floors rule out rescaling partial results.  Up to 4096 keys the
// logits of a query tile are kept as bytes in the registers of one, two or four waves and
// Q.K^T is computed once (two passes, second kernel below); beyond that Q.K^T is recomputed
// three times (first kernel): pass A finds the maximum, pass B the sum Z, pass C the
// probabilities and O = P.V.  Same arithmetic per element as the resident kernels
// (hccs_attention_common.h).
//
// One block per (query tile of 64, batch*head) on a one-dimensional grid, block numbers remapped
// so that the tiles of one (batch, head) share a die's L2; a wave owns 16 queries (and, in the
// two-pass kernel, a share of the keys).  A chunk is double-buffered: the global loads of chunk
// c+1 are issued before chunk c is computed and written to the other LDS buffer afterwards, one
// barrier per chunk.  K and V are both staged row-major with padded rows; V's operands are
// formed by the transposing LDS read.
#include "hccs_attention_common.h"
#include <type_traits>

namespace hccs {

constexpr int kGroupsPerChunk = 2;   // the two-pass kernel stages 128 keys per chunk

template <int ND, int RQ, bool PS>   // head size d = 64*ND; PS: every P <= 127, goes in as it is
__global__ __launch_bounds__(256) void hccs_attention_stream_kernel(const int8_t *__restrict__ q,
                                                                    const int8_t *__restrict__ k,
                                                                    const int8_t *__restrict__ v,
                                                                    int32_t *__restrict__ o, int H, int Lq, int Lk,
                                                                    uint32_t qtiles, HeadTable table,
                                                                    RequantTable requant)
{
    constexpr int DH = 64 * ND;          // head size
    constexpr int KSTR = DH + 16;        // padded K row in LDS (bank spread)
    constexpr int KPARTS = DH / 16;      // 16-byte parts of a K row
    __shared__ __attribute__((aligned(16))) uint8_t lds_k[2][64 * KSTR];
    __shared__ __attribute__((aligned(16))) uint8_t lds_v[2][64 * KSTR];   // row-major like K

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int qi = lane & 15, g = lane >> 4;
    // logical block number: all query tiles of an item on one die, so its K and V stay in that L2
    const uint32_t logical = die_major_block(blockIdx.x, gridDim.x);
    const int item = (int)(logical / qtiles);
    const int head = item % H;
    const int4 hp = table.e[head];
    const int B = hp.x, S = hp.y, D = hp.z;
    const int mult = requant.e[head].x, shift = requant.e[head].y;
    const int round_c = 1 << (shift - 1);
    const int lim_lo = requant.e[head].z, lim_hi = requant.e[head].w;   // accumulator saturation bounds
    const int8_t *kb = k + (size_t)item * Lk * DH;
    const int8_t *vb = v + (size_t)item * Lk * DH;
    const int tile = (int)(logical % qtiles) * 4 + wave;
    // A wave whose queries do not exist works on the last query row instead (the Q operand below is
    // clamped to it): no branch around the arithmetic, only its result is not stored.
    const bool active = tile * 16 < Lq;
    const int nchunks = (Lk + 63) / 64;

    // Q operand: row clamped into range for the tail tile (those rows are never stored)
    v4i qop[ND];
    {
        const int row = min(tile * 16 + qi, Lq - 1);
#pragma unroll
        for (int kd = 0; kd < ND; ++kd)
            qop[kd] = *(const v4i *)(q + ((size_t)item * Lq + row) * DH + 64 * kd + 16 * g);
    }

    // ---- chunk staging -------------------------------------------------------------------
    u32x4 kreg[ND], vreg[ND];
    // K rows past the end are read from the last row instead (their logits are masked anyway);
    // V rows past the end must be zero, which only the last, partial chunk has to check.
    // A whole chunk is one contiguous block of 64*DH bytes: thread t takes bytes 16t .. 16t+15 of each
    // 4 KiB of it (block address wave-uniform, the thread's offset a constant).
    auto load_chunk = [&](int chunk, bool with_v) {
        const int key0 = chunk * 64;
        if (key0 + 64 <= Lk) {
            const size_t at = (size_t)key0 * DH;
#pragma unroll
            for (int i = 0; i < ND; ++i) {
                kreg[i] = *(const u32x4 *)(kb + at + (uint32_t)(tid * 16 + i * 4096));
                if (with_v) vreg[i] = *(const u32x4 *)(vb + at + (uint32_t)(tid * 16 + i * 4096));
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < ND; ++i) {
            const int c = tid + i * 256;
            const int key = key0 + c / KPARTS;
            kreg[i] = *(const u32x4 *)(kb + (size_t)min(key, Lk - 1) * DH + (c % KPARTS) * 16);
            if (with_v) {
                if (key < Lk)
                    vreg[i] = *(const u32x4 *)(vb + (size_t)key * DH + (c % KPARTS) * 16);
                else
                    vreg[i] = (u32x4){0, 0, 0, 0};
            }
        }
    };
    auto store_chunk = [&](int buf, bool with_v) {
#pragma unroll
        for (int i = 0; i < ND; ++i) {
            const int c = tid + i * 256;
            const int at = (c / KPARTS) * KSTR + (c % KPARTS) * 16;
            *(u32x4 *)(lds_k[buf] + at) = kreg[i];
            if (with_v) *(u32x4 *)(lds_v[buf] + at) = vreg[i];
        }
    };

    // logits of key tile tt of the chunk in `buf`, as two 16-bit pairs
    auto tile_logits = [&](int buf, int tt, short2_t &p01, short2_t &p23) {
        v4i acc = {0, 0, 0, 0};
#pragma unroll
        for (int kd = 0; kd < ND; ++kd) {
            const v4i kop = *(const v4i *)(lds_k[buf] + (16 * tt + qi) * KSTR + 64 * kd + 16 * g);
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(kop, qop[kd], acc, 0, 0, 0);
        }
        rescale_tile<RQ>(acc, mult, shift, round_c, lim_lo, lim_hi, p01, p23);
    };

    // Chunks of 64 whole keys take a branch-free body (the four tiles of a chunk overlap); the one
    // chunk that may be partial runs the masked body, once per pass.  `body(buf, key0, masked)`
    // computes one chunk; `with_v` says whether V is staged along with K.
    const int nfull = Lk >> 6;
    const bool tail = (Lk & 63) != 0;
    auto sweep = [&](bool with_v, auto body) {
        load_chunk(0, with_v);
        store_chunk(0, with_v);
        __syncthreads();
        for (int c = 0; c < nfull; ++c) {
            if (c + 1 < nchunks) load_chunk(c + 1, with_v);
            body(c & 1, c * 64, std::false_type{});
            if (c + 1 < nchunks) store_chunk((c + 1) & 1, with_v);
            __syncthreads();
        }
        if (tail) {
            body(nfull & 1, nfull * 64, std::true_type{});
            __syncthreads();
        }
    };

    // ---- pass A: row maximum -------------------------------------------------------------
    short2_t mx2 = {-32768, -32768};
    sweep(false, [&](int buf, int key0, auto masked) {
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            short2_t p01, p23;
            tile_logits(buf, tt, p01, p23);
            if constexpr (decltype(masked)::value) {   // missing keys cannot win the maximum
                uint32_t m01, m23;
                key_pair_masks(key0 + 16 * tt + 4 * g, Lk, m01, m23);
                p01 = mask_pair(p01, m01, 0x80008000u);
                p23 = mask_pair(p23, m23, 0x80008000u);
            }
            mx2 = __builtin_elementwise_max(mx2, __builtin_elementwise_max(p01, p23));
        }
    });
    int mx = max((int)mx2.x, (int)mx2.y);
    mx = max(mx, xor16(mx));
    mx = max(mx, xor32(mx));
    const int m = clamp_i32(mx, -128, 127);
    const short lo = (short)max(m - D, -128);
    const short2_t lo2 = {lo, lo}, hi2 = {127, 127};

    // ---- pass B: sum of the window-clamped logits -> Z, reciprocal ----------------------------
    int sx = 0;
    sweep(false, [&](int buf, int key0, auto masked) {
        short2_t sum2 = {0, 0};
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            short2_t p01, p23;
            tile_logits(buf, tt, p01, p23);
            short2_t x01 = __builtin_elementwise_min(__builtin_elementwise_max(p01, lo2), hi2);
            short2_t x23 = __builtin_elementwise_min(__builtin_elementwise_max(p23, lo2), hi2);
            if constexpr (decltype(masked)::value) {   // missing keys add nothing to the sum
                uint32_t m01, m23;
                key_pair_masks(key0 + 16 * tt + 4 * g, Lk, m01, m23);
                x01 = mask_pair(x01, m01, 0u);
                x23 = mask_pair(x23, m23, 0u);
            }
            sum2 += x01;
            sum2 += x23;
        }
        sx += (int)sum2.x + (int)sum2.y;     // at most 8 values of magnitude <= 128 per half and chunk
    });
    sx += xor16(sx);
    sx += xor32(sx);
    // Z = sum (B - S*(m - x')) = Lk*B - S*(Lk*m - sum x')      (Eq. (3), (5))
    const uint32_t Z = (uint32_t)(Lk * B - S * (Lk * m - sx));
    const uint32_t rho2 = reciprocal_u8(Z) * 2u;
    // a row's largest probability is that of its maximum, whose score is B
    const bool top_tile = !PS && __builtin_amdgcn_ballot_w64((((uint32_t)B * rho2) >> 16) > 127u) != 0;
    const ushort2_t s2 = {(unsigned short)S, (unsigned short)S};
    const unsigned short cc = (unsigned short)(B - S * m);
    const ushort2_t c2 = {cc, cc};

    // ---- pass C: probabilities and O = P.V ---------------------------------------------------
    const int slot = qi >> 1;   // contraction slot (tt, r) = (slot >> 2, slot & 3) is key 16*tt + 4*g + r of a 64-key group
    const int v_lane_off = (16 * (slot >> 2) + 4 * g + (slot & 3)) * KSTR + 8 * (qi & 1);
    v4i oacc[ND][4];
#pragma unroll
    for (int cg = 0; cg < ND; ++cg)
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) oacc[cg][dt] = (v4i){0, 0, 0, 0};
    sweep(true, [&](int buf, int key0, auto masked) {
        v4i pop;
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            short2_t p01, p23;
            tile_logits(buf, tt, p01, p23);
            const short2_t x01 = __builtin_elementwise_min(__builtin_elementwise_max(p01, lo2), hi2);
            const short2_t x23 = __builtin_elementwise_min(__builtin_elementwise_max(p23, lo2), hi2);
            uint32_t s01 = __builtin_bit_cast(uint32_t, __builtin_bit_cast(ushort2_t, x01) * s2 + c2);
            uint32_t s23 = __builtin_bit_cast(uint32_t, __builtin_bit_cast(ushort2_t, x23) * s2 + c2);
            if constexpr (decltype(masked)::value) {   // a zero score gives P = 0; those V rows are staged as zero too
                uint32_t m01, m23;
                key_pair_masks(key0 + 16 * tt + 4 * g, Lk, m01, m23);
                s01 &= m01;
                s23 &= m23;
            }
            pop[tt] = (int)probabilities_plain(s01, s23, rho2);
        }
        // V operand through the transposing LDS read (see the two-pass kernel below): lane pair j
        // of a 16-lane group points at the key of contraction slot j, the lane receives its column.
        // The contraction runs transposed, O^T tile = V^T . P^T, with V^T as the first operand.
        v4i top = pop;
        const bool fix = top_bits_as_64s<PS>(top_tile, top);
#pragma unroll
        for (int n16 = 0; n16 < 4 * ND; ++n16) {
            const uint8_t *at = lds_v[buf] + v_lane_off + 16 * n16;
            const v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)at);
            const v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(at + 32 * KSTR));
            const v4i vop = {lo[0], lo[1], hi[0], hi[1]};
            v4i &acc = oacc[n16 / 4][n16 % 4];
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(vop, pop, acc, 0, 0, 0);
            if constexpr (!PS) {
                if (fix) {
#pragma unroll
                    for (int again = 0; again < 4; ++again) acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(vop, top, acc, 0, 0, 0);
                }
            }
        }
    });

    // ---- store: the contraction ran transposed (V^T . P^T), so lane (g, qi) holds columns
    // 16*n16 + 4g .. +3 of query qi: 16 contiguous bytes per lane
    // 16 bytes per lane where the contraction left them: these stores hide behind the arithmetic of
    // other blocks, and trading accumulators for whole-line stores (store_rows_whole_lines) measured
    // no faster here while costing registers the split kernels do not have
    if (active) {
        const int row = tile * 16 + qi;
        if (row < Lq) {
#pragma unroll
            for (int n16 = 0; n16 < 4 * ND; ++n16)
                __builtin_nontemporal_store(oacc[n16 / 4][n16 % 4],
                                            (v4i *)(o + ((size_t)item * Lq + row) * DH + 16 * n16 + 4 * g));
        }
    }
}

// ---------------------------------------------------------------------------
// Two-pass form for key lengths up to 64*NCMAX: the logits of a query tile are kept in
// registers as offset-binary bytes (u = x + 128, four keys per register), so Q.K^T is computed
// once.  Pass 1 streams K and fills the bytes; the HCCS stage then runs on them with the
// byte-parallel steps of the stand-alone kernel (distances by one subtraction per four keys,
// the clamped sum from two byte-SADs, one exact fma and a saturating pack per probability);
// pass 2 streams V for O = P.V.  Key slots that do not exist hold u = 0: that is the identity
// of the maximum, their distance to it is m + 128 -- a known amount taken out of the sum -- and
// their V rows are staged as zero, so whatever P they get multiplies nothing.
//
// A chunk is GPC groups of 64 keys (one barrier per chunk).  Chunks of whole keys take a
// branch-free path, so that the tiles of a chunk overlap (operand reads, contractions and
// rescales of different tiles interleave); the one chunk that may be partial is handled once,
// after them, with registers of its own.
//
// KS = 2 or 4: the keys of a row are dealt out to KS waves (blocks of 4*KS waves: 4 query tiles
// x KS shares, each share staging its own chunks).  A wave then holds 1/KS of the logits, more
// waves fit a compute unit, and rows up to 4096 keys fit two passes.  The shares exchange
// their row maxima and clamped sums through LDS and hand their accumulators to the first share
// at the end.
// The matrix unit multiplies signed bytes, P is unsigned: P goes in as it is.  Unless the host has
// shown that no P of this table exceeds 127 (PS), a tile whose rows can reach 128 looks for such
// bytes per 64 keys and makes up for what the unit lost (top_bits_as_64s).
// ---------------------------------------------------------------------------
template <int NCMAX, int ND, int RQ, int GPC, bool PS, int KS, bool KT>
__global__ __launch_bounds__(256 * KS, KS > 1 ? 4 : (NCMAX <= 16 ? 3 : 2)) void hccs_attention_stream2_kernel(
    const int8_t *__restrict__ q, const int8_t *__restrict__ k, const int8_t *__restrict__ v,
    int32_t *__restrict__ o, int H, int Lq, int Lk, uint32_t qtiles, HeadTable table, RequantTable requant)
{
    constexpr int DH = 64 * ND;
    constexpr int KSTR = DH + 16;
    constexpr int KPARTS = DH / 16;
    constexpr int CK = 64 * GPC;             // keys per chunk
    constexpr int TPC = 4 * GPC;             // 16-key tiles per chunk
    constexpr int NCH = NCMAX / GPC;         // chunks of whole keys at most
    constexpr int KU = ND * GPC;             // staging units per thread (K: 16-byte pieces; V: 4x4 byte blocks)
    static_assert(NCMAX % GPC == 0, "whole chunks");
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[KS][2][CK * KSTR];   // pass 1: K chunks; pass 2: V chunks
    __shared__ int exchange[KS][4][16];   // KS > 1: row maxima and clamped sums of the key shares

    // KS = 2 or 4: 4*KS waves, wave w works on query tile w & 3 and on key share w >> 2; the four
    // waves of a share stage its chunks.  Every share has the same number of whole chunks, and with
    // KT one more, partial chunk of fewer than CK keys (possibly none): the host sees to that, so all
    // waves of the block meet at the same barriers.
    const int lane = threadIdx.x & 63, wave = (threadIdx.x >> 6) & 3;
    const int half = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 8));   // wave-uniform: the share's bounds stay scalar
    const int tid = threadIdx.x & 255;    // thread number among the waves that share chunks
    const int qi = lane & 15, g = lane >> 4;
    uint8_t(*lds_k)[CK * KSTR] = lds_all[half];
    // logical block number: all query tiles of an item on one die, so its K and V stay in that L2
    const uint32_t logical = die_major_block(blockIdx.x, gridDim.x);
    const int item = (int)(logical / qtiles);
    const int head = item % H;
    const int4 hp = table.e[head];
    const int B = hp.x, S = hp.y, D = hp.z;
    const int mult = requant.e[head].x, shift = requant.e[head].y;
    const int round_c = 1 << (shift - 1);
    const int lim_lo = requant.e[head].z, lim_hi = requant.e[head].w;   // accumulator saturation bounds
    const int Lk_all = Lk;               // keys of the row; Lk from here on: keys of this wave's share
    int first_key = 0;
    if constexpr (KS > 1) {
        // what is left beyond KS equal sets of whole chunks is dealt out evenly, the first shares
        // taking one key more
        const int whole = Lk_all / (KS * CK) * CK, rest = Lk_all - KS * whole;
        const int each = rest / KS, more = rest % KS;
        Lk = whole + each + (half < more ? 1 : 0);
        first_key = half * (whole + each) + min(half, more);
    }
    const int8_t *kb = k + ((size_t)item * Lk_all + (size_t)first_key) * DH;
    const int8_t *vb = v + ((size_t)item * Lk_all + (size_t)first_key) * DH;
    const int tile = (int)(logical % qtiles) * 4 + wave;
    const bool active = tile * 16 < Lq;   // otherwise the wave works on the last query row and stores nothing
    const int nfull = Lk / CK;
    const bool tail = KS == 1 ? (Lk % CK) != 0 : KT;
    const int nchunks = nfull + (tail ? 1 : 0);
    const int tail_buf = nfull & 1;      // the chunk after the whole ones was staged by their last iteration

    v4i qop[ND];
    {
        const int row = min(tile * 16 + qi, Lq - 1);
#pragma unroll
        for (int kd = 0; kd < ND; ++kd)
            qop[kd] = *(const v4i *)(q + ((size_t)item * Lq + row) * DH + 64 * kd + 16 * g);
    }

    u32x4 kreg[KU];
    // K rows past the end are read from the last row instead: their logits are masked anyway
    // A whole chunk is one contiguous block of CK*DH bytes: thread t takes bytes 16t .. 16t+15 of
    // each 4 KiB of it (block address wave-uniform, the thread's offset a constant).
    auto load_k = [&](int chunk) {
        if (chunk * CK + CK <= Lk) {
            const int8_t *block = kb + (size_t)chunk * (CK * DH);
#pragma unroll
            for (int i = 0; i < KU; ++i) kreg[i] = *(const u32x4 *)(block + (uint32_t)(tid * 16 + i * 4096));
        } else {
#pragma unroll
            for (int i = 0; i < KU; ++i) {
                const int c = tid + i * 256;
                const int key = min(chunk * CK + c / KPARTS, Lk - 1);
                kreg[i] = *(const u32x4 *)(kb + (size_t)key * DH + (c % KPARTS) * 16);
            }
        }
    };
    auto store_k = [&](int buf) {
#pragma unroll
        for (int i = 0; i < KU; ++i) {
            const int c = tid + i * 256;
            *(u32x4 *)(lds_k[buf] + (c / KPARTS) * KSTR + (c % KPARTS) * 16) = kreg[i];
        }
    };
    // V is staged row-major like K (rows past the end as zeros, which only the last, partial chunk
    // has to check); its operands are formed by the transposing LDS read, see chunk_pv.
    auto load_v = [&](int chunk) {
        if (chunk * CK + CK <= Lk) {
            const int8_t *block = vb + (size_t)chunk * (CK * DH);
#pragma unroll
            for (int i = 0; i < KU; ++i) kreg[i] = *(const u32x4 *)(block + (uint32_t)(tid * 16 + i * 4096));
        } else {
#pragma unroll
            for (int i = 0; i < KU; ++i) {
                const int c = tid + i * 256;
                const int key = chunk * CK + c / KPARTS;
                if (key < Lk)
                    kreg[i] = *(const u32x4 *)(vb + (size_t)key * DH + (c % KPARTS) * 16);
                else
                    kreg[i] = (u32x4){0, 0, 0, 0};
            }
        }
    };

    // ---- pass 1: logits as offset-binary bytes, running maximum --------------------------------
    constexpr int TT = (KS == 1 || KT) ? TPC : 0;   // tiles of the partial chunk
    uint32_t xb[NCMAX * 4], xt[TT + 1];
#pragma unroll
    for (int i = 0; i < NCMAX * 4; ++i) xb[i] = 0;
#pragma unroll
    for (int i = 0; i < TT; ++i) xt[i] = 0;
    short2_t mx2 = {-32768, -32768};
    // tile tt of the chunk in `buf`: logits -> running maximum, bytes u = clamp(x, -128, 127) + 128
    auto tile_bytes = [&](const uint8_t *buf, int tt, auto masked, int key0) -> uint32_t {
        v4i acc = {0, 0, 0, 0};
#pragma unroll
        for (int kd = 0; kd < ND; ++kd) {
            const v4i kop = *(const v4i *)(buf + (16 * tt + qi) * KSTR + 64 * kd + 16 * g);
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(kop, qop[kd], acc, 0, 0, 0);
        }
        // logits + 128 (the maximum is tracked with the same offset); in the high-half form the
        // offset rides on the rounding constant (the host has checked the headroom for it)
        short2_t p01, p23;
        if constexpr (RQ == kRescaleHigh16) {
            rescale_tile<RQ>(acc, mult, shift, round_c + (128 << 16), lim_lo, lim_hi, p01, p23);
        } else {
            rescale_tile<RQ>(acc, mult, shift, round_c, lim_lo, lim_hi, p01, p23);
            const short2_t c128 = {128, 128};
            p01 = __builtin_elementwise_add_sat(p01, c128);
            p23 = __builtin_elementwise_add_sat(p23, c128);
        }
        if constexpr (decltype(masked)::value) {
            // key slots that do not exist get the lowest 16-bit value: they cannot win the
            // maximum and saturate to u = 0 below
            uint32_t m01, m23;
            key_pair_masks(key0 + 16 * tt + 4 * g, Lk, m01, m23);
            p01 = mask_pair(p01, m01, 0x80008000u);
            p23 = mask_pair(p23, m23, 0x80008000u);
        }
        mx2 = __builtin_elementwise_max(mx2, __builtin_elementwise_max(p01, p23));
        const uint32_t lo8 = sat_pk_u8_i16(__builtin_bit_cast(uint32_t, p01));
        const uint32_t hi8 = sat_pk_u8_i16(__builtin_bit_cast(uint32_t, p23));
        return __builtin_amdgcn_perm(hi8, lo8, 0x05040100u);
    };
    load_k(0);
    store_k(0);
    __syncthreads();
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        if (c < nfull) {
            if (c + 1 < nchunks) load_k(c + 1);
#pragma unroll
            for (int tt = 0; tt < TPC; ++tt) xb[c * TPC + tt] = tile_bytes(lds_k[c & 1], tt, std::false_type{}, 0);
            if (c + 1 < nchunks) store_k((c + 1) & 1);
            __syncthreads();
        }
        __builtin_amdgcn_sched_barrier(0);   // keep the unrolled chunks in order: registers, not latency, are scarce
    }
    if (tail) {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) xt[tt] = tile_bytes(lds_k[tail_buf], tt, std::true_type{}, nfull * CK);
        __syncthreads();                     // the buffers are refilled with V next
    }
    int mx = max((int)mx2.x, (int)mx2.y);
    mx = max(mx, xor16(mx));
    mx = max(mx, xor32(mx));
    if constexpr (KS > 1) {   // the row's maximum is the largest of the shares'
        if (g == 0) exchange[half][wave][qi] = mx;
        __syncthreads();
#pragma unroll
        for (int other = 1; other < KS; ++other) mx = max(mx, exchange[(half + other) % KS][wave][qi]);
        __syncthreads();       // the array is used again for the sums
    }
    const uint32_t mu = (uint32_t)clamp_i32(mx, 0, 255);   // saturation is monotone; mx carries the +128

    // ---- HCCS on the bytes: distances, clamped sum, row constants -------------------------------
    const uint32_t mu4 = mu * 0x01010101u, D4 = (uint32_t)D * 0x01010101u;
    uint32_t acc_d = 0, acc_abs = 0;
#pragma unroll
    for (int i = 0; i < NCMAX * 4; ++i) {
        const uint32_t dl = mu4 - xb[i];       // every byte is <= mu: no borrow
        xb[i] = dl;
        acc_d = __builtin_amdgcn_sad_u8(dl, 0u, acc_d);
        acc_abs = __builtin_amdgcn_sad_u8(dl, D4, acc_abs);
    }
#pragma unroll
    for (int i = 0; i < TT; ++i) {
        const uint32_t dl = mu4 - xt[i];
        xt[i] = dl;
        acc_d = __builtin_amdgcn_sad_u8(dl, 0u, acc_d);
        acc_abs = __builtin_amdgcn_sad_u8(dl, D4, acc_abs);
    }
    int tsum = (int)acc_d - (int)acc_abs;
    tsum += xor16(tsum);
    tsum += xor32(tsum);
    constexpr int kSlots = NCMAX * 64 + TT * 16;    // every slot that is not a key holds u = 0
    int sum_clamped = (tsum + kSlots * D) / 2 - (kSlots - Lk) * (int)min(mu, (uint32_t)D);
    if constexpr (KS > 1) {   // Eq. (5) runs over the whole row: every share's sum
        if (g == 0) exchange[half][wave][qi] = sum_clamped;
        __syncthreads();
#pragma unroll
        for (int other = 1; other < KS; ++other) sum_clamped += exchange[(half + other) % KS][wave][qi];
    }
    const uint32_t Z = (uint32_t)(Lk_all * B - S * sum_clamped);
    const RowAffine ra = row_affine(Z, B, S, D);
    // a row's largest probability is that of its maximum, whose score is B
    const bool top_tile = !PS && __builtin_amdgcn_ballot_w64((((uint32_t)B * reciprocal_u8(Z)) >> 15) > 127u) != 0;

    // ---- pass 2: O = P.V -----------------------------------------------------------------------
    v4i oacc[ND][4];
#pragma unroll
    for (int cg = 0; cg < ND; ++cg)
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) oacc[cg][dt] = (v4i){0, 0, 0, 0};
    // V operand of the second contraction, which runs transposed (O^T tile = V^T . P^T, so that a
    // lane ends up with four consecutive columns of one query), for lane (g, qi), 64-key group T,
    // columns 16*n16 .. +15:
    // contraction slot (tt, r) of lane group g is key 64*T + 16*tt + 4*g + r (that is how pass 1
    // left the logits), and the lane's column is 16*n16 + qi.  ds_read_tr8_b64 takes, in each
    // group of 16 lanes, the 8 bytes at every lane's address, pairs lanes (2j, 2j+1) into eight
    // 16-byte rows j, and gives lane i the eight bytes of column i: so lane pair j points at the
    // two halves of the 16 columns of the key of slot j (first read: tt = 0, 1; second: tt = 2, 3).
    const int slot = qi >> 1;
    const int v_lane_off = (16 * (slot >> 2) + 4 * g + (slot & 3)) * KSTR + 8 * (qi & 1);
    auto chunk_pv = [&](const uint8_t *buf, const uint32_t *dist) {
#pragma unroll
        for (int T = 0; T < GPC; ++T) {
            v4i pop;
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) pop[tt] = (int)normalise4(dist[T * 4 + tt], ra);
            v4i top = pop;
            const bool fix = top_bits_as_64s<PS>(top_tile, top);
#pragma unroll
            for (int n16 = 0; n16 < 4 * ND; ++n16) {
                const uint8_t *at = buf + 64 * T * KSTR + v_lane_off + 16 * n16;
                const v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)at);
                const v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(at + 32 * KSTR));
                const v4i vop = {lo[0], lo[1], hi[0], hi[1]};
                v4i &acc = oacc[n16 / 4][n16 % 4];
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(vop, pop, acc, 0, 0, 0);
                if constexpr (!PS) {
                    if (fix) {
#pragma unroll
                        for (int again = 0; again < 4; ++again)
                            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(vop, top, acc, 0, 0, 0);
                    }
                }
            }
        }
    };
    load_v(0);
    store_k(0);
    __syncthreads();
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        if (c < nfull) {
            if (c + 1 < nchunks) load_v(c + 1);
            chunk_pv(lds_k[c & 1], &xb[c * TPC]);
            if (c + 1 < nchunks) store_k((c + 1) & 1);
            __syncthreads();
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (TT > 0) {
        if (tail) chunk_pv(lds_k[tail_buf], xt);   // V rows past the end were staged as zero
    }

    if constexpr (KS > 1) {
        // O is the sum of the shares' results: all but the first hand their accumulators over
        // through LDS (lane-major, 4*ND*4 dwords per lane; the chunk buffers are free by now)
        constexpr int kHandDwords = 4 * ND * 4 * 256;   // of one share
        int32_t *hand = (int32_t *)&lds_all[0][0][0] + (wave * 64 + lane) * 4;
        static_assert(sizeof(lds_all) >= (size_t)(KS - 1) * kHandDwords * 4, "room for the other shares' accumulators");
        __syncthreads();       // everybody is done with the last chunk
        if (half > 0) {
#pragma unroll
            for (int n16 = 0; n16 < 4 * ND; ++n16)
                *(v4i *)(hand + (half - 1) * kHandDwords + n16 * 1024) = oacc[n16 / 4][n16 % 4];
        }
        __syncthreads();
        if (half > 0) return;
#pragma unroll
        for (int other = 1; other < KS; ++other)
#pragma unroll
            for (int n16 = 0; n16 < 4 * ND; ++n16)
                oacc[n16 / 4][n16 % 4] += *(const v4i *)(hand + (other - 1) * kHandDwords + n16 * 1024);
    }

    // the contraction ran transposed (V^T . P^T), so lane (g, qi) holds columns
    // 16*n16 + 4g .. +3 of query qi: 16 contiguous bytes per lane
    // 16 bytes per lane where the contraction left them: these stores hide behind the arithmetic of
    // other blocks, and trading accumulators for whole-line stores (store_rows_whole_lines) measured
    // no faster here while costing registers the split kernels do not have
    if (active) {
        const int row = tile * 16 + qi;
        if (row < Lq) {
#pragma unroll
            for (int n16 = 0; n16 < 4 * ND; ++n16)
                __builtin_nontemporal_store(oacc[n16 / 4][n16 % 4],
                                            (v4i *)(o + ((size_t)item * Lq + row) * DH + 16 * n16 + 4 * g));
        }
    }
}

template <int NCMAX, int ND, int GPC, bool PS, int KS = 1, bool KT = false>
static hipError_t launch_stream2(const int8_t *q, const int8_t *k, const int8_t *v, int32_t *o, int64_t items, int H,
                                 int Lq, int Lk, const HeadTable &tab, const RequantTable &rq, int kind,
                                 hipStream_t st)
{
    const uint32_t qtiles = (uint32_t)((Lq + 63) / 64);
    const dim3 grid((uint32_t)(qtiles * items)), block(256 * KS);
    if (kind == kRescaleHigh16)
        return launch(hccs_attention_stream2_kernel<NCMAX, ND, kRescaleHigh16, GPC, PS, KS, KT>, grid, block, st, q, k, v, o, H,
                      Lq, Lk, qtiles, tab, rq);
    if (kind == kRescaleShift)
        return launch(hccs_attention_stream2_kernel<NCMAX, ND, kRescaleShift, GPC, PS, KS, KT>, grid, block, st, q, k, v, o, H,
                      Lq, Lk, qtiles, tab, rq);
    return launch(hccs_attention_stream2_kernel<NCMAX, ND, kRescalePreclamp, GPC, PS, KS, KT>, grid, block, st, q, k, v, o, H, Lq,
                  Lk, qtiles, tab, rq);
}

template <int ND, bool PS>
static hipError_t launch_stream_nd(const int8_t *q, const int8_t *k, const int8_t *v, int32_t *o, int64_t items, int H,
                                   int Lq, int Lk, const HeadTable &tab, const RequantTable &rq, int kind,
                                   hipStream_t st)
{
    const uint32_t qtiles = (uint32_t)((Lq + 63) / 64);
    const dim3 grid((uint32_t)(qtiles * items)), block(256);
    if (kind == kRescaleHigh16)
        return launch(hccs_attention_stream_kernel<ND, kRescaleHigh16, PS>, grid, block, st, q, k, v, o, H, Lq, Lk,
                      qtiles, tab, rq);
    if (kind == kRescaleShift)
        return launch(hccs_attention_stream_kernel<ND, kRescaleShift, PS>, grid, block, st, q, k, v, o, H, Lq, Lk,
                      qtiles, tab, rq);
    return launch(hccs_attention_stream_kernel<ND, kRescalePreclamp, PS>, grid, block, st, q, k, v, o, H, Lq, Lk,
                  qtiles, tab, rq);
}

// How the two-pass kernel takes a row: 1 = one wave per query tile holds all its logits (up to 2048
// keys), 2 or 4 = the keys in that many shares on different waves (each share's logits take that
// much less of the registers, so more waves fit a compute unit; head size 64 only: at 128 the
// wider accumulators do not fit the smaller register budget, measured [2,8,2048,2048,128] 42.7
// against 38.3 us), 0 = the row goes to the three-pass kernel.  Shares are equal sets of whole
// chunks plus an even part of the rest, which must stay below a chunk for every share
// (`partial` says whether there is such a rest).
static int key_shares(int Lk, int d, bool &partial)
{
    constexpr int kChunk = 64 * kGroupsPerChunk;
    partial = false;
    if (Lk <= 1024) return 1;
    const int shares = Lk <= 2048 ? 2 : 4;
    const int rest = Lk % (shares * kChunk);
    if (d == 64 && Lk <= 4096 && rest <= shares * (kChunk - 1)) {
        partial = rest != 0;
        return shares;
    }
    return Lk <= 2048 ? 1 : 0;
}

template <int ND, bool PS>
static hipError_t launch_stream_for(const int8_t *q, const int8_t *k, const int8_t *v, int32_t *o, int64_t items, int H,
                                    int Lq, int Lk, int shares, bool partial, const HeadTable &tab,
                                    const RequantTable &rq, int kind, hipStream_t st)
{
    constexpr int G = kGroupsPerChunk;
    if (shares == 0) return launch_stream_nd<ND, PS>(q, k, v, o, items, H, Lq, Lk, tab, rq, kind, st);
    if constexpr (ND == 1) {
        if (shares == 4)
            return partial ? launch_stream2<16, ND, G, PS, 4, true>(q, k, v, o, items, H, Lq, Lk, tab, rq, kind, st)
                           : launch_stream2<16, ND, G, PS, 4, false>(q, k, v, o, items, H, Lq, Lk, tab, rq, kind, st);
        if (shares == 2)
            return partial ? launch_stream2<16, ND, G, PS, 2, true>(q, k, v, o, items, H, Lq, Lk, tab, rq, kind, st)
                           : launch_stream2<16, ND, G, PS, 2, false>(q, k, v, o, items, H, Lq, Lk, tab, rq, kind, st);
    }
    if (Lk <= 1024) return launch_stream2<16, ND, G, PS>(q, k, v, o, items, H, Lq, Lk, tab, rq, kind, st);
    return launch_stream2<32, ND, G, PS>(q, k, v, o, items, H, Lq, Lk, tab, rq, kind, st);
}

hipError_t launch_attention_stream(const int8_t *q, const int8_t *k, const int8_t *v, int32_t *o, int64_t Bt, int H,
                                   int Lq, int Lk, int d, const HeadTable &tab, const RequantTable &rq_in,
                                   hipStream_t st)
{
    if (d != 64 && d != 128) return hipErrorInvalidValue;
    bool partial;
    const int shares = key_shares(Lk, d, partial);
    RequantTable rq;
    // |acc| <= d*128*128; the two-pass kernel adds 128 << 16 to the rounding constant
    const int kind = choose_rescale(rq_in, H, (int64_t)d << 14, rq, shares > 0 ? (int64_t)128 << 16 : 0);
    const int64_t items = Bt * H;
    const bool ps = probabilities_fit_signed(tab, H, Lk);
    if (d == 64)
        return ps ? launch_stream_for<1, true>(q, k, v, o, items, H, Lq, Lk, shares, partial, tab, rq, kind, st)
                  : launch_stream_for<1, false>(q, k, v, o, items, H, Lq, Lk, shares, partial, tab, rq, kind, st);
    return ps ? launch_stream_for<2, true>(q, k, v, o, items, H, Lq, Lk, shares, partial, tab, rq, kind, st)
              : launch_stream_for<2, false>(q, k, v, o, items, H, Lq, Lk, shares, partial, tab, rq, kind, st);
}

}  // namespace hccs
