// Fused int8 attention block: A = Q.K^T (int8 MFMA, int32 accumulate), per-head
// fixed-point rescale to int8 logits, row-wise HCCS (Alg. 1 with the 8-bit output
// path of Sec. III-B, n = L), O = P.V (int8 MFMA).  Logits and probabilities stay
// in registers; K and V are staged once per (batch, head) in LDS.
//
// Two kernels.  The first is launched for 448 keys only, where it measured faster.  The second,
// further down, brings K and V straight into LDS, feeds P to the matrix unit as it is and takes
// every other length up to 896, whole 64s of keys or not.  What follows describes the first.
//
// The matrix unit is used for the two dense contractions only.  Both use
// v_mfma_i32_16x16x64_i8, whose operand layout on a 64-lane wave is
//   A (16 x 64): lane l holds row l%16, columns 16*(l/16) .. +15   (16 bytes)
//   B (64 x 16): lane l holds column l%16, rows 16*(l/16) .. +15   (16 bytes)
//   C (16 x 16): lane l holds column l%16, rows 4*(l/16) .. +3      (4 dwords)
//
// Step 1 computes the transposed tile (keys x queries) = K_tile . Q^T, so a lane
// ends up holding, for ONE query (l%16), four consecutive keys of every key tile.
// The order in which keys enter the second contraction is free as long as P and V
// agree, so those registers, packed to bytes, are directly the A operand of
// O = P.V -- no cross-lane movement between the two contractions.  V is re-laid
// out once per block (4x4 byte transposes) so that its matching B operand is one
// 16-byte LDS read.  Output column j of the d-tile dt is d = 4*j + dt, which makes
// each lane's four results of a row contiguous in memory.
//
// P is unsigned (0..255) but the matrix unit multiplies signed bytes: the kernel
// feeds P - 128 (= P ^ 0x80) and starts the accumulator at 128 * sum_j V[j][d].
//
// Every global load of K and V is issued before the first LDS write, and the next
// tile's Q operand is fetched while the current tile is still in its HCCS stage.
#include "hccs_attention_common.h"

// The block of 56 key tiles keeps its loop over a wave's seven query tiles rolled (the compiler says so for every
// "#pragma unroll" it does not follow); its registers still hold every array, nothing goes to scratch memory.
#pragma clang diagnostic ignored "-Wpass-failed"

namespace hccs {

// The HCCS stage runs on 16-bit pairs (two logits per register, v_pk_* instructions):
//   x' = clamp(y, max(m - D, -128), 127), s = B - S*(m - x')             (Eq. (2), (3))
//   Z = L*B - S*(L*m - sum x')                                           (Eq. (5))
//   p = (s*rho) >> 15 = bits 16..23 of s*(2*rho)                         (Eq. (8))
// so the normalise step is one 16x16->32 multiply-add per element whose byte 2 is the
// probability; adding 0x800000 in the same instruction turns it into P - 128.
template <int NT, int RQ, int WAVES>   // NT = L/16 key tiles (a multiple of 4), RQ = rescale kind, WAVES per block
__global__ __launch_bounds__(64 * WAVES, (NT <= 16 ? 4 : 2)) void hccs_attention_kernel(const int8_t *__restrict__ q,
                                                             const int8_t *__restrict__ k,
                                                             const int8_t *__restrict__ v,
                                                             int32_t *__restrict__ o, int H, HeadTable table,
                                                             RequantTable requant)
{
    constexpr int L = NT * 16;
    constexpr int NQ = NT / 4;     // 64-key groups = MFMAs along the key axis of P.V
    constexpr int NTHR = 64 * WAVES;
    constexpr int KCH = (L * 4 + NTHR - 1) / NTHR;   // 16-byte chunks of K per thread
    constexpr int VUN = (L + NTHR - 1) / NTHR;       // V staging units per thread
    __shared__ __attribute__((aligned(16))) uint8_t lds_k[L * kKStride];
    __shared__ __attribute__((aligned(16))) uint8_t lds_v[L * 64];
    __shared__ __attribute__((aligned(16))) int32_t lds_colsum[64];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int head = blockIdx.x % H;
    const int4 hp = table.e[head];
    const int B = hp.x, S = hp.y, D = hp.z;
    const int mult = requant.e[head].x, shift = requant.e[head].y;
    const size_t base = (size_t)blockIdx.x * L * 64;

    if (tid < 64) lds_colsum[tid] = 0;
    __syncthreads();   // nothing is in flight yet; orders the zeroing before the atomics below

    // ---- issue every global load of the block's K and V, then fill LDS ------------------
    // K: row-major with padded rows.
    // V: staging unit u = (T, g, nn) covers the 16 keys 64*T + 16*tt + 4*g + r (tt, r = 0..3) and
    // the 4 columns 4*nn .. +3.  Each 4x4 byte block (fixed tt) is transposed with byte permutes;
    // the four blocks of a unit then form, per column dt, exactly the 16 operand bytes of lane
    // (g, nn) for the pair (T, dt): key 64*T + 16*tt + 4*g + r is byte r of dword tt.
    {
        u32x4 kreg[KCH];
#pragma unroll
        for (int i = 0; i < KCH; ++i) {
            const int c = tid + i * NTHR;
            if (c < L * 4) kreg[i] = *(const u32x4 *)(k + base + (size_t)c * 16);
        }
        uint32_t vreg[VUN][4][4];
#pragma unroll
        for (int i = 0; i < VUN; ++i) {
            const int u = tid + i * NTHR;
            if (u < L) {
                const int nn = u & 15, g = (u >> 4) & 3, T = u >> 6;
#pragma unroll
                for (int tt = 0; tt < 4; ++tt) {
                    const int8_t *src = v + base + (size_t)(64 * T + 16 * tt + 4 * g) * 64 + nn * 4;
#pragma unroll
                    for (int r = 0; r < 4; ++r) vreg[i][tt][r] = *(const uint32_t *)(src + 64 * r);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < KCH; ++i) {
            const int c = tid + i * NTHR;
            if (c < L * 4) *(u32x4 *)(lds_k + (c >> 2) * kKStride + (c & 3) * 16) = kreg[i];
        }
#pragma unroll
        for (int i = 0; i < VUN; ++i) {
            const int u = tid + i * NTHR;
            if (u < L) {
                const int nn = u & 15, g = (u >> 4) & 3, T = u >> 6;
                u32x4 w[4];   // w[dt][tt]
#pragma unroll
                for (int tt = 0; tt < 4; ++tt) {
                    uint32_t col[4];
                    transpose4x4(vreg[i][tt], col);
#pragma unroll
                    for (int dt = 0; dt < 4; ++dt) w[dt][tt] = col[dt];
                }
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) {
                    *(u32x4 *)(lds_v + (((T * 4 + dt) * 4 + g) * 16 + nn) * 16) = w[dt];
                    int cs = 0;
#pragma unroll
                    for (int tt = 0; tt < 4; ++tt) cs = __builtin_amdgcn_sdot4((int)w[dt][tt], 0x01010101, cs, false);
                    atomicAdd(&lds_colsum[nn * 4 + dt], cs);
                }
            }
        }
    }
    __syncthreads();

    const int qi = lane & 15;      // query inside the 16-row tile / output column group
    const int g = lane >> 4;       // which quarter of the contraction slots this lane feeds
    const int round_c = 1 << (shift - 1);
    // saturation bounds for the accumulator when acc*mult could leave 32 bits (from the host)
    const int lim_lo = requant.e[head].z, lim_hi = requant.e[head].w;

    v4i qop = {0, 0, 0, 0};
    if (wave < NT) qop = *(const v4i *)(q + base + (size_t)(wave * 16 + qi) * 64 + g * 16);
    for (int rt = wave; rt < NT; rt += WAVES) {
        // ---- A^T tiles = K_tile . Q^T, rescaled to 16-bit pairs tile by tile ----------------
        short2_t xp[NT][2];        // logits of keys 16t + 4g + {0,1} and {2,3}; later their scores
        short2_t mx2 = {-32768, -32768};
        // one tile ahead: the matrix unit works on tile t+1 while the vector unit rescales tile t;
        // the scheduling barrier keeps the compiler from hoisting every operand read to the top
        v4i acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(*(const v4i *)(lds_k + qi * kKStride + g * 16), qop,
                                                        (v4i){0, 0, 0, 0}, 0, 0, 0);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            v4i acc_next = acc;
            if (t + 1 < NT) {
                const v4i kop = *(const v4i *)(lds_k + ((t + 1) * 16 + qi) * kKStride + g * 16);
                acc_next = __builtin_amdgcn_mfma_i32_16x16x64_i8(kop, qop, (v4i){0, 0, 0, 0}, 0, 0, 0);
            }
            rescale_tile<RQ>(acc, mult, shift, round_c, lim_lo, lim_hi, xp[t][0], xp[t][1]);
            mx2 = __builtin_elementwise_max(mx2, __builtin_elementwise_max(xp[t][0], xp[t][1]));
            acc = acc_next;
            __builtin_amdgcn_sched_barrier(0);
        }
        // next tile's Q operand: in flight during the HCCS stage and the second contraction
        if (rt + WAVES < NT) qop = *(const v4i *)(q + base + (size_t)((rt + WAVES) * 16 + qi) * 64 + g * 16);

        int mx = max((int)mx2.x, (int)mx2.y);
        mx = max(mx, xor16(mx));
        mx = max(mx, xor32(mx));
        const int m = clamp_i32(mx, -128, 127);   // saturation is monotone: max of clamped = clamp of max

        // ---- window clamp, sum, scores ---------------------------------------------------
        const short lo = (short)max(m - D, -128);
        const short2_t lo2 = {lo, lo}, hi2 = {127, 127};
        const ushort2_t s2 = {(unsigned short)S, (unsigned short)S};
        const unsigned short cc = (unsigned short)(B - S * m);
        const ushort2_t c2 = {cc, cc};
        short2_t sum2 = {0, 0};
#pragma unroll
        for (int t = 0; t < NT; ++t) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const short2_t xc = __builtin_elementwise_min(__builtin_elementwise_max(xp[t][h], lo2), hi2);
                sum2 += xc;                            // at most 64 values of magnitude <= 128 per half
                // s = B - S*(m - x'), computed modulo 2^16 (the result is in [0, 32767])
                xp[t][h] = __builtin_bit_cast(short2_t, __builtin_bit_cast(ushort2_t, xc) * s2 + c2);
            }
        }
        int sx = (int)sum2.x + (int)sum2.y;
        sx += xor16(sx);
        sx += xor32(sx);
        const uint32_t Z = (uint32_t)(L * B - S * (L * m - sx));     // Eq. (3), (5)
        const uint32_t rho2 = reciprocal_u8(Z) * 2u;                 // <= 65280: fits 16 bits

        // ---- P - 128 as the A operand, O = P.V ------------------------------------
        v4i oacc[4];
        {
            const v4i cs = *(const v4i *)(lds_colsum + qi * 4);
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
                const int init = cs[dt] * 128;
                oacc[dt] = (v4i){init, init, init, init};
            }
        }
#pragma unroll
        for (int T = 0; T < NQ; ++T) {
            v4i pop;
#pragma unroll
            for (int tt = 0; tt < 4; ++tt)
                pop[tt] = (int)probabilities_minus_128(__builtin_bit_cast(uint32_t, xp[T * 4 + tt][0]),
                                                       __builtin_bit_cast(uint32_t, xp[T * 4 + tt][1]), rho2);
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
                const v4i vop = *(const v4i *)(lds_v + (((T * 4 + dt) * 4 + g) * 16 + qi) * 16);
                oacc[dt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(pop, vop, oacc[dt], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }

        // ---- store: lane (g, qi) holds rows 4g..4g+3 of the tile, columns 4*qi .. 4*qi+3 ----
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const v4i out = {oacc[0][r], oacc[1][r], oacc[2][r], oacc[3][r]};
            __builtin_nontemporal_store(out, (v4i *)(o + base + (size_t)(rt * 16 + g * 4 + r) * 64 + qi * 4));
        }
    }
}

// ---------------------------------------------------------------------------
// The block in another form: K and V go straight from memory into LDS (global_load_lds_dwordx4: no
// staging registers, no staging instructions), V while the first contraction already runs.
//
// Both K and V are row-major in LDS (64 bytes per key), as the loads deliver them: an instruction
// of a wave moves 16 keys, lane l bringing 16 bytes of key l/4.  Which 16 bytes is permuted per
// key (position p holds chunk p ^ f(key)), so that the operand reads of the matrix unit spread
// over the LDS banks without padding:
//   K, f = (key >> 2) & 3: the first contraction reads, per 16 lanes, one chunk of 16 consecutive
//      keys; their positions 4*key + (chunk ^ f) are 16 different bank groups.
//   V, f = ((key >> 4) + (key >> 2)) & 3: the second contraction takes its operand through the
//      transposing read (ds_read_b64_tr_b8), which touches 32 keys per instruction.
// The second contraction runs transposed (O^T tile = V^T . P^T) like in the streaming kernels, so a
// lane ends with four consecutive columns of one query per accumulator.
//
// The matrix unit multiplies signed bytes and P is unsigned.  P goes in as it is.  When the host
// can show P <= 127 for every row the table allows (true for every table of the band of Eq. (11) at
// 256 keys and more) that is all; otherwise (WIDE) a tile whose rows can reach 128 (a row's largest
// probability is (B*rho) >> 15, known before the contraction) adds what the unit lost, see
// weighted_values_of_tile.  Measured against the kernel above, tables that prove P <= 127, about 88 MB
// of traffic each: L = 64 16.8 against 17.0 us, 128 16.4 against 18.3, 192 19.9 against 21.1, 256 19.3
// against 20.8, 320 27.3 against 27.2, 384 30.8 against 34.6, 512 35.0 against 41.8; tables that do not,
// rows that reach P > 127, 768 items: 64 4.9 against 5.6, 256 20.8 against 22.4, 384 37.6 against 39.8,
// 512 57.3 against 63.0, and 448 (as 512 slots) 53.3 against 48.1, hence its place there.
// ---------------------------------------------------------------------------
typedef const __attribute__((address_space(1))) void *global_void_ptr;
typedef __attribute__((address_space(3))) void *lds_void_ptr;

// 16 bytes per lane from global memory into LDS: lane l's bytes land at lds_wave_base + 16*l
// (the LDS address is wave-uniform, the global address per lane).
// Written out as an instruction, so that the compiler keeps no record of it: every wait for these
// loads is placed by hand (s_waitcnt vmcnt and a barrier), where the compiler's own bookkeeping of
// loads into LDS would also wait for loads that are meant to stay in flight.  M0 carries the LDS
// address.
__device__ __forceinline__ void load_to_lds16(const void *global_lane, void *lds_wave_base)
{
    const int lds_addr = __builtin_amdgcn_readfirstlane((int)(uintptr_t)(lds_void_ptr)lds_wave_base);
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"   // M0 is reserved; nothing else in these kernels uses it
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds_addr), "v"(global_lane)
                 : "memory", "m0");
#pragma clang diagnostic pop
}

// One instruction moves 16 rows (1 KiB): lane l brings chunk (l & 3) ^ f(row) of row 16u + l/4 to
// position l & 3 of that row.  The waves of a block share the NT instructions of an item evenly.
// `last` is the last row the item has.  No load leaves the item: the LDS rows of K behind it receive that row again, so
// their logits repeat the last key's; the rows of V behind it are zero, so those keys add nothing to the output.
template <int NT, int WAVES>
__device__ __forceinline__ void k_rows_to_lds(const int8_t *k_item, uint8_t *k_lds, int wave, int lane, int last)
{
#pragma unroll
    for (int i = 0; i < NT / WAVES; ++i) {
        const int u = wave + i * WAVES;
        const int row = 16 * u + (lane >> 2), pos = lane & 3;
        load_to_lds16(k_item + min(row, last) * 64 + 16 * (pos ^ ((row >> 2) & 3)), k_lds + u * 1024);
    }
}
template <int NT, int WAVES>
__device__ __forceinline__ void v_rows_to_lds(const int8_t *v_item, uint8_t *v_lds, int wave, int lane, int last)
{
#pragma unroll
    for (int i = 0; i < NT / WAVES; ++i) {
        const int u = wave + i * WAVES;
        const int key = 16 * u + (lane >> 2), pos = lane & 3;
        if (key <= last)
            load_to_lds16(v_item + key * 64 + 16 * (pos ^ (((key >> 4) + (key >> 2)) & 3)), v_lds + u * 1024);
        else   // the 16 bytes the load would have filled
            *(v4i *)(v_lds + u * 1024 + lane * 16) = (v4i){0, 0, 0, 0};
    }
}

// Where a lane finds its operands in LDS.
struct OperandOffsets {
    int k;      // K operand of key tile t at t*1024 + k: key 16t + qi, chunk g
    int v[4];   // V operand, chunk n16, of 64-key group T: first read at T*4096 + v[n16], second at
                // T*4096 + 2048 + v[n16 ^ 2]
};
__device__ __forceinline__ OperandOffsets operand_offsets(int lane)
{
    const int qi = lane & 15, g = lane >> 4;
    OperandOffsets off;
    off.k = qi * 64 + 16 * (g ^ ((qi >> 2) & 3));
    // The transposing read: in each group of 16 lanes, lane pair j points at the 16 bytes (chunk n16)
    // of the key of contraction slot j, the lane's half of them; lane i gets column i.  Slot j of lane
    // group g is key 16*(j >> 2) + 4g + (j & 3) of the 64-key group (first read; the second read is
    // 32 keys further, slots 8..15, and its chunk permutation is the first's ^ 2).
    const int slot = qi >> 1;
    const int v_key = 16 * (slot >> 2) + 4 * g + (slot & 3);
    const int v_f = ((slot >> 2) + g) & 3;
#pragma unroll
    for (int n16 = 0; n16 < 4; ++n16) off.v[n16] = v_key * 64 + 16 * (n16 ^ v_f) + 8 * (qi & 1);
    return off;
}

// Block-wide barrier for data that loads bring into LDS.  Every wave first waits (s_waitcnt vmcnt)
// for its own loads; the barrier then tells it that everybody else's have landed too.  No release
// fence: it would wait for every load in flight, also for those meant to overlap with arithmetic,
// and the waves write LDS by no other means.  The acquire fence keeps later LDS reads behind the
// barrier.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}
// every vector-memory operation of this wave has completed: vmcnt(0), other counters untouched
__device__ __forceinline__ void wait_vector_memory() { __builtin_amdgcn_s_waitcnt(0x0F70); }
// as above, and every LDS operation too: vmcnt(0) lgkmcnt(0)
__device__ __forceinline__ void wait_memory() { __builtin_amdgcn_s_waitcnt(0x0070); }

// The launcher lays a block out for the next multiple of 64 keys up to 512, then for 640, 768 or 896, so at most this many of the
// last key tiles can be wholly absent.
template <int NT>
constexpr int kAbsentTiles = NT >= 32 ? 7 : 3;
// whether key tile t holds a key of an item of L keys (the same for the whole wave)
template <int NT, bool PART>
__device__ __forceinline__ bool has_keys(int t, int L)
{
    return !PART || t < NT - kAbsentTiles<NT> || 16 * t < L;
}

struct HeadRule {
    int B, S, D, mult, shift, lim_lo, lim_hi;
};
__device__ __forceinline__ HeadRule head_rule(const HeadTable &table, const RequantTable &requant, int head)
{
    const int4 hp = table.e[head], rq = requant.e[head];
    return {hp.x, hp.y, hp.z, rq.x, rq.y, rq.z, rq.w};
}

// First half of a query tile: A^T tiles = K_tile . Q^T rescaled to 16-bit pairs tile by tile (the K
// operand of a tile is read from LDS one tile ahead of the contraction that uses it), row maximum,
// window clamp, sum and scores (Eq. (2), (3), (5)).  Leaves the scores in xp and 2*rho (Eq. (8)).
// PART: the item has L < 16*NT keys.  Key tiles wholly behind them are left out (wave-uniform branches) and get the
// score 0.  In the tile of the last key the slots behind it repeat that key (see k_rows_to_lds): copies of a key
// leave the maximum as it is; the sum counts the last key's clamped logit once per copy too often, which the lanes
// that hold the tile's last slot take off again; the scores of the copies meet zero rows of V.
template <int NT, int RQ, bool PART>
__device__ __forceinline__ void scores_of_tile(const uint8_t *k_lds, int k_off, const v4i &qop, const HeadRule &r,
                                               short2_t (&xp)[NT][2], uint32_t &rho2, uint32_t &p_top, int L, int g)
{
    const int round_c = 1 << (r.shift - 1);
    short2_t mx2 = {-32768, -32768};
    auto k_operand = [&](int t) { return *(const v4i *)(k_lds + t * 1024 + k_off); };
    v4i acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(k_operand(0), qop, (v4i){0, 0, 0, 0}, 0, 0, 0);
    v4i knext = k_operand(1);
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        v4i acc_next = acc;
        if (t + 1 < NT) acc_next = __builtin_amdgcn_mfma_i32_16x16x64_i8(knext, qop, (v4i){0, 0, 0, 0}, 0, 0, 0);
        if (t + 2 < NT) knext = k_operand(t + 2);
        if (has_keys<NT, PART>(t, L)) {
            rescale_tile<RQ>(acc, r.mult, r.shift, round_c, r.lim_lo, r.lim_hi, xp[t][0], xp[t][1]);
            mx2 = __builtin_elementwise_max(mx2, __builtin_elementwise_max(xp[t][0], xp[t][1]));
        }
        acc = acc_next;
        __builtin_amdgcn_sched_barrier(0);
    }
    int mx = max((int)mx2.x, (int)mx2.y);
    mx = max(mx, xor16(mx));
    mx = max(mx, xor32(mx));
    const int m = clamp_i32(mx, -128, 127);   // saturation is monotone: max of clamped = clamp of max

    const short lo = (short)max(m - r.D, -128);
    const short2_t lo2 = {lo, lo}, hi2 = {127, 127};
    const ushort2_t s2 = {(unsigned short)r.S, (unsigned short)r.S};
    const unsigned short cc = (unsigned short)(r.B - r.S * m);
    const ushort2_t c2 = {cc, cc};
    // The int8 saturation from above matters only for a query whose largest logit exceeds 127; the
    // tile takes that pass only if one of its 16 queries has such a logit.
    if (__builtin_amdgcn_ballot_w64(mx > 127) != 0) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if (has_keys<NT, PART>(t, L)) {
                xp[t][0] = __builtin_elementwise_min(xp[t][0], hi2);
                xp[t][1] = __builtin_elementwise_min(xp[t][1], hi2);
            }
        }
    }
    int last_slot = 0;   // the last slot of the tile that holds the last key (the lanes g = 3 hold it)
    short2_t sum2 = {0, 0};
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        if (has_keys<NT, PART>(t, L)) {
            if (PART && t >= NT - kAbsentTiles<NT> - 1 && 16 * t + 16 >= L) last_slot = (int)xp[t][1].y;   // the last key's tile
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const short2_t xc = __builtin_elementwise_max(xp[t][h], lo2);   // the window's lower edge, >= -128
                sum2 += xc;                            // at most 64 values of magnitude <= 128 per half
                xp[t][h] = __builtin_bit_cast(short2_t, __builtin_bit_cast(ushort2_t, xc) * s2 + c2);
            }
        } else {
            xp[t][0] = xp[t][1] = (short2_t){0, 0};
        }
    }
    int sx = (int)sum2.x + (int)sum2.y;
    if constexpr (PART) sx -= g == 3 ? (((L + 15) & ~15) - L) * clamp_i32(last_slot, (int)lo, 127) : 0;
    sx += xor16(sx);
    sx += xor32(sx);
    const uint32_t Z = (uint32_t)(L * r.B - r.S * (L * m - sx));
    rho2 = reciprocal_u8(Z) * 2u;                 // <= 65280: fits 16 bits
    p_top = ((uint32_t)r.B * rho2) >> 16;         // the row's largest probability: its maximum has the score B
}

// Second half: O^T tile = V^T . P^T.  Lane (g, qi) ends with columns 16*n16 + 4g .. +3 of query qi.
// The matrix unit multiplies signed bytes.  top (wave-uniform): some query of the tile has a probability above 127 (a
// row has at most one, its sum being at most 255), which the unit reads as P - 256.  Where a set of 64 keys holds
// such a probability for any query, the top bits then go in again as 64s, four times, into the same accumulators.
template <int NT, bool PART, bool WIDE>
__device__ __forceinline__ void weighted_values_of_tile(const uint8_t *v_lds, const int (&v_off)[4],
                                                        const short2_t (&xp)[NT][2], uint32_t rho2, v4i (&oacc)[4], int L,
                                                        bool top)
{
#pragma unroll
    for (int n16 = 0; n16 < 4; ++n16) oacc[n16] = (v4i){0, 0, 0, 0};
#pragma unroll
    for (int T = 0; T < NT / 4; ++T) {
        if (PART && T > 0 && 64 * T >= L) continue;   // 64 keys that the item lacks
        v4i vop[4];
#pragma unroll
        for (int n16 = 0; n16 < 4; ++n16) {
            const v2i a = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(v_lds + T * 4096 + v_off[n16]));
            const v2i b = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(v_lds + T * 4096 + 2048 + v_off[n16 ^ 2]));
            vop[n16] = (v4i){a[0], a[1], b[0], b[1]};
        }
        v4i pop;
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            const uint32_t s01 = __builtin_bit_cast(uint32_t, xp[T * 4 + tt][0]);
            const uint32_t s23 = __builtin_bit_cast(uint32_t, xp[T * 4 + tt][1]);
            if (!has_keys<NT, PART>(T * 4 + tt, L))
                pop[tt] = 0;
            else
                pop[tt] = (int)probabilities_plain(s01, s23, rho2);
        }
#pragma unroll
        for (int n16 = 0; n16 < 4; ++n16)
            oacc[n16] = __builtin_amdgcn_mfma_i32_16x16x64_i8(vop[n16], pop, oacc[n16], 0, 0, 0);
        if constexpr (WIDE) {
            if (top && __builtin_amdgcn_ballot_w64(((pop[0] | pop[1] | pop[2] | pop[3]) & 0x80808080) != 0) != 0) {
#pragma unroll
                for (int tt = 0; tt < 4; ++tt) pop[tt] = (int)(((uint32_t)pop[tt] & 0x80808080u) >> 1);
#pragma unroll
                for (int rep = 0; rep < 4; ++rep) {
#pragma unroll
                    for (int n16 = 0; n16 < 4; ++n16)
                        oacc[n16] = __builtin_amdgcn_mfma_i32_16x16x64_i8(vop[n16], pop, oacc[n16], 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// rows of query tile rt of an item
__device__ __forceinline__ void store_tile(int32_t *o_rows, int L, int rt, int lane, const v4i (&oacc)[4])
{
    store_rows_whole_lines<4>(o_rows + (size_t)rt * 16 * 64, 64, min(16, L - 16 * rt), lane, oacc);
}

// One block per (batch, head) item, NT / WAVES query tiles per wave.  The first contraction starts
// when K has landed; V is asked for then and lands during it.  (Measured against blocks that take a
// half or a quarter of an item's queries, and against blocks that stay and take item after item
// with the next item's loads in flight: at 768 items this form was the fastest.)
// PART: items of Lq_rows queries and Lk_rows <= 16*NT keys (else both are 16*NT); block (x, y) takes the queries from
// 16*NT*y on, 16*NT of them at most.  The rows of Q and K that a block lacks are loaded as copies of the last one and
// those of V are zero; their query rows are not stored, and a wave whose tile lies behind the block's queries only
// keeps the barriers.
// WIDE: the table does not prove P <= 127; a tile then looks at its rows' largest probabilities.
template <int NT, int RQ, int WAVES, bool PART, bool WIDE>
__global__ __launch_bounds__(64 * WAVES, (NT <= 16 ? 6 : (NT <= 32 ? 4 : 2))) void hccs_attention_direct_kernel(
    const int8_t *__restrict__ q, const int8_t *__restrict__ k, const int8_t *__restrict__ v, int32_t *__restrict__ o,
    int H, int Lq_rows, int Lk_rows, HeadTable table, RequantTable requant)
{
    constexpr int KV = NT * 16 * 64;       // bytes of K (or V) of one item in LDS
    constexpr int kTiles = NT / WAVES;     // query tiles per wave
    const int L = PART ? Lk_rows : NT * 16;
    const int q0 = PART ? (int)blockIdx.y * (NT * 16) : 0;          // the block's first query
    const int Lq = PART ? min(NT * 16, Lq_rows - q0) : NT * 16;     // and how many it has
    static_assert(NT % WAVES == 0, "equal shares of tiles and of loads");
    __shared__ __attribute__((aligned(16))) uint8_t k_lds[KV];
    __shared__ __attribute__((aligned(16))) uint8_t v_lds[KV];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int qi = lane & 15, g = lane >> 4;
    const int item = (int)blockIdx.x;
    const size_t base = (size_t)item * (size_t)(L * 64);
    const size_t q_base = ((size_t)item * (size_t)(PART ? Lq_rows : NT * 16) + (size_t)q0) * 64;

    k_rows_to_lds<NT, WAVES>(k + base, k_lds, wave, lane, L - 1);
    // the Q operands of the wave's tiles: query 16*rt + qi, bytes 16g .. 16g+15
    v4i qops[kTiles];
#pragma unroll
    for (int i = 0; i < kTiles; ++i)
        qops[i] = *(const v4i *)(q + q_base + min((wave + i * WAVES) * 16 + qi, Lq - 1) * 64 + 16 * g);
    const HeadRule rule = head_rule(table, requant, item % H);
    const OperandOffsets off = operand_offsets(lane);

    wait_vector_memory();
    // The Q registers count as arrived from here on: without this the compiler would wait for them
    // at their first use, which comes after the V loads, and its wait would cover those too.
#pragma unroll
    for (int i = 0; i < kTiles; ++i) asm volatile("" : "+v"(qops[i]));
    lds_barrier();   // K is in
    v_rows_to_lds<NT, WAVES>(v + base, v_lds, wave, lane, L - 1);

#pragma unroll
    for (int i = 0; i < kTiles; ++i) {
        const int rt = wave + i * WAVES;
        const bool has_rows = !PART || 16 * rt < Lq;   // wave-uniform
        short2_t xp[NT][2];
        uint32_t rho2 = 0, p_top = 0;
        if (has_rows) scores_of_tile<NT, RQ, PART>(k_lds, off.k, qops[i], rule, xp, rho2, p_top, L, g);
        if (i == 0) {   // the wave's first tile: V must have landed by now
            if constexpr (PART)
                wait_memory();   // and the zero rows this wave wrote
            else
                wait_vector_memory();
            lds_barrier();
        }
        if (has_rows) {
            v4i oacc[4];
            const bool top = WIDE && __builtin_amdgcn_ballot_w64(p_top > 127u) != 0;
            weighted_values_of_tile<NT, PART, WIDE>(v_lds, off.v, xp, rho2, oacc, L, top);
            store_tile(o + q_base, Lq, rt, lane, oacc);
        }
    }
}

template <int NT, bool PART, bool WIDE>
static hipError_t launch_direct_wide(const int8_t *q, const int8_t *k, const int8_t *v, int32_t *o, int64_t items, int H,
                                     int Lq, int L, const HeadTable &tab, const RequantTable &rq, int kind, hipStream_t st)
{
    // as many waves as divide the query tiles evenly, at most 8
    constexpr int WAVES = NT % 8 == 0 ? 8 : (NT % 7 == 0 ? 7 : (NT % 6 == 0 ? 6 : (NT % 5 == 0 ? 5 : 4)));
    const dim3 grid((uint32_t)items, (uint32_t)((Lq + NT * 16 - 1) / (NT * 16))), block(64 * WAVES);
    if (kind == kRescaleHigh16)
        return launch(hccs_attention_direct_kernel<NT, kRescaleHigh16, WAVES, PART, WIDE>, grid, block, st, q, k, v, o, H, Lq, L, tab, rq);
    if (kind == kRescaleShift)
        return launch(hccs_attention_direct_kernel<NT, kRescaleShift, WAVES, PART, WIDE>, grid, block, st, q, k, v, o, H, Lq, L, tab, rq);
    return launch(hccs_attention_direct_kernel<NT, kRescalePreclamp, WAVES, PART, WIDE>, grid, block, st, q, k, v, o, H, Lq, L, tab, rq);
}
template <int NT, bool PART>
static hipError_t launch_direct_nt(const int8_t *q, const int8_t *k, const int8_t *v, int32_t *o, int64_t items, int H,
                                   int Lq, int L, const HeadTable &tab, const RequantTable &rq, int kind, hipStream_t st)
{
    if (probabilities_fit_signed(tab, H, L))
        return launch_direct_wide<NT, PART, false>(q, k, v, o, items, H, Lq, L, tab, rq, kind, st);
    return launch_direct_wide<NT, PART, true>(q, k, v, o, items, H, Lq, L, tab, rq, kind, st);
}

template <int NT>
static hipError_t launch_nt(const int8_t *q, const int8_t *k, const int8_t *v, int32_t *o, int64_t blocks, int H,
                            const HeadTable &tab, const RequantTable &rq, int kind, hipStream_t st)
{
    // eight waves per block (two per SIMD) when there are at least eight query tiles
    constexpr int WAVES = NT >= 8 ? 8 : 4;
    const dim3 grid((uint32_t)blocks), block(64 * WAVES);
    if (kind == kRescaleHigh16)
        return launch(hccs_attention_kernel<NT, kRescaleHigh16, WAVES>, grid, block, st, q, k, v, o, H, tab, rq);
    if (kind == kRescaleShift)
        return launch(hccs_attention_kernel<NT, kRescaleShift, WAVES>, grid, block, st, q, k, v, o, H, tab, rq);
    return launch(hccs_attention_kernel<NT, kRescalePreclamp, WAVES>, grid, block, st, q, k, v, o, H, tab, rq);
}

// key slots of the resident block for Lk keys; 0: too many keys for it
static int attention_key_slots(int Lk)
{
    const int sets = (Lk + 63) / 64;   // of 64 keys
    return sets <= 8 ? 64 * sets : (sets <= 10 ? 640 : (sets <= 12 ? 768 : (sets <= 14 ? 896 : 0)));
}

// Whether a block of Lq queries and Lk keys (head size 64) goes to the resident kernel: its keys fit LDS.  Side by side with the streaming kernels (768 items, us, resident / streaming):
// 64 x 256 9.7 / 12.9, 197 x 256 20.0 / 33.0, 77 x 197 9.2 / 18.5, 100 x 400 18.6 / 27.0, 1 x 256 6.8 / 9.5, 16 x 384 11.1 /
// 12.5, 16 x 448 12.8 / 15.1, 250 x 500 38.4 / 47.8, 128 x 512 24.2 / 27.3; only the largest block (more than 448 keys) with
// at most four query tiles loses: 16 x 512 17.9 / 14.5, 64 x 512 19.4 / 16.8 (97 x 512 22.6 / 26.2).  Items with more queries than
// the block has key slots get several blocks: 197 x 77 12.0 / 23.4, 2048 x 64 (48 items) 7.6 / 13.8, 2048 x 512 (192 items) 60.2 / 86.2.
// Blocks of 640, 768 and 896 key slots (80, 96 and 112 KB of LDS, one block per compute unit): 513 x 513 74.0 / 107.8, 577 x 577 87.8 / 122.0,
// 640 x 640 94.5 / 118.9, 700 x 700 118.0 / 150.2, 768 x 768 139.0 / 162.8, 100 x 700 33.6 / 35.6, 2048 x 768 (192 items) 103.0 / 111.2, 800 x 800 156 / 192,
// 896 x 896 183 / 205; 1024 slots lose: 1024 x 1024 283 / 265, 2048 x 1024 (192 items) 178 / 136.
bool attention_is_resident(int Lq, int Lk)
{
    const int slots = attention_key_slots(Lk);
    return Lk >= 1 && Lq >= 1 && slots > 0 && (Lk <= 448 || Lq > 64);
}

hipError_t launch_attention(const int8_t *q, const int8_t *k, const int8_t *v, int32_t *o, int64_t Bt, int H, int Lq,
                            int L, int d, const HeadTable &tab, const RequantTable &rq_in, hipStream_t st)
{
    (void)d;   // 64, checked by the caller
    if (L < 1 || Lq < 1 || attention_key_slots(L) == 0 || (Lq + 15) / 16 > 65535 * 4) return hipErrorInvalidValue;
    RequantTable rq;
    const int kind = choose_rescale(rq_in, H, (int64_t)1 << 20, rq);   // |acc| <= 64*128*128 = 2^20
    const int64_t blocks = Bt * H;
    if (L % 64 != 0 || Lq != L || L > 512) {
        switch ((L + 63) / 64) {
            case 1: return launch_direct_nt<4, true>(q, k, v, o, blocks, H, Lq, L, tab, rq, kind, st);
            case 2: return launch_direct_nt<8, true>(q, k, v, o, blocks, H, Lq, L, tab, rq, kind, st);
            case 3: return launch_direct_nt<12, true>(q, k, v, o, blocks, H, Lq, L, tab, rq, kind, st);
            case 4: return launch_direct_nt<16, true>(q, k, v, o, blocks, H, Lq, L, tab, rq, kind, st);
            case 5: return launch_direct_nt<20, true>(q, k, v, o, blocks, H, Lq, L, tab, rq, kind, st);
            case 6: return launch_direct_nt<24, true>(q, k, v, o, blocks, H, Lq, L, tab, rq, kind, st);
            case 7: return launch_direct_nt<28, true>(q, k, v, o, blocks, H, Lq, L, tab, rq, kind, st);
            case 8: return launch_direct_nt<32, true>(q, k, v, o, blocks, H, Lq, L, tab, rq, kind, st);
            case 9:
            case 10: return launch_direct_nt<40, true>(q, k, v, o, blocks, H, Lq, L, tab, rq, kind, st);
            case 11:
            case 12: return launch_direct_nt<48, true>(q, k, v, o, blocks, H, Lq, L, tab, rq, kind, st);
            case 13:
            case 14: return launch_direct_nt<56, true>(q, k, v, o, blocks, H, Lq, L, tab, rq, kind, st);
            default: return hipErrorInvalidValue;
        }
    }
    switch (L / 16) {
        case 4: return launch_direct_nt<4, false>(q, k, v, o, blocks, H, L, L, tab, rq, kind, st);
        case 8: return launch_direct_nt<8, false>(q, k, v, o, blocks, H, L, L, tab, rq, kind, st);
        case 12: return launch_direct_nt<12, false>(q, k, v, o, blocks, H, L, L, tab, rq, kind, st);
        case 16: return launch_direct_nt<16, false>(q, k, v, o, blocks, H, L, L, tab, rq, kind, st);
        case 20: return launch_direct_nt<20, false>(q, k, v, o, blocks, H, L, L, tab, rq, kind, st);
        case 24: return launch_direct_nt<24, false>(q, k, v, o, blocks, H, L, L, tab, rq, kind, st);
        case 32: return launch_direct_nt<32, false>(q, k, v, o, blocks, H, L, L, tab, rq, kind, st);
        default: break;   // 448 keys (7 waves of 4 tiles) measured slower than the first kernel: 31.4 against 29.1 us
    }
    if (L == 448) return launch_nt<28>(q, k, v, o, blocks, H, tab, rq, kind, st);
    return hipErrorInvalidValue;
}

}  // namespace hccs
