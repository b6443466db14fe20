// Row-wise HCCS on int8 logits (Alg. 1).  Output modes: 8-bit (Sec. III-B "int8
// output path", Eq. (8)) or 16-bit (Eq. (6), (7)), each with the exact or the
// leading-bit reciprocal (Eq. (9)).  One HBM read per element and one HBM write
// of the output width; the three logical sweeps over a row (maximum, scores and
// sum, normalise) run on registers.
#include "hccs_device.h"

namespace hccs {

// Output of four elements (one dword of distances) in a 16-bit mode: two dwords.
template <int MODE>
__device__ __forceinline__ void normalise4_wide(uint32_t delta4, int B, int S, int D, uint32_t rho,
                                                uint32_t &out_lo, uint32_t &out_hi)
{
    const unsigned short negS = (unsigned short)(0 - S);
    const ushort2_t r2 = {(unsigned short)rho, (unsigned short)rho};
    ushort2_t lo = scores2(bytes_lo_pair(delta4), (unsigned short)D, negS, (unsigned short)B) * r2;
    ushort2_t hi = scores2(bytes_hi_pair(delta4), (unsigned short)D, negS, (unsigned short)B) * r2;
    if constexpr (MODE == kModeClbI16) {
        // s < 2^(k+1) and rho < 2^(15-k): the product fits 16 bits, then saturates at T
        const ushort2_t cap = {32767, 32767};
        lo = __builtin_elementwise_min(lo, cap);
        hi = __builtin_elementwise_min(hi, cap);
    }
    out_lo = __builtin_bit_cast(uint32_t, lo);
    out_hi = __builtin_bit_cast(uint32_t, hi);
}

// Leading-bit 8-bit mode: s*rho can reach 2x the exact product, so the pack trick of
// the exact path (which needs p - pmin <= 255) does not apply; plain integer form.
__device__ __forceinline__ uint32_t normalise4_clb_u8(uint32_t delta4, int B, int S, int D, uint32_t rho)
{
    const unsigned short negS = (unsigned short)(0 - S);
    const ushort2_t lo = scores2(bytes_lo_pair(delta4), (unsigned short)D, negS, (unsigned short)B);
    const ushort2_t hi = scores2(bytes_hi_pair(delta4), (unsigned short)D, negS, (unsigned short)B);
    const uint32_t p0 = scale_score<kModeClbU8>(lo.x, rho), p1 = scale_score<kModeClbU8>(lo.y, rho);
    const uint32_t p2 = scale_score<kModeClbU8>(hi.x, rho), p3 = scale_score<kModeClbU8>(hi.y, rho);
    return p0 | (p1 << 8) | (p2 << 16) | (p3 << 24);
}

// Stages 3-5 for one row once Z is known: the reciprocal of the row and the 16 output
// bytes of one vector of distances (4 dwords in the 8-bit modes, 2 in the 16-bit modes).
template <int MODE>
struct RowOutput {
    int B, S, D;
    uint32_t rho;
    RowAffine ra;
    __device__ __forceinline__ RowOutput(uint32_t Z, int B_, int S_, int D_) : B(B_), S(S_), D(D_)
    {
        if constexpr (MODE == kModeU8)
            ra = row_affine(Z, B, S, D), rho = 0;
        else
            rho = reciprocal_for_mode<MODE>(Z);
    }
    // The same constants as held by lane J of each quad (quad_perm broadcast).
    template <int J>
    __device__ __forceinline__ RowOutput from_quad_lane() const
    {
        RowOutput r = *this;
        if constexpr (MODE == kModeU8) {
            r.ra.slope = __builtin_bit_cast(float, dpp<J * 0x55>(__builtin_bit_cast(int, ra.slope)));
            r.ra.offset = __builtin_bit_cast(float, dpp<J * 0x55>(__builtin_bit_cast(int, ra.offset)));
            r.ra.pmin4 = (uint32_t)dpp<J * 0x55>((int)ra.pmin4);
        } else {
            r.rho = (uint32_t)dpp<J * 0x55>((int)rho);
        }
        return r;
    }
    __device__ __forceinline__ u32x4 vector(const uint32_t *dl) const
    {
        u32x4 o;
        if constexpr (MODE == kModeU8) {
#pragma unroll
            for (int c = 0; c < 4; ++c) o[c] = normalise4(dl[c], ra);
        } else if constexpr (MODE == kModeClbU8) {
#pragma unroll
            for (int c = 0; c < 4; ++c) o[c] = normalise4_clb_u8(dl[c], B, S, D, rho);
        } else {
            uint32_t w[4];
#pragma unroll
            for (int c = 0; c < 2; ++c) normalise4_wide<MODE>(dl[c], B, S, D, rho, w[2 * c], w[2 * c + 1]);
            o = (u32x4){w[0], w[1], w[2], w[3]};
        }
        return o;
    }
};

// Stage 1 of a lane's share of a row (Alg. 1, first step): the maximum of its V x DW dwords of
// int8 bytes; the caller reduces it over the lanes that share the row.
template <int V, int DW>
__device__ __forceinline__ int lane_max(const uint32_t (&d)[V][DW])
{
    ByteMax bm;
    bm.init(d[0][0]);
#pragma unroll
    for (int c = 1; c < DW; ++c) bm.add(d[0][c]);
#pragma unroll
    for (int v = 1; v < V; ++v)
#pragma unroll
        for (int c = 0; c < DW; ++c) bm.add(d[v][c]);
    return bm.result();
}

// Stage 2: the bytes become their unclamped distances to the row maximum m, and the lane's
// part of (sum delta - sum |delta - D|) is returned; over a row of `count` slots
// sum min(delta, D) = (sum delta + count*D - sum |delta - D|) / 2: two byte-SAD accumulations.
template <int V, int DW>
__device__ __forceinline__ int lane_distances(uint32_t (&d)[V][DW], int m, int D)
{
    const uint32_t D4 = (uint32_t)D * 0x01010101u;
    const uint32_t neg_base4 = 0u - (uint32_t)(127 - m) * 0x01010101u;
    uint32_t acc_d = 0, acc_abs = 0;
#pragma unroll
    for (int v = 0; v < V; ++v)
#pragma unroll
        for (int c = 0; c < DW; ++c) {
            const uint32_t dl = distance4(d[v][c], neg_base4);
            d[v][c] = dl;
            acc_d = __builtin_amdgcn_sad_u8(dl, 0u, acc_d);
            acc_abs = __builtin_amdgcn_sad_u8(dl, D4, acc_abs);
        }
    return (int)acc_d - (int)acc_abs;
}

// Sum of the clamped distances of the n real elements of a row held in `slots` byte slots: the
// slots that are not elements hold -128, whose distance m + 128 is taken out again.
__device__ __forceinline__ int clamped_sum(int t, int slots, int n, uint32_t mu, int D)
{
    return (t + slots * D) / 2 - (slots - n) * (int)min(mu, (uint32_t)D);
}

// ---------------------------------------------------------------------------
// Register-resident kernel for rows whose length is a multiple of 16.
//
// A row is shared by G adjacent lanes (G a power of two, 4..64); each lane holds V
// vectors of it, vector number v*G + lane_in_group, so one load instruction of a
// group covers G contiguous vectors.  A vector is 16 input bytes in the 8-bit modes
// and 8 input bytes in the 16-bit modes, i.e. always 16 output bytes: every store
// instruction of a group writes G*16 contiguous bytes.  A wave works on R batches
// of 64/G rows at once (R*V loads in flight per lane).  The grid is (row tiles, H,
// B): a block never straddles heads, so the head's constants are wave-uniform.
//
// Vectors past the end of a short row, and rows past the end of the slab, are
// replaced by the byte -128: that is the identity of the maximum, and its
// distance to the maximum is (m + 128), a known amount that is taken out of
// the sum again.
// ---------------------------------------------------------------------------
template <int G, int V, int R, int WPB, int MODE>
__global__ __launch_bounds__(64 * WPB) void hccs_rows_kernel(const int8_t *__restrict__ logits,
                                                             uint8_t *__restrict__ out, int Lq, int nvec,
                                                             BlockPlace place, HeadTable table)
{
    constexpr int kRowsPerBatch = 64 / G;
    constexpr int kRowsPerWave = R * kRowsPerBatch;
    constexpr int kOutBytes = (MODE & 1) ? 2 : 1;   // bytes per output element
    constexpr int DW = 4 / kOutBytes;               // dwords per input vector
    constexpr int kVecBytes = DW * 4;
    constexpr int kPaddedLen = G * V * kVecBytes;

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int sub = lane % G;        // position inside the row's lane group
    const int grp = lane / G;        // row inside the batch
    uint32_t tile, head, slab_no;
    place.locate(tile, head, slab_no);
    const int4 hp = table.e[head];
    const int B = hp.x, S = hp.y, D = hp.z;
    const int n = nvec * kVecBytes;

    const size_t slab = (size_t)slab_no * (size_t)Lq;
    const int wave_row0 = ((int)tile * WPB + wave) * kRowsPerWave;
    if (wave_row0 >= Lq) return;   // whole wave past the slab
    const int row0 = wave_row0 + grp;

    uint32_t d[R][V][DW];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const int row = row0 + j * kRowsPerBatch;
        const int8_t *src = logits + (slab + row) * (size_t)n;
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const int vi = v * G + sub;
            if (row < Lq && vi < nvec) {
                if constexpr (DW == 4) {
                    const u32x4 t = load_stream(src + vi * 16);
                    d[j][v][0] = t[0], d[j][v][1] = t[1], d[j][v][2] = t[2], d[j][v][3] = t[3];
                } else {
                    const u32x2 t = load_stream8(src + vi * 8);
                    d[j][v][0] = t[0], d[j][v][1] = t[1];
                }
            } else {
#pragma unroll
                for (int c = 0; c < DW; ++c) d[j][v][c] = kPadWord;
            }
        }
    }

    int tsum[R];                       // sum delta - sum |delta - D| of each batch's row
    uint32_t mu[R];                    // row maximum in offset-binary form
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const int m = group_max<G>(lane_max(d[j]));
        mu[j] = (uint32_t)(m + 128);
        tsum[j] = group_sum<G>(lane_distances(d[j], m, D));
    }

    // stages 3-5: Z = n*B - S*sum min(delta, D)  (Eq. (3), (5)), reciprocal, normalise.
    // Every lane of a group holds the sums of all R rows the group works on.  With R = 2 or 4
    // lane i of each quad takes row i % R, so the reciprocal and the row constants are computed
    // once per R rows instead of R times, and come back through quad broadcasts.
    auto row_output = [&](int t, uint32_t mu_) {
        return RowOutput<MODE>((uint32_t)(n * B - S * clamped_sum(t, kPaddedLen, n, mu_, D)), B, S, D);
    };
    auto emit = [&](int j, const RowOutput<MODE> &ro) {
        const int row = row0 + j * kRowsPerBatch;
        uint8_t *dst = out + (slab + row) * (size_t)n * kOutBytes;
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const int vi = v * G + sub;
            const u32x4 o = ro.vector(d[j][v]);
            if (row < Lq && vi < nvec) store_stream(dst + vi * 16, o);
        }
    };
    if constexpr (R == 2) {
        const bool odd = lane & 1;
        const RowOutput<MODE> mine = row_output(odd ? tsum[1] : tsum[0], odd ? mu[1] : mu[0]);
        emit(0, mine.template from_quad_lane<0>());
        emit(1, mine.template from_quad_lane<1>());
    } else if constexpr (R == 4) {
        const int w = lane & 3;
        const int t = w == 0 ? tsum[0] : (w == 1 ? tsum[1] : (w == 2 ? tsum[2] : tsum[3]));
        const uint32_t u = w == 0 ? mu[0] : (w == 1 ? mu[1] : (w == 2 ? mu[2] : mu[3]));
        const RowOutput<MODE> mine = row_output(t, u);
        emit(0, mine.template from_quad_lane<0>());
        emit(1, mine.template from_quad_lane<1>());
        emit(2, mine.template from_quad_lane<2>());
        emit(3, mine.template from_quad_lane<3>());
    } else {
#pragma unroll
        for (int j = 0; j < R; ++j) emit(j, row_output(tsum[j], mu[j]));
    }
}

// ---------------------------------------------------------------------------
// One block (four waves) per row, for rows beyond a wave's registers (16384 < Lk <= 65536):
// thread t holds vectors t, t + 256, ...; the maximum and the sum cross waves through LDS.
// Same arithmetic and the same padding rule as the kernel above.
// ---------------------------------------------------------------------------
template <int V, int MODE>
__global__ __launch_bounds__(256) void hccs_row_block_kernel(const int8_t *__restrict__ logits,
                                                             uint8_t *__restrict__ out, int Lq, int nvec,
                                                             BlockPlace place, HeadTable table)
{
    constexpr int kOutBytes = (MODE & 1) ? 2 : 1;
    constexpr int DW = 4 / kOutBytes;
    constexpr int kVecBytes = DW * 4;
    constexpr int kPaddedLen = 256 * V * kVecBytes;
    __shared__ int red[2][4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t tile, head, slab_no;   // one block per row: the tile is the row inside the slab
    place.locate(tile, head, slab_no);
    const int4 hp = table.e[head];
    const int B = hp.x, S = hp.y, D = hp.z;
    const int n = nvec * kVecBytes;
    const size_t row = (size_t)slab_no * (size_t)Lq + tile;
    const int8_t *src = logits + row * (size_t)n;
    uint8_t *dst = out + row * (size_t)n * kOutBytes;

    uint32_t d[V][DW];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int vi = v * 256 + tid;
        if (vi < nvec) {
            if constexpr (DW == 4) {
                const u32x4 t = load_stream(src + vi * 16);
                d[v][0] = t[0], d[v][1] = t[1], d[v][2] = t[2], d[v][3] = t[3];
            } else {
                const u32x2 t = load_stream8(src + vi * 8);
                d[v][0] = t[0], d[v][1] = t[1];
            }
        } else {
#pragma unroll
            for (int c = 0; c < DW; ++c) d[v][c] = kPadWord;
        }
    }
    int m = group_max<64>(lane_max(d));
    if (lane == 0) red[0][wave] = m;
    __syncthreads();
    m = max(max(red[0][0], red[0][1]), max(red[0][2], red[0][3]));
    const uint32_t mu = (uint32_t)(m + 128);

    int t = group_sum<64>(lane_distances(d, m, D));
    if (lane == 0) red[1][wave] = t;
    __syncthreads();
    t = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    const int sum_clamped = clamped_sum(t, kPaddedLen, n, mu, D);
    const uint32_t Z = (uint32_t)(n * B - S * sum_clamped);
    const RowOutput<MODE> ro(Z, B, S, D);
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int vi = v * 256 + tid;
        const u32x4 o = ro.vector(d[v]);
        if (vi < nvec) store_stream(dst + vi * 16, o);
    }
}

// ---------------------------------------------------------------------------
// Rows of any length on 16-byte aligned tensors: row r starts at byte r*n of the input, which
// is aligned to an input vector only when n is a multiple of the vector size VB (16 bytes in the
// 8-bit modes, 8 bytes in the 16-bit modes, so that an output vector is 16 bytes in both).  A
// lane group loads the ALIGNED vectors that cover the row; bytes of the first and last vector
// that belong to the neighbouring rows are overwritten with -128 before use, i.e. they become
// padding (identity of the maximum, known distance, taken out of the sum like every other pad).
// Element positions are kept, so a lane's result is an aligned 16-byte vector of the output as
// well, and one set of masks serves both.
//
// Interior vectors are stored whole.  The vector in which one row ends and the next begins is
// put together inside the block: the upper row leaves its part of it in LDS, the lower row's
// first lane adds its own and stores the whole vector.  Rows are numbered through the whole
// tensor (the head comes from the row number), a block owns 4*(64/G) consecutive rows, and
// that is a multiple of 16 rows whenever G <= 16: then every block begins and ends on a vector
// boundary.  Only where it does not (longer rows of odd length, the end of the tensor) the
// first and last vector of a block are stored element by element, in branches that whole waves
// skip.  With LONG = false (rows shorter than a vector, which can then hold several rows) every
// boundary vector is stored element by element instead.
// ---------------------------------------------------------------------------
template <int G, int V, int MODE, bool LONG>
__global__ __launch_bounds__(256) void hccs_rows_ragged_kernel(const int8_t *__restrict__ logits,
                                                               uint8_t *__restrict__ out, uint32_t rows,
                                                               uint32_t first, FastDiv by_Lq, FastDiv by_H, int n,
                                                               HeadTable table)
{
    // `logits` and `out` are the tensors' base addresses rounded down to a vector boundary; the
    // tensor's first element sits `first` input bytes (elements) behind them in both.
    constexpr int kOutBytes = (MODE & 1) ? 2 : 1;   // bytes per output element
    constexpr int DW = 4 / kOutBytes;               // dwords per input vector
    constexpr int VB = DW * 4;                      // bytes per input vector
    constexpr int kRowsPerWave = 64 / G;
    constexpr int kRowsPerBlock = 4 * kRowsPerWave;
    constexpr int kPaddedLen = G * V * VB;
    __shared__ int4 lds_table[64];
    __shared__ __attribute__((aligned(16))) u32x4 lds_tail[kRowsPerBlock];
    __shared__ __attribute__((aligned(16))) u32x4 lds_low[VB + 1];   // entry c: the low c input bytes of a vector set
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane % G, grp = lane / G;
    if (tid < 64) lds_table[tid] = table.e[tid];
    if (tid >= 64 && tid < 64 + VB + 1) {
        const int c = tid - 64;
        u32x4 mk = {0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < DW; ++j) {
            const int cj = c - 4 * j;
            mk[j] = cj >= 4 ? 0xffffffffu : (cj <= 0 ? 0u : ((1u << (8 * cj)) - 1u));
        }
        lds_low[c] = mk;
    }
    __syncthreads();

    const int rib = wave * kRowsPerWave + grp;                  // row inside the block
    const uint32_t row_raw = blockIdx.x * (uint32_t)kRowsPerBlock + (uint32_t)rib;
    const bool live = row_raw < rows;
    const uint32_t row = live ? row_raw : 0;
    const uint32_t slab = by_Lq.quotient(row);
    const int4 hp = lds_table[slab - by_H.quotient(slab) * by_H.divisor];
    const int B = hp.x, S = hp.y, D = hp.z;
    const size_t total = (size_t)first + (size_t)rows * (size_t)n;   // end of the tensor
    const size_t begin = (size_t)first + (size_t)row * (size_t)n;    // first byte of the row in the input
    const size_t base = begin & ~(size_t)(VB - 1);        // aligned start of the covering vectors
    const int lo = (int)(begin - base), hi = lo + n;      // the row is bytes [lo, hi) relative to base
    const int nspan = (hi + VB - 1) / VB;                 // vectors that touch the row

    // input bytes of vector vi that belong to the row: offsets k of the span with lo <= k < hi
    struct Mask {
        uint32_t w[DW];
    };
    auto own_bytes = [&](int vi) -> Mask {
        const u32x4 below = lds_low[min(max(lo - VB * vi, 0), VB)], upto = lds_low[min(max(hi - VB * vi, 0), VB)];
        Mask mk;
#pragma unroll
        for (int c = 0; c < DW; ++c) mk.w[c] = upto[c] & ~below[c];
        return mk;
    };
    // the same as a mask over the 16 output bytes of the vector
    auto own_out = [&](int vi) -> u32x4 {
        const Mask mk = own_bytes(vi);
        if constexpr (DW == 4) {
            return (u32x4){mk.w[0], mk.w[1], mk.w[2], mk.w[3]};
        } else {
            return (u32x4){__builtin_amdgcn_perm(mk.w[0], mk.w[0], 0x01010000u),
                           __builtin_amdgcn_perm(mk.w[0], mk.w[0], 0x03030202u),
                           __builtin_amdgcn_perm(mk.w[1], mk.w[1], 0x01010000u),
                           __builtin_amdgcn_perm(mk.w[1], mk.w[1], 0x03030202u)};
        }
    };

    uint32_t d[V][DW];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int vi = v * G + sub;
        if (live && vi < nspan) {
            const size_t at = base + (size_t)vi * VB;
            if (at >= first && at + VB <= total) {
                if constexpr (DW == 4) {
                    const u32x4 t = load_stream(logits + at);
                    d[v][0] = t[0], d[v][1] = t[1], d[v][2] = t[2], d[v][3] = t[3];
                } else {
                    const u32x2 t = load_stream8(logits + at);
                    d[v][0] = t[0], d[v][1] = t[1];
                }
            } else {                                      // the tensor begins or ends inside this vector: no read outside it
#pragma unroll
                for (int c = 0; c < DW; ++c) {
                    uint32_t w = 0;
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const size_t k = at + 4 * c + b;
                        w |= (uint32_t)(k >= first && k < total ? (uint8_t)logits[k] : 0x80u) << (8 * b);
                    }
                    d[v][c] = w;
                }
            }
            if (vi == 0 || vi == nspan - 1) {             // boundary vectors: foreign bytes become padding
                const Mask mk = own_bytes(vi);
#pragma unroll
                for (int c = 0; c < DW; ++c) d[v][c] = (d[v][c] & mk.w[c]) | (kPadWord & ~mk.w[c]);
            }
        } else {
#pragma unroll
            for (int c = 0; c < DW; ++c) d[v][c] = kPadWord;
        }
    }

    const int m = group_max<G>(lane_max(d));
    const uint32_t mu = (uint32_t)(m + 128);
    const int t = group_sum<G>(lane_distances(d, m, D));
    const RowOutput<MODE> ro((uint32_t)(n * B - S * clamped_sum(t, kPaddedLen, n, mu, D)), B, S, D);

    // own elements of a boundary vector, one at a time
    auto store_elements = [&](uint8_t *dst, const u32x4 &o, int vi) {
#pragma unroll
        for (int e = 0; e < VB; ++e) {
            const int kk = VB * vi + e;                   // input byte = element number
            if (kk >= lo && kk < hi) {
                if constexpr (kOutBytes == 1)
                    dst[e] = (uint8_t)(o[e >> 2] >> (8 * (e & 3)));
                else
                    ((uint16_t *)dst)[e] = (uint16_t)(o[e >> 1] >> (16 * (e & 1)));
            }
        }
    };
    // the row's last vector is shared with the next row, which is in this block and exists
    const bool tail_shared = (hi % VB) != 0;
    const bool tail_to_lds = LONG && live && tail_shared && rib + 1 < kRowsPerBlock && row_raw + 1 < rows;
    const bool head_shared = lo != 0;
    const bool head_from_lds = LONG && live && head_shared && rib > 0;
    u32x4 head_o = {0, 0, 0, 0};
    uint8_t *out_base = out + base * kOutBytes;
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int vi = v * G + sub;
        if (!live || vi >= nspan) continue;
        u32x4 o = ro.vector(d[v]);
        uint8_t *dst = out_base + (size_t)vi * 16;
        if (VB * vi >= lo && VB * vi + VB <= hi) {
            store_stream(dst, o);
        } else if (v == 0 && vi == 0 && head_from_lds) {
            const u32x4 mk = own_out(0);
#pragma unroll
            for (int c = 0; c < 4; ++c) head_o[c] = o[c] & mk[c];   // finished after the barrier
        } else if (vi == nspan - 1 && tail_to_lds) {
            const u32x4 mk = own_out(vi);
#pragma unroll
            for (int c = 0; c < 4; ++c) o[c] &= mk[c];
            lds_tail[rib] = o;
        } else {
            store_elements(dst, o, vi);
        }
    }
    if constexpr (LONG) {
        __syncthreads();
        if (sub == 0 && head_from_lds) {
            const u32x4 above = lds_tail[rib - 1];
            store_stream(out_base, (u32x4){head_o[0] | above[0], head_o[1] | above[1], head_o[2] | above[2],
                                           head_o[3] | above[3]});
        }
    }
}

// ---------------------------------------------------------------------------
// One block per row, any length and alignment: the plain integer form of
// Alg. 1 with byte accesses.  Slow; it exists so that every admissible shape
// has a path.  Three passes over the row (the second and third re-read it
// through the caches), LDS for the cross-wave maximum and sum.
// ---------------------------------------------------------------------------
template <int MODE>
__global__ __launch_bounds__(256) void hccs_row_bytes_kernel(const int8_t *__restrict__ logits,
                                                             uint8_t *__restrict__ out, int Lq, int n,
                                                             BlockPlace place, HeadTable table)
{
    __shared__ int red[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t tile, head, slab_no;   // one block per row: the tile is the row inside the slab
    place.locate(tile, head, slab_no);
    const int4 hp = table.e[head];
    const int B = hp.x, S = hp.y, D = hp.z;
    const size_t row = (size_t)slab_no * (size_t)Lq + tile;
    const int8_t *x = logits + row * (size_t)n;

    int m = -128;
    for (int i = threadIdx.x; i < n; i += 256) m = max(m, (int)x[i]);
    m = group_max<64>(m);
    if (lane == 0) red[wave] = m;
    __syncthreads();
    m = max(max(red[0], red[1]), max(red[2], red[3]));
    __syncthreads();

    int z = 0;
    for (int i = threadIdx.x; i < n; i += 256) z += B - S * min(m - (int)x[i], D);
    z = group_sum<64>(z);
    if (lane == 0) red[wave] = z;
    __syncthreads();
    const uint32_t Z = (uint32_t)(red[0] + red[1] + red[2] + red[3]);
    const uint32_t rho = reciprocal_for_mode<MODE>(Z);
    // 8-bit modes: every thread reads only the bytes it later overwrites, so in-place use is safe
    for (int i = threadIdx.x; i < n; i += 256) {
        const uint32_t s = (uint32_t)(B - S * min(m - (int)x[i], D));
        const uint32_t p = scale_score<MODE>(s, rho);
        if constexpr (MODE & 1)
            ((uint16_t *)out)[row * (size_t)n + i] = (uint16_t)p;
        else
            out[row * (size_t)n + i] = (uint8_t)p;
    }
}

__global__ void reciprocal_kernel(const uint32_t *z, uint32_t *rho, int64_t count)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) rho[i] = reciprocal_u8(z[i]);
}

// Test hook: the normalise stage alone.  Entry i has constants (B, S, Dmax) and a row sum Z; the
// 256 output bytes are p(delta) for delta = 0..255 through the same row_affine / normalise4 path
// as the row kernel.
__global__ __launch_bounds__(64) void normalise_table_kernel(const int4 *__restrict__ bsdz, uint32_t *__restrict__ out,
                                                             int64_t count)
{
    const int64_t i = blockIdx.x;
    if (i >= count) return;
    const int4 e = bsdz[i];
    const RowAffine ra = row_affine((uint32_t)e.w, e.x, e.y, e.z);
    const uint32_t d0 = threadIdx.x * 4u;
    out[i * 64 + threadIdx.x] = normalise4(d0 | ((d0 + 1) << 8) | ((d0 + 2) << 16) | ((d0 + 3) << 24), ra);
}

__global__ __launch_bounds__(256) void copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst,
                                                   int64_t count)
{
    // four vectors per lane, each a fully coalesced 4 KiB block-wide access
    const int64_t base = (int64_t)blockIdx.x * 1024 + threadIdx.x;
    u32x4 v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
        if (base + k * 256 < count) v[k] = load_stream(src + base + k * 256);
#pragma unroll
    for (int k = 0; k < 4; ++k)
        if (base + k * 256 < count) store_stream(dst + base + k * 256, v[k]);
}

// ---------------------------------------------------------------------------
// host side: choose the lane-group shape for a row length
// ---------------------------------------------------------------------------
template <int G, int V, int R, int WPB = 4, int MODE = kModeU8>
static hipError_t launch_rows(const int8_t *x, uint8_t *p, int64_t Bt, int H, int Lq, int nvec,
                              const HeadTable &tab, hipStream_t st)
{
    constexpr int kRowsPerBlock = WPB * R * (64 / G);
    dim3 grid;
    const BlockPlace place = place_blocks((Lq + kRowsPerBlock - 1) / kRowsPerBlock, H, Bt, grid);
    return launch(hccs_rows_kernel<G, V, R, WPB, MODE>, grid, dim3(64 * WPB), st, x, p, Lq, nvec, place, tab);
}

template <int MODE>
static hipError_t launch_mode(const int8_t *x, uint8_t *p, int64_t Bt, int H, int Lq, int Lk, const HeadTable &tab,
                              bool vector_ok, hipStream_t st)
{
    if (vector_ok && Lk % ((MODE & 1) ? 8 : 16) == 0 && Lk <= 16384) {
        // Lane-group width G: a power of two that covers the row with one or two vectors
        // per lane, so that each load/store instruction touches G contiguous vectors of a
        // row; beyond 128 vectors the row takes V vectors per lane of a whole wave.  Few rows
        // in flight per wave (R) and many waves measured faster than the reverse.
        const int nvec = Lk / ((MODE & 1) ? 8 : 16);
        if (nvec <= 4) return launch_rows<4, 1, 2, 4, MODE>(x, p, Bt, H, Lq, nvec, tab, st);
        if (nvec <= 8) return launch_rows<8, 1, 2, 4, MODE>(x, p, Bt, H, Lq, nvec, tab, st);
        if (nvec <= 16) return launch_rows<16, 1, 2, 4, MODE>(x, p, Bt, H, Lq, nvec, tab, st);
        if (nvec <= 32) return launch_rows<16, 2, 1, 4, MODE>(x, p, Bt, H, Lq, nvec, tab, st);
        if (nvec <= 64) return launch_rows<32, 2, 1, 4, MODE>(x, p, Bt, H, Lq, nvec, tab, st);   // measured against <64,1,2>: up to 20 % faster below 48 vectors, equal at 64
        if (nvec <= 128) return launch_rows<64, 2, 1, 4, MODE>(x, p, Bt, H, Lq, nvec, tab, st);
        if (nvec <= 256) return launch_rows<64, 4, 1, 4, MODE>(x, p, Bt, H, Lq, nvec, tab, st);
        if (nvec <= 512) return launch_rows<64, 8, 1, 4, MODE>(x, p, Bt, H, Lq, nvec, tab, st);
        if (nvec <= 1024) return launch_rows<64, 16, 1, 4, MODE>(x, p, Bt, H, Lq, nvec, tab, st);
        return launch_rows<64, 32, 1, 4, MODE>(x, p, Bt, H, Lq, nvec, tab, st);   // 16-bit modes, 8192 < Lk <= 16384
    }
    {
        // Ragged row length, or tensors that begin inside a vector at matching offsets (element e
        // of the input `first` bytes behind a vector boundary, element e of the output behind a
        // 16-byte boundary by as many elements): aligned vectors over each row's span.
        constexpr int VB = (MODE & 1) ? 8 : 16;   // input bytes per vector
        constexpr int kOutBytes = (MODE & 1) ? 2 : 1;
        const int64_t rows = Bt * H * Lq;
        const uint32_t first = (uint32_t)((uintptr_t)x % VB);
        const bool matching = (uintptr_t)p % 16 == (uintptr_t)first * kOutBytes;
        if (matching && Lk <= 16384 - 32) {
            // widest span of a row over aligned vectors: rows start at first + multiples of gcd(Lk, VB)
            const int step = (Lk & -Lk & (VB - 1)) ? (Lk & -Lk & (VB - 1)) : VB;
            const int nspan = (VB - step + (int)(first % step) + Lk + VB - 1) / VB;
            const int8_t *x_al = x - first;
            uint8_t *p_al = p - first * kOutBytes;
#define HCCS_LAUNCH_RAGGED(G_, V_, LONG_)                                                                    \
    {                                                                                                      \
        const int64_t per_block = 4 * (64 / G_);                                                           \
        return launch(hccs_rows_ragged_kernel<G_, V_, MODE, LONG_>,                                         \
                      dim3((uint32_t)((rows + per_block - 1) / per_block)), dim3(256), st, x_al, p_al,      \
                      (uint32_t)rows, first, make_fast_div((uint32_t)Lq), make_fast_div((uint32_t)H), Lk,   \
                      tab);                                                                                 \
    }
            if (Lk < VB) HCCS_LAUNCH_RAGGED(4, 1, false)
            if (nspan <= 4) HCCS_LAUNCH_RAGGED(4, 1, true)
            if (nspan <= 8) HCCS_LAUNCH_RAGGED(8, 1, true)
            // measured: two vectors per lane in a narrower group beat one per lane in a wide,
            // half-empty one (the per-row index and mask work is shared by more payload)
            if (nspan <= 12) HCCS_LAUNCH_RAGGED(8, 2, true)
            if (nspan <= 16) HCCS_LAUNCH_RAGGED(16, 1, true)
            if (nspan <= 32) HCCS_LAUNCH_RAGGED(16, 2, true)
            if (nspan <= 64) HCCS_LAUNCH_RAGGED(32, 2, true)
            if (nspan <= 128) HCCS_LAUNCH_RAGGED(32, 4, true)
            if (nspan <= 256) HCCS_LAUNCH_RAGGED(64, 4, true)
            if (nspan <= 512) HCCS_LAUNCH_RAGGED(64, 8, true)
            if (nspan <= 1024) HCCS_LAUNCH_RAGGED(64, 16, true)
            HCCS_LAUNCH_RAGGED(64, 32, true)
#undef HCCS_LAUNCH_RAGGED
        }
    }
    dim3 grid;
    const BlockPlace place = place_blocks(Lq, H, Bt, grid);   // one block per row
    if (vector_ok && Lk % 16 == 0) {   // 16384 < Lk <= 65536: one block per row, the row in the block's registers
        const int nvec = Lk / ((MODE & 1) ? 8 : 16);
        if (nvec <= 2048) return launch(hccs_row_block_kernel<8, MODE>, grid, dim3(256), st, x, p, Lq, nvec, place, tab);
        // at most 4096: Lk <= 65536 in the 8-bit modes, and the 16-bit modes need Lk*B <= 32767
        return launch(hccs_row_block_kernel<16, MODE>, grid, dim3(256), st, x, p, Lq, nvec, place, tab);
    }
    return launch(hccs_row_bytes_kernel<MODE>, grid, dim3(256), st, x, p, Lq, Lk, place, tab);
}

hipError_t launch_softmax(const int8_t *x, void *out, int64_t Bt, int H, int Lq, int Lk, const HeadTable &tab,
                          int mode, bool vector_ok, hipStream_t st)
{
    if (Bt == 0 || Lq == 0) return hipSuccess;
    uint8_t *p = (uint8_t *)out;
    switch (mode) {
        case kModeU8: return launch_mode<kModeU8>(x, p, Bt, H, Lq, Lk, tab, vector_ok, st);
        case kModeI16: return launch_mode<kModeI16>(x, p, Bt, H, Lq, Lk, tab, vector_ok, st);
        case kModeClbU8: return launch_mode<kModeClbU8>(x, p, Bt, H, Lq, Lk, tab, vector_ok, st);
        case kModeClbI16: return launch_mode<kModeClbI16>(x, p, Bt, H, Lq, Lk, tab, vector_ok, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_reciprocal(const uint32_t *z, uint32_t *rho, int64_t count, hipStream_t st)
{
    if (count == 0) return hipSuccess;
    return launch(reciprocal_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), st, z, rho, count);
}

hipError_t launch_normalise_table(const int32_t *bsdz, uint8_t *out, int64_t count, hipStream_t st)
{
    if (count == 0) return hipSuccess;
    return launch(normalise_table_kernel, dim3((unsigned)count), dim3(64), st, (const int4 *)bsdz, (uint32_t *)out,
                  count);
}

hipError_t launch_copy(const void *src, void *dst, int64_t bytes, hipStream_t st)
{
    const int64_t count = bytes / 16;
    if (count == 0) return hipSuccess;
    return launch(copy_kernel, dim3((unsigned)((count + 1023) / 1024)), dim3(256), st, (const u32x4 *)src,
                  (u32x4 *)dst, count);
}

}  // namespace hccs
