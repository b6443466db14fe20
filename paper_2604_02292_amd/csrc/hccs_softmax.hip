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
// Vector access at any byte address.  The unaligned-access mode of this target lets a 16-byte
// (8-, 4-, 2-byte) global access start at any byte; the under-aligned pointee types below tell
// the compiler so, and it still emits one global_load/store_dwordx4 (x2, dword, short) for them.
// ---------------------------------------------------------------------------
typedef u32x4 __attribute__((aligned(1))) u32x4_any;
typedef u32x2 __attribute__((aligned(1))) u32x2_any;
typedef uint32_t __attribute__((aligned(1))) u32_any;
typedef uint16_t __attribute__((aligned(1))) u16_any;

// One input vector (DW dwords) of a row.  ANY = false: the address is a multiple of the vector
// size.  ANY = true: any address.
template <int DW, bool ANY>
__device__ __forceinline__ void load_vector(const int8_t *p, uint32_t (&d)[DW])
{
    if constexpr (DW == 4) {
        u32x4 t;
        if constexpr (ANY) t = __builtin_nontemporal_load((const u32x4_any *)p);
        else t = load_stream(p);
        d[0] = t[0], d[1] = t[1], d[2] = t[2], d[3] = t[3];
    } else {
        u32x2 t;
        if constexpr (ANY) t = __builtin_nontemporal_load((const u32x2_any *)p);
        else t = load_stream8(p);
        d[0] = t[0], d[1] = t[1];
    }
}
// The last `count` input bytes of the tensor, one by one (the one vector that would reach past
// the tensor's end); the other bytes become padding.
template <int DW>
__device__ __forceinline__ void load_vector_bytes(const int8_t *p, int count, uint32_t (&d)[DW])
{
#pragma unroll
    for (int c = 0; c < DW; ++c) {
        uint32_t w = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) w |= (uint32_t)(4 * c + b < count ? (uint8_t)p[4 * c + b] : 0x80u) << (8 * b);
        d[c] = w;
    }
}
template <bool ANY>
__device__ __forceinline__ void store_vector(uint8_t *p, u32x4 o)
{
    if constexpr (ANY) __builtin_nontemporal_store(o, (u32x4_any *)p);
    else store_stream(p, o);
}
// The first `bytes` (1..15, the same in every lane that gets here) bytes of an output vector, as
// at most four stores of 8, 4, 2 and 1 bytes.
__device__ __forceinline__ void store_vector_head(uint8_t *p, u32x4 o, int bytes)
{
    if (bytes & 8) {
        __builtin_nontemporal_store((u32x2){o[0], o[1]}, (u32x2_any *)p);
        o[0] = o[2], o[1] = o[3], p += 8;
    }
    if (bytes & 4) {
        __builtin_nontemporal_store(o[0], (u32_any *)p);
        o[0] = o[1], p += 4;
    }
    if (bytes & 2) {
        __builtin_nontemporal_store((uint16_t)o[0], (u16_any *)p);
        o[0] >>= 16, p += 2;
    }
    if (bytes & 1) __builtin_nontemporal_store((uint8_t)o[0], p);
}

// What a lane has to know about the row's last vector when the row length is not a multiple of
// the vector size (RAGGED kernels).  It is the same for every row, so it is worked out once per
// lane: `tail_elems` elements of vector `last_vec` exist, the other byte slots are padding.
template <int DW>
struct RowTail {
    int last_vec, tail_elems;   // tail_elems in 1..VB (VB: the last vector is whole)
    uint32_t keep[DW];          // byte mask of the existing elements of the last vector
    __device__ __forceinline__ RowTail(int n, int nvec) : last_vec(nvec - 1), tail_elems(n - (nvec - 1) * DW * 4)
    {
#pragma unroll
        for (int c = 0; c < DW; ++c) {
            const int left = tail_elems - 4 * c;
            keep[c] = left >= 4 ? 0xffffffffu : (left <= 0 ? 0u : ((1u << (8 * left)) - 1u));
        }
    }
    __device__ __forceinline__ void pad(uint32_t (&d)[DW]) const
    {
#pragma unroll
        for (int c = 0; c < DW; ++c) d[c] = (d[c] & keep[c]) | (kPadWord & ~keep[c]);
    }
};

// ---------------------------------------------------------------------------
// Register-resident kernel.
//
// A row is shared by G adjacent lanes (G a power of two, 4..64); each lane holds V
// vectors of it, vector number v*G + lane_in_group, so one load instruction of a
// group covers G contiguous vectors.  A vector is 16 input bytes in the 8-bit modes
// and 8 input bytes in the 16-bit modes, i.e. always 16 output bytes: every store
// instruction of a group writes G*16 contiguous bytes.  A wave works on R batches
// of 64/G rows at once (R*V loads in flight per lane).  A block never straddles
// heads, so the head's constants are wave-uniform.
//
// Vectors past the end of a short row, and rows past the end of the slab, are
// replaced by the byte -128: that is the identity of the maximum, and its
// distance to the maximum is (m + 128), a known amount that is taken out of
// the sum again.
//
// RAGGED = false: the row length is a multiple of the vector size and both tensors
// begin on a 16-byte boundary, so every vector is aligned.
// RAGGED = true: any row length, tensors at any address.  Row r begins at byte r*n,
// wherever that falls; vectors are read and written where they lie.  The byte slots of
// the row's last vector beyond its n-th element are overwritten with padding after the
// load (the load itself reads the first bytes of the next row there; only the vector that
// would reach past the end of the whole tensor is read byte by byte), and only the
// existing elements of that vector are stored.  Which vector is the last one, and how
// many of its elements exist, is the same for every row.
// ---------------------------------------------------------------------------
template <int G, int V, int R, int WPB, int MODE, bool RAGGED>
__global__ __launch_bounds__(64 * WPB) void hccs_rows_kernel(const int8_t *__restrict__ logits,
                                                             uint8_t *__restrict__ out, int Lq, int n,
                                                             uint32_t last_slab, BlockPlace place, HeadTable table)
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
    const int nvec = RAGGED ? (n + kVecBytes - 1) / kVecBytes : n / kVecBytes;
    const RowTail<DW> tail(n, nvec);

    const size_t slab = (size_t)slab_no * (size_t)Lq;
    const int wave_row0 = ((int)tile * WPB + wave) * kRowsPerWave;
    if (wave_row0 >= Lq) return;   // whole wave past the slab
    const int row0 = wave_row0 + grp;
    // The last vector of a row is read whole, i.e. kVecBytes - tail_elems bytes into the rows that
    // follow.  A row with fewer bytes than that between its end and the end of the tensor reads
    // its last vector byte by byte instead: the tensor's last row, or its last few rows when
    // rows are shorter than a vector.  `near_end` (block-uniform) says whether this slab can
    // hold such a row at all.
    const int over_read = kVecBytes - tail.tail_elems;
    const uint64_t rows_behind_slab = (uint64_t)(last_slab - slab_no) * (uint64_t)Lq;
    const bool near_end = RAGGED && over_read > 0 && rows_behind_slab * (uint64_t)n < (uint64_t)over_read;

    uint32_t d[R][V][DW];
    uint32_t row_off[R];   // element offset of each batch's row from that of the wave's first row
#pragma unroll
    for (int j = 0; j < R; ++j) row_off[j] = (uint32_t)(j * kRowsPerBatch) * (uint32_t)n;
    const size_t first_elem = (slab + row0) * (size_t)n + (size_t)sub * kVecBytes;   // the lane's first vector
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const int row = row0 + j * kRowsPerBatch;
        const int8_t *src = logits + first_elem + row_off[j] - sub * kVecBytes;
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const int vi = v * G + sub;
            if (row < Lq && vi < nvec) {
                if (RAGGED && near_end && vi == tail.last_vec &&
                    (rows_behind_slab + (uint64_t)(Lq - 1 - row)) * (uint64_t)n < (uint64_t)over_read)
                    load_vector_bytes<DW>(src + vi * kVecBytes, tail.tail_elems, d[j][v]);
                else
                    load_vector<DW, RAGGED>(src + vi * kVecBytes, d[j][v]);
                if (RAGGED && vi == tail.last_vec) tail.pad(d[j][v]);
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
        uint8_t *dst = out + (first_elem + row_off[j] - sub * kVecBytes) * kOutBytes;
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const int vi = v * G + sub;
            const u32x4 o = ro.vector(d[j][v]);
            if (row < Lq && vi < nvec) {
                if (RAGGED && vi == tail.last_vec && tail.tail_elems < kVecBytes)
                    store_vector_head(dst + vi * 16, o, tail.tail_elems * kOutBytes);
                else
                    store_vector<RAGGED>(dst + vi * 16, o);
            }
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
// One block of WAVES waves per row, for rows of more than 4096 bytes (256 vectors): thread t holds vectors
// t, t + 64*WAVES, ...; the maximum and the sum cross waves through LDS.
// Same arithmetic, the same padding rule and the same RAGGED forms as the kernel above.
// ---------------------------------------------------------------------------
template <int V, int WAVES, int MODE, bool RAGGED>
__global__ __launch_bounds__(64 * WAVES) void hccs_row_block_kernel(const int8_t *__restrict__ logits,
                                                             uint8_t *__restrict__ out, int Lq, int n,
                                                             uint32_t last_slab, BlockPlace place, HeadTable table)
{
    constexpr int kOutBytes = (MODE & 1) ? 2 : 1;
    constexpr int DW = 4 / kOutBytes;
    constexpr int kVecBytes = DW * 4;
    constexpr int kThreads = 64 * WAVES;
    constexpr int kPaddedLen = kThreads * V * kVecBytes;
    __shared__ int red[2][WAVES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t tile, head, slab_no;   // one block per row: the tile is the row inside the slab
    place.locate(tile, head, slab_no);
    const int4 hp = table.e[head];
    const int B = hp.x, S = hp.y, D = hp.z;
    const int nvec = RAGGED ? (n + kVecBytes - 1) / kVecBytes : n / kVecBytes;
    const RowTail<DW> tail(n, nvec);
    const size_t row = (size_t)slab_no * (size_t)Lq + tile;
    const int8_t *src = logits + row * (size_t)n;
    uint8_t *dst = out + row * (size_t)n * kOutBytes;
    const bool last_row = RAGGED && slab_no == last_slab && (int)tile == Lq - 1 && tail.tail_elems < kVecBytes;

    uint32_t d[V][DW];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int vi = v * kThreads + tid;
        if (vi < nvec) {
            if (RAGGED && last_row && vi == tail.last_vec)
                load_vector_bytes<DW>(src + vi * kVecBytes, tail.tail_elems, d[v]);
            else
                load_vector<DW, RAGGED>(src + vi * kVecBytes, d[v]);
            if (RAGGED && vi == tail.last_vec) tail.pad(d[v]);
        } else {
#pragma unroll
            for (int c = 0; c < DW; ++c) d[v][c] = kPadWord;
        }
    }
    int m = group_max<64>(lane_max(d));
    if (lane == 0) red[0][wave] = m;
    __syncthreads();
    m = red[0][0];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) m = max(m, red[0][w]);
    const uint32_t mu = (uint32_t)(m + 128);

    int t = group_sum<64>(lane_distances(d, m, D));
    if (lane == 0) red[1][wave] = t;
    __syncthreads();
    t = red[1][0];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) t += red[1][w];
    const int sum_clamped = clamped_sum(t, kPaddedLen, n, mu, D);
    const uint32_t Z = (uint32_t)(n * B - S * sum_clamped);
    const RowOutput<MODE> ro(Z, B, S, D);
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int vi = v * kThreads + tid;
        const u32x4 o = ro.vector(d[v]);
        if (vi < nvec) {
            if (RAGGED && vi == tail.last_vec && tail.tail_elems < kVecBytes)
                store_vector_head(dst + vi * 16, o, tail.tail_elems * kOutBytes);
            else
                store_vector<RAGGED>(dst + vi * 16, o);
        }
    }
}

// min(max(x, 0), 16) (one v_med3_i32)
__device__ __forceinline__ int clamp_bytes(int x) { return min(max(x, 0), 16); }

// Byte masks of a 16-byte vector, as four dwords: entry k of the first half has ones in bytes k..15
// (k = 0..15), entry k of the second half in bytes 0..k-1 (k = 0..16).
struct ByteMasks {
    uint32_t w[33][4];
};
constexpr ByteMasks make_byte_masks()
{
    ByteMasks t{};
    for (int k = 0; k <= 16; ++k)
        for (int c = 0; c < 4; ++c) {
            const int left = k - 4 * c;
            const uint32_t below = left >= 4 ? 0xffffffffu : (left <= 0 ? 0u : ((1u << (8 * left)) - 1u));
            if (k < 16) t.w[k][c] = ~below;
            t.w[16 + k][c] = below;
        }
    return t;
}
__device__ const ByteMasks kByteMasks = make_byte_masks();

// ---------------------------------------------------------------------------
// Rows of any length through LDS (8-bit outputs; both tensors begin on a 16-byte boundary;
// 16 < n <= 16*G*V - 15; Lq >= 64/G).
//
// The tensor is contiguous even where its rows are not vector-aligned, and 16 consecutive rows
// are a whole number of vectors whatever n is.  A block takes WPB*64/G rows, a multiple of 16:
// its byte range begins on a vector boundary and, except at the tensor's end, ends on one, and it
// goes into LDS as whole aligned vectors: every global access of the block is one contiguous run
// of full vectors.  That frees the lane layout from the memory access pattern: G lanes hold V
// vectors of a row each, so the per-row work (reductions, reciprocal, constants) is spread over
// 16*V elements per lane, not 16, while no global access gets narrower for it.
// LDS serves a 16-byte access that is not 16-byte aligned one lane per cycle (64 cycles per wave
// instruction against 6 for reads and 14 for writes when aligned, measured), so the lanes do not
// read their rows where they begin: a lane takes the aligned vectors of the block's range that its
// row touches, and replaces the bytes of the first and the last of them that belong to the
// neighbouring rows with padding (byte masks from a small table in LDS).  A vector that two
// rows share is thus read by a lane of each.  On the way back the lane with a row's last vector
// writes it first, whole; after a barrier the lane with the next row's first vector reads it back,
// puts its own bytes in and writes it again, and all other vectors are written; after another
// barrier the block stores its range as whole aligned vectors.  Only the block that holds the
// tensor's last rows may end inside a vector: it reads and writes that vector's bytes one by one.
// In-place use is safe: a block reads and writes the bytes of its own rows only.
// Rows are numbered through the whole tensor, so the rows of a block may belong to two heads, those of
// a wave too (never three: Lq >= 64/G): a lane picks its row's constants from the two candidates of
// its wave.
// ---------------------------------------------------------------------------
template <int G, int V, int WPB, int MODE>
__global__ __launch_bounds__(64 * WPB) void hccs_rows_staged_kernel(const int8_t *__restrict__ logits,
                                                                    uint8_t *__restrict__ out, uint32_t total_rows,
                                                                    int n, FastDiv by_Lq, FastDiv by_H, HeadTable table)
{
    static_assert((MODE & 1) == 0, "8-bit outputs: input and output ranges coincide");
    constexpr int kRowsPerWave = 64 / G, kRowsPerBlock = WPB * kRowsPerWave;
    static_assert(kRowsPerBlock % 16 == 0, "a block's first row begins on a vector boundary");
    constexpr int kSlots = G * V * 16;   // byte slots of a row's lanes; n + 15 <= kSlots
    constexpr int kThreads = 64 * WPB;
    static_assert(kThreads >= 33, "one thread per mask table entry");
    constexpr int kStageVectors = kRowsPerBlock * G * V;   // V per thread; the block's rows are fewer
    __shared__ u32x4 stage_in[kStageVectors + G * V];     // lanes past their row's end read (and mask) what follows
    __shared__ u32x4 stage_out[kStageVectors];
    __shared__ u32x4 keep[33];   // [k]: ones in bytes k..15 (k = 0..15); [16 + k]: ones in bytes 0..k-1 (k = 0..16)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int sub = lane % G, grp = lane / G;
    // Workgroups go to the 8 dies round-robin.  Neighbouring blocks share the 128-byte lines their
    // ranges meet in, so of every 64 consecutive blocks each die takes 8 neighbours, which lets its L2 put such a
    // line together; the blocks behind the last full 64 keep their numbers.
    const uint32_t in_full_groups = gridDim.x & ~63u;
    const uint32_t block_no = blockIdx.x < in_full_groups
                                  ? (blockIdx.x & ~63u) + (blockIdx.x & 7u) * 8u + ((blockIdx.x >> 3) & 7u)
                                  : blockIdx.x;
    const uint32_t block_row0 = block_no * (uint32_t)kRowsPerBlock;
    const int rows_here = (int)min((uint32_t)kRowsPerBlock, total_rows - block_row0);
    const size_t start = (size_t)block_row0 * (size_t)n;   // first byte of the block's rows, a multiple of 16
    const int span = rows_here * n;                         // bytes of the block's rows
    const int whole = span >> 4, rest = span & 15;          // whole vectors, bytes of the tensor's last, partial vector
    const int8_t *src = logits + start;
    uint8_t *dst = out + start;

    // ---- the block's vectors -> LDS; the byte masks
    {
        u32x4 w[V];
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const int c = i * kThreads + tid;
            if (c < whole) w[i] = load_stream(src + c * 16);
        }
        if (tid < 33) keep[tid] = *(const u32x4 *)kByteMasks.w[tid];
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const int c = i * kThreads + tid;
            if (c < whole) stage_in[c] = w[i];
        }
        if (rest != 0 && tid == 0) {   // the tensor ends inside this vector: its bytes one by one
            uint32_t t[4];
            load_vector_bytes<4>(src + whole * 16, rest, t);
            stage_in[whole] = (u32x4){t[0], t[1], t[2], t[3]};
        }
    }
    __syncthreads();

    // ---- the head of the lane's row
    const uint32_t wave_row0 = block_row0 + (uint32_t)(wave * kRowsPerWave);
    const uint32_t slab0 = by_Lq.quotient(wave_row0);
    const uint32_t head0 = slab0 - by_H.quotient(slab0) * by_H.divisor;
    const uint32_t head1 = head0 + 1 == by_H.divisor ? 0u : head0 + 1;
    const int change = (int)((slab0 + 1) * by_Lq.divisor - wave_row0);   // the wave's first row (counted from its own first) of the next head
    const int4 hp0 = table.e[head0], hp1 = table.e[head1];

    // ---- the lane's vectors of its row: vector first + v*G + sub of the block's range; the bytes of other
    // rows in it, and all of it if the row ends before it, become padding
    const int row_in_block = wave * kRowsPerWave + grp;
    const bool row_exists = row_in_block < rows_here;
    const int row_begin = (int)__umul24((uint32_t)row_in_block, (uint32_t)n), row_last = row_begin + n - 1;   // bytes of the block's range
    const int first = row_begin >> 4, last = row_last >> 4;
    const u32x4 from = keep[sub == 0 ? (row_begin & 15) : 0];
    const int row_end = row_exists ? row_last + 1 : 0;
    uint32_t d[V][4];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int c = first + v * G + sub;
        const int bytes = clamp_bytes(row_end - 16 * c);   // of the row in this vector, counted from the vector's first byte
        u32x4 mine = keep[16 + bytes];
        if (v == 0) mine &= from;
        const u32x4 t = stage_in[c];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            d[v][e] = (t[e] & mine[e]) | (kPadWord & ~mine[e]);
            asm("" : "+v"(d[v][e]));   // one value: the compiler would otherwise derive a second masked form for the distances
        }
    }

    u32x4 o[V];
    auto outputs = [&](int B, int S, int D) {
        const int m = group_max<G>(lane_max(d));
        const int t = group_sum<G>(lane_distances(d, m, D));
        const RowOutput<MODE> ro((uint32_t)(n * B - S * clamped_sum(t, kSlots, n, (uint32_t)(m + 128), D)), B, S, D);
#pragma unroll
        for (int v = 0; v < V; ++v) o[v] = ro.vector(d[v]);
    };
    // Most waves lie inside one head: its constants then stay scalar (and what is computed from them alone, too).
    if (change >= kRowsPerWave) {
        outputs(hp0.x, hp0.y, hp0.z);
    } else {
        const bool next_head = grp >= change;
        outputs(next_head ? hp1.x : hp0.x, next_head ? hp1.y : hp0.y, next_head ? hp1.z : hp0.z);
    }

    // ---- results -> LDS: each row's last vector first, whole
#pragma unroll
    for (int v = 0; v < V; ++v)
        if (row_exists && first + v * G + sub == last) stage_out[last] = o[v];
    __syncthreads();
    // then the others; a first vector that begins with the previous row's last bytes keeps those
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int c = first + v * G + sub;
        if (row_exists && c < last) {
            u32x4 r = o[v];
            if (v == 0 && sub == 0 && (row_begin & 15) != 0) {
                const u32x4 theirs = stage_out[c];
                r = (r & from) | (theirs & ~from);
            }
            stage_out[c] = r;
        }
    }
    __syncthreads();

    // ---- LDS -> the block's vectors
#pragma unroll
    for (int i = 0; i < V; ++i) {
        const int c = i * kThreads + tid;
        if (c < whole) store_stream(dst + c * 16, stage_out[c]);
    }
    if (tid < rest) __builtin_nontemporal_store(((const uint8_t *)stage_out)[whole * 16 + tid], dst + whole * 16 + tid);
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

// One vector per thread, blocks of one wave: the fastest of the forms measured for a plain copy (1 GiB each way:
// 0.84 of 8 TB/s against 0.76-0.78 with four vectors per thread in blocks of four waves; 32 MiB each way: 0.71 against 0.68).
__global__ __launch_bounds__(64) void copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int64_t count)
{
    const int64_t i = (int64_t)blockIdx.x * 64 + threadIdx.x;
    if (i < count) store_stream(dst + i, load_stream(src + i));
}

// ---------------------------------------------------------------------------
// host side: choose the lane-group shape for a row length
// ---------------------------------------------------------------------------
template <int G, int V, int R, int WPB, int MODE, bool RAGGED>
static hipError_t launch_rows(const int8_t *x, uint8_t *p, int64_t Bt, int H, int Lq, int n, const HeadTable &tab,
                              hipStream_t st)
{
    constexpr int kRowsPerBlock = WPB * R * (64 / G);
    dim3 grid;
    // neighbouring blocks on one die when they meet inside 128-byte lines, for rows of more than 2048 bytes (shorter
    // rows lose with it: 2000 bytes 180 against 174 us, 1040 bytes 104 against 102)
    const BlockPlace place = place_blocks((Lq + kRowsPerBlock - 1) / kRowsPerBlock, H, Bt, grid,
                                          G == 64 && V == 4 && (kRowsPerBlock * n) % 128 != 0);
    // Rows of 2049..4096 bytes, a wave each with four vectors per lane in flight: with all eight blocks a compute
    // unit can hold, 128 KiB per unit are under way and memory serves them more slowly than 64 KiB (a plain copy shows
    // the same: 0.76 of peak with 128 KiB per unit in flight, 0.79-0.82 with 32-64 KiB).  32 KiB of untouched LDS per block leave
    // four blocks per unit: [4,16,4096,4096] 333 against 343 us, [4,16,1024,4096] 82.1 against 83.7 us; no gain at the
    // other row lengths (2048: 173 against 167 us with four blocks; 8192, 16384: equal).
    constexpr size_t kHeldBack = (G == 64 && V == 4 && (MODE & 1) == 0 && !RAGGED) ? (32u << 10) : 0;
    return launch_fewer(hccs_rows_kernel<G, V, R, WPB, MODE, RAGGED>, grid, dim3(64 * WPB), kHeldBack, st, x, p, Lq, n,
                        (uint32_t)(Bt * H - 1), place, tab);
}

template <int MODE, bool RAGGED>
static hipError_t launch_shape(const int8_t *x, uint8_t *p, int64_t Bt, int H, int Lq, int Lk, const HeadTable &tab,
                               hipStream_t st)
{
    constexpr int VB = (MODE & 1) ? 8 : 16;   // input bytes per vector
    const int nvec = (Lk + VB - 1) / VB;
    // Whole aligned rows of 3968..4096 bytes run 2-3 % faster as blocks of two waves than as a wave each
    // ([4,16,4096,4096] 328 against 334 us, 3968 bytes 320 against 329; 3840 bytes 321 against 318: the wave form).
    const bool two_waves = !RAGGED && (MODE & 1) == 0 && nvec >= 248;
    if (nvec <= 256 && !two_waves) {          // a wave holds the row
        // Lane-group width G: a power of two that covers the row with one or two vectors
        // per lane, so that each load/store instruction touches G contiguous vectors of a
        // row; beyond 128 vectors the row takes four vectors per lane of a whole wave.  Few rows
        // in flight per wave (R) and many waves measured faster than the reverse; with vectors
        // at any address one row batch per wave measured best ([64,12,197,197]: 15.3 against
        // 16.0 us, [256,8,128,250]: 26.2 against 29.4 us).
        // Whole rows of exactly 4 or 8 vectors fill their lane group with one vector per lane; blocks of one wave
        // with one row batch then run 2 % faster than the forms below in the 8-bit modes (the same in a plain copy: one
        // vector per thread in blocks of one wave is its fastest form): [256,8,128,128] 12.4 against 12.7 us,
        // [512,8,128,64] 12.4 against 12.7.  Not so the 16-bit modes ([256,8,128,128]: 19.0 against 17.9 us), rows that
        // leave lanes of the group empty (96 bytes 11.1 against 10.8 us), or rows of 16, 32 and 64 vectors: back to back
        // they gain 2-3 % too ([64,12,512,512] 60.6 against 62.5 us), but a launch on its own, as a profiler times it,
        // loses as much to its hundreds of thousands of one-wave blocks (64.7 against 62.7 us).
        if constexpr (!RAGGED && (MODE & 1) == 0) {
            if (nvec == 4) return launch_rows<4, 1, 1, 1, MODE, RAGGED>(x, p, Bt, H, Lq, Lk, tab, st);
            if (nvec == 8) return launch_rows<8, 1, 1, 1, MODE, RAGGED>(x, p, Bt, H, Lq, Lk, tab, st);
        }
        constexpr int R = RAGGED ? 1 : 2;
        if (nvec <= 4) return launch_rows<4, 1, R, 4, MODE, RAGGED>(x, p, Bt, H, Lq, Lk, tab, st);
        if (nvec <= 8) return launch_rows<8, 1, R, 4, MODE, RAGGED>(x, p, Bt, H, Lq, Lk, tab, st);
        if (nvec <= 16) return launch_rows<16, 1, R, 4, MODE, RAGGED>(x, p, Bt, H, Lq, Lk, tab, st);
        if (nvec <= 32) return launch_rows<16, 2, 1, 4, MODE, RAGGED>(x, p, Bt, H, Lq, Lk, tab, st);
        if (nvec <= 64) return launch_rows<32, 2, 1, 4, MODE, RAGGED>(x, p, Bt, H, Lq, Lk, tab, st);   // measured against <64,1,2>: up to 20 % faster below 48 vectors, equal at 64
        if (nvec <= 128) return launch_rows<64, 2, 1, 4, MODE, RAGGED>(x, p, Bt, H, Lq, Lk, tab, st);
        return launch_rows<64, 4, 1, 4, MODE, RAGGED>(x, p, Bt, H, Lq, Lk, tab, st);
    }
    // Longer rows: one block per row, two vectors per thread (four beyond 2048 vectors) and as many waves as
    // that takes.  Measured against a wave per row with 8, 16 or 32 vectors per lane, and, beyond 16 KiB, against
    // four waves with 8 or 16 vectors per thread (fraction of 8 TB/s, that form / this one): 4112 bytes 0.66 / 0.73,
    // 6000 0.70 / 0.74, 8192 0.77 / 0.80, 10240 0.77 / 0.79, 12000 0.72 / 0.73, 16384 0.74 / 0.80, 20000 0.70 / 0.76,
    // 32768 0.78 / 0.78, 50000 0.70 / 0.75, 65536 0.70 / 0.72: about 64 KiB per compute unit are in flight at full occupancy.
    dim3 grid;
    const BlockPlace place = place_blocks(Lq, H, Bt, grid, Lk % 128 != 0);
    const uint32_t last_slab = (uint32_t)(Bt * H - 1);
    if (nvec <= 256)
        return launch(hccs_row_block_kernel<2, 2, MODE, RAGGED>, grid, dim3(128), st, x, p, Lq, Lk, last_slab, place, tab);
    if (nvec <= 512)
        return launch(hccs_row_block_kernel<2, 4, MODE, RAGGED>, grid, dim3(256), st, x, p, Lq, Lk, last_slab, place, tab);
    if (nvec <= 1024)
        return launch(hccs_row_block_kernel<2, 8, MODE, RAGGED>, grid, dim3(512), st, x, p, Lq, Lk, last_slab, place, tab);
    if (nvec <= 2048)
        return launch(hccs_row_block_kernel<2, 16, MODE, RAGGED>, grid, dim3(1024), st, x, p, Lq, Lk, last_slab, place, tab);
    // at most 4096 vectors: Lk <= 65536 in the 8-bit modes, and the 16-bit modes need Lk*B <= 32767
    return launch(hccs_row_block_kernel<4, 16, MODE, RAGGED>, grid, dim3(1024), st, x, p, Lq, Lk, last_slab, place, tab);
}

// Rows through LDS: G lanes x V vectors per row, blocks of WPB waves.  The caller keeps n + 15 within 16*G*V
// and Lq at 64/G or more.  Measured on [64,12,197,197]: 8 lanes x 2 vectors per row in blocks of 2 waves 13.3 us;
// blocks of 1, 4, 8 waves 13.6, 13.7, 15.4; 16 lanes x 1 vector 15.6; 4 lanes x 4 vectors 18.9; 8 x 3 19.3.
template <int G, int V, int WPB, int MODE>
static hipError_t launch_staged(const int8_t *x, uint8_t *p, int64_t Bt, int H, int Lq, int Lk, const HeadTable &tab,
                                hipStream_t st)
{
    constexpr int kRowsPerBlock = WPB * (64 / G);
    const int64_t rows = Bt * H * Lq;
    return launch(hccs_rows_staged_kernel<G, V, WPB, MODE>, dim3((uint32_t)((rows + kRowsPerBlock - 1) / kRowsPerBlock)),
                  dim3(64 * WPB), st, x, p, (uint32_t)rows, Lk, make_fast_div((uint32_t)Lq), make_fast_div((uint32_t)H), tab);
}

template <int MODE>
static hipError_t launch_mode(const int8_t *x, uint8_t *p, int64_t Bt, int H, int Lq, int Lk, const HeadTable &tab,
                              bool aligned, hipStream_t st)
{
    // aligned vectors when both tensors begin on a 16-byte boundary and rows are whole vectors
    if (aligned && Lk % ((MODE & 1) ? 8 : 16) == 0) return launch_shape<MODE, false>(x, p, Bt, H, Lq, Lk, tab, st);
    if constexpr ((MODE & 1) == 0) {
        // Rows of other lengths in tensors that begin on a 16-byte boundary go through LDS where that measured
        // faster than vectors at any address ([64,12,197,n] in us, through LDS / at any address: n = 70 7.9 / 8.8,
        // 100 8.1 / 9.1, 113 8.6 / 9.5, 150 12.2 / 14.4, 197 13.3 / 15.1, 241 14.8 / 15.6, 270 20.1 / 20.5,
        // 300 20.5 / 22.2, 380 21.9 / 28.5, 450 24.5 / 30.8, 497 27.2 / 33.6, 785 42.2 / 43.2, 900 45.7 / 48.5,
        // 1000 49.0 / 53.8; slower or equal in the gaps: 120 11.6 / 9.6, 250 19.9 / 16.4, 520 37.7 / 33.4,
        // 700 39.9 / 38.9).  The time of a lane layout hardly depends on n, so each serves the lengths that fill it.
        // (row numbers of the last block's empty waves stay below 2^31: the divisions by Lq and H hold up to there)
        if (aligned && Lq >= 16 && Bt * H * Lq < 0x7fffff00ll) {
            if (Lk > 64 && Lk <= 113) return launch_staged<4, 2, 2, MODE>(x, p, Bt, H, Lq, Lk, tab, st);
            if (Lk > 128 && Lk <= 241) return launch_staged<8, 2, 2, MODE>(x, p, Bt, H, Lq, Lk, tab, st);
            if (Lk > 256 && Lk <= 497) return launch_staged<16, 2, 4, MODE>(x, p, Bt, H, Lq, Lk, tab, st);
            if (Lk > 768 && Lk <= 1009) return launch_staged<32, 2, 8, MODE>(x, p, Bt, H, Lq, Lk, tab, st);
        }
    }
    return launch_shape<MODE, true>(x, p, Bt, H, Lq, Lk, tab, st);
}

hipError_t launch_softmax(const int8_t *x, void *out, int64_t Bt, int H, int Lq, int Lk, const HeadTable &tab,
                          int mode, bool aligned, hipStream_t st)
{
    if (Bt == 0 || Lq == 0) return hipSuccess;
    uint8_t *p = (uint8_t *)out;
    switch (mode) {
        case kModeU8: return launch_mode<kModeU8>(x, p, Bt, H, Lq, Lk, tab, aligned, st);
        case kModeI16: return launch_mode<kModeI16>(x, p, Bt, H, Lq, Lk, tab, aligned, st);
        case kModeClbU8: return launch_mode<kModeClbU8>(x, p, Bt, H, Lq, Lk, tab, aligned, st);
        case kModeClbI16: return launch_mode<kModeClbI16>(x, p, Bt, H, Lq, Lk, tab, aligned, st);
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
    if ((count + 63) / 64 > 0x7fffffff) return hipErrorInvalidValue;
    return launch(copy_kernel, dim3((unsigned)((count + 63) / 64)), dim3(64), st, (const u32x4 *)src, (u32x4 *)dst, count);
}

}  // namespace hccs
