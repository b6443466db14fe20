// Offline calibration by grid search (Sec. III-C, Eq. (10)): for every head and every
// candidate (B, S, Dmax), the mean over the head's rows of KL(softmax(alpha*x) || q), q the
// normalised 16-bit HCCS output, and the arg-min per head.
//
// The divergence of a row depends on its logits only through the histogram c[delta] of
// distances to the row maximum (delta = 0..255), because both distributions are functions of
// delta alone: softmax weight E[delta] = exp(-alpha*delta), score s(delta) = B - S*min(delta, D),
// and the 16-bit output normalises to s/Z exactly (the reciprocal cancels).  With
// w[delta] = c[delta]*E[delta]/sum(c*E) the row's divergence is
//     KL = (-alpha*sum(delta*w) - log sum(c*E))  -  sum_delta w[delta]*log s(delta)  +  log Z,
//     Z  = n*B - S*C(D),   C(D) = sum_delta c[delta]*min(delta, D).
// So one pass over the logits leaves, per row, a constant and the integer table C(0..127), and
// per head the summed weights W[delta]; a candidate then costs 256 logarithms plus one per row.
// All sums are taken in a fixed order (no floating-point atomics): results are reproducible.
#include "hccs_device.h"

#include <mutex>

namespace hccs {

// Work memory of hccs_calibrate_grid_static: the same layout launch_calibrate gives a caller's
// workspace, but owned by the library so that the call allocates nothing.  Each device holds its
// own copy of the array at its own address; `scratch` itself is only a host-side stand-in for it.
static __device__ __align__(256) unsigned char scratch[HCCS_STATIC_SCRATCH_BYTES];

struct AlphaTable {
    double e[HCCS_MAX_HEADS];
};

__device__ __forceinline__ double shfl_xor_f64(double v, int mask)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __shfl_xor(lo, mask);
    hi = __shfl_xor(hi, mask);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) v += shfl_xor_f64(v, m);
    return v;
}
__device__ __forceinline__ int wave_inclusive_scan(int v, int lane)
{
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int t = __shfl_up(v, d);
        if (lane >= d) v += t;
    }
    return v;
}
// block-wide sum of one double per thread (256 threads), fixed tree; result valid in thread 0
__device__ __forceinline__ double block_sum_f64(double v, double *scratch4)
{
    v = wave_sum_f64(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch4[threadIdx.x >> 6] = v;
    __syncthreads();
    return (scratch4[0] + scratch4[1]) + (scratch4[2] + scratch4[3]);
}

// Pass 1: one block per (batch, head) slab, a wave per row.  Writes the row constants, the
// D-major table ctab[D][row] and the slab's summed weights wpart[slab][delta].
__global__ __launch_bounds__(256) void calib_stats_kernel(const int8_t *__restrict__ logits, int H, int Lq, int n,
                                                          AlphaTable alpha, int64_t rows_total,
                                                          int32_t *__restrict__ ctab, double *__restrict__ rowconst,
                                                          double *__restrict__ wpart)
{
    __shared__ int hist[4][256];
    __shared__ double wsum[4][256];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t slab = blockIdx.x;
    const int head = (int)(blockIdx.x % (uint32_t)H);
    const double a = alpha.e[head];
    double wacc[4] = {0.0, 0.0, 0.0, 0.0};   // weights of delta = lane + 64*k, summed over this wave's rows
    double e[4];                             // exp(-alpha*delta) of the lane's four distances: the same for every row
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) e[kk] = exp(-a * (double)(lane + 64 * kk));

    for (int q0 = 0; q0 < Lq; q0 += 4) {     // same trip count in every wave
        const int q = q0 + wave;
        const bool live = q < Lq;
        const int64_t row = slab * Lq + q;
        const int8_t *x = logits + row * (int64_t)n;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) hist[wave][lane + 64 * kk] = 0;
        int m = -128;
        if (live)
            for (int i = lane; i < n; i += 64) m = max(m, (int)x[i]);
        m = group_max<64>(m);
        __syncthreads();
        if (live)
            for (int i = lane; i < n; i += 64) atomicAdd(&hist[wave][m - (int)x[i]], 1);
        __syncthreads();
        if (live) {
            int c[4];
            double ce[4], den = 0.0, t1 = 0.0;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                c[kk] = hist[wave][lane + 64 * kk];
                ce[kk] = (double)c[kk] * e[kk];
                den += ce[kk];
            }
            den = wave_sum_f64(den);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const double w = ce[kk] / den;
                wacc[kk] += w;
                t1 += (double)(lane + 64 * kk) * w;
            }
            t1 = wave_sum_f64(t1);
            if (lane == 0) rowconst[row] = -a * t1 - log(den);

            // C(D) = C(D-1) + #{delta >= D}: two prefix scans over the lanes
            const int cum0 = wave_inclusive_scan(c[0], lane);            // #{delta <= lane}
            const int tot0 = __shfl(cum0, 63);
            const int cum1 = tot0 + wave_inclusive_scan(c[1], lane);     // #{delta <= 64 + lane}
            const int a0 = lane == 0 ? 0 : n - (cum0 - c[0]);            // #{delta >= lane}
            const int a1 = n - (cum1 - c[1]);                            // #{delta >= 64 + lane}
            const int C0 = wave_inclusive_scan(a0, lane);
            const int C1 = __shfl(C0, 63) + wave_inclusive_scan(a1, lane);
            ctab[(int64_t)lane * rows_total + row] = C0;
            ctab[(int64_t)(64 + lane) * rows_total + row] = C1;
        }
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) wsum[wave][lane + 64 * kk] = wacc[kk];
    __syncthreads();
    const int t = threadIdx.x;
    wpart[slab * 256 + t] = (wsum[0][t] + wsum[1][t]) + (wsum[2][t] + wsum[3][t]);
}

// Pass 2: per head, W[delta] = sum over batches of the slab weights; K = sum of the row constants.
__global__ __launch_bounds__(256) void calib_reduce_kernel(const double *__restrict__ wpart,
                                                           const double *__restrict__ rowconst, int Bt, int H,
                                                           int Lq, double *__restrict__ W, double *__restrict__ K)
{
    __shared__ double scratch[4];
    const int head = blockIdx.x, t = threadIdx.x;
    double w = 0.0;
    for (int b = 0; b < Bt; ++b) w += wpart[((int64_t)b * H + head) * 256 + t];
    W[head * 256 + t] = w;
    // rows of the head: (batch b, query q) for i = b*Lq + q = t, t + 256, ...; no division per row
    double k = 0.0;
    const int64_t R = (int64_t)Bt * Lq;
    const int step_b = 256 / Lq, step_q = 256 % Lq;
    int b = t / Lq, q = t % Lq;
    for (int64_t i = t; i < R; i += 256) {
        k += rowconst[((int64_t)b * H + head) * Lq + q];
        b += step_b, q += step_q;
        if (q >= Lq) q -= Lq, ++b;
    }
    k = block_sum_f64(k, scratch);
    if (t == 0) K[head] = k;
}

// log(z) for z = 1 .. 32767 (entry 0 unused): every Z of an admissible candidate is an integer in
// [256, 32767] (strict band), so the per-row logarithm of pass 3 is a table lookup of the same
// double the logarithm routine returns.
__global__ __launch_bounds__(256) void calib_logtab_kernel(double *__restrict__ logtab)
{
    const int z = blockIdx.x * 256 + threadIdx.x;
    if (z < 32768) logtab[z] = z > 0 ? log((double)z) : 0.0;
}

// Pass 3: one block per (candidate, head).
__global__ __launch_bounds__(256) void calib_objective_kernel(const hccs_head_params *__restrict__ cand, int nc,
                                                              int Bt, int H, int Lq, int n, int64_t rows_total,
                                                              const int32_t *__restrict__ ctab,
                                                              const double *__restrict__ W,
                                                              const double *__restrict__ K,
                                                              const double *__restrict__ logtab,
                                                              double *__restrict__ objective)
{
    __shared__ double scratch[4];
    const int c = blockIdx.x, head = blockIdx.y, t = threadIdx.x;
    const int64_t B = cand[c].B, S = cand[c].S, D = cand[c].Dmax;
    // strict band of Sec. IV-C for rows of length n; anything else scores +infinity
    const bool ok = D >= 0 && D <= 127 && S >= 0 && S <= 127 && B >= 1 && B <= 32767 && B - S * D >= 0 &&
                    (int64_t)n * (B - S * D) >= 256 && (int64_t)n * B <= 32767;
    if (!ok) {
        if (t == 0) objective[(int64_t)head * nc + c] = __longlong_as_double(0x7ff0000000000000ll);
        return;
    }
    const double term2 = block_sum_f64(W[head * 256 + t] * logtab[B - S * min((int64_t)t, D)], scratch);
    // rows of the head: (batch b, query q) for i = b*Lq + q = t, t + 256, ...; b and q advance
    // without a division per row
    double z = 0.0;
    const int64_t R = (int64_t)Bt * Lq;
    const int32_t *col = ctab + D * rows_total;
    const int nB = n * (int)B, iS = (int)S;
    const int step_b = 256 / Lq, step_q = 256 % Lq;
    int b = t / Lq, q = t % Lq;
    for (int64_t i = t; i < R; i += 256) {
        const int64_t row = ((int64_t)b * H + head) * Lq + q;
        z += logtab[nB - iS * col[row]];
        b += step_b, q += step_q;
        if (q >= Lq) q -= Lq, ++b;
    }
    const double term3 = block_sum_f64(z, scratch);
    if (t == 0) objective[(int64_t)head * nc + c] = (K[head] - term2 + term3) / (double)R;
}

// Pass 4: first index of the minimum per head (-1 if every candidate is inadmissible).
__global__ __launch_bounds__(256) void calib_argmin_kernel(const double *__restrict__ objective, int nc,
                                                           int32_t *__restrict__ best)
{
    __shared__ double sv[256];
    __shared__ int si[256];
    const int head = blockIdx.x, t = threadIdx.x;
    const double inf = __longlong_as_double(0x7ff0000000000000ll);
    double bv = inf;
    int bi = -1;
    for (int c = t; c < nc; c += 256) {
        const double v = objective[(int64_t)head * nc + c];
        if (v < bv) bv = v, bi = c;
    }
    sv[t] = bv, si[t] = bi;
    __syncthreads();
    for (int step = 128; step > 0; step >>= 1) {
        if (t < step) {
            const double ov = sv[t + step];
            const int oi = si[t + step];
            if (oi >= 0 && (si[t] < 0 || ov < sv[t] || (ov == sv[t] && oi < si[t]))) sv[t] = ov, si[t] = oi;
        }
        __syncthreads();
    }
    if (t == 0) best[head] = si[0];
}

int64_t calibrate_workspace_bytes(int64_t Bt, int64_t H, int64_t Lq)
{
    const int64_t rows = Bt * H * Lq;
    return rows * 128 * 4 + rows * 8 + Bt * H * 256 * 8 + H * 256 * 8 + H * 8 + 32768 * 8;
}

hipError_t launch_calibrate(const int8_t *logits, int Bt, int H, int Lq, int Lk, const double *alpha,
                            const hccs_head_params *cand, int nc, double *objective, int32_t *best, void *workspace,
                            hipStream_t st)
{
    const int64_t rows = (int64_t)Bt * H * Lq;
    int32_t *ctab = (int32_t *)workspace;
    double *rowconst = (double *)(ctab + rows * 128);
    double *wpart = rowconst + rows;
    double *W = wpart + (int64_t)Bt * H * 256;
    double *K = W + (int64_t)H * 256;
    double *logtab = K + H;
    AlphaTable at;
    for (int h = 0; h < HCCS_MAX_HEADS; ++h) at.e[h] = h < H ? alpha[h] : 0.0;
    const dim3 block(256);
    hipError_t e = launch(calib_stats_kernel, dim3((uint32_t)(Bt * H)), block, st, logits, H, Lq, Lk, at, rows, ctab,
                          rowconst, wpart);
    if (e == hipSuccess) e = launch(calib_reduce_kernel, dim3(H), block, st, wpart, rowconst, Bt, H, Lq, W, K);
    if (e == hipSuccess) e = launch(calib_logtab_kernel, dim3(128), block, st, logtab);
    if (e == hipSuccess)
        e = launch(calib_objective_kernel, dim3(nc, H), block, st, cand, nc, Bt, H, Lq, Lk, rows, ctab, W, K, logtab,
                   objective);
    if (e == hipSuccess) e = launch(calib_argmin_kernel, dim3(H), block, st, objective, nc, best);
    return e;
}

// Device address of `scratch` on the current device, looked up once per device.
hipError_t static_scratch(void **ptr)
{
    constexpr int kMaxDevices = 64;
    static void *address[kMaxDevices] = {};
    static std::mutex guard;
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(guard);
    if (!address[device]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        address[device] = p;
    }
    *ptr = address[device];
    return hipSuccess;
}

}  // namespace hccs
