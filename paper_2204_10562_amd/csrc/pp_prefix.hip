// pp_prefix_costs: prefix sums of the per-layer times and the transfer-time tables.
//
// Stage compute time is a difference of prefix sums of p^f_l + p^b_l (Lemma 1, definition
// of C); transfer time over a link is size / bandwidth (Sec. III-B, c^f and c^b with one GPU
// per stage), rounded up to whole microseconds per direction.
//
// Both parts are bandwidth-trivial: 4L int64 in, 2(L+1) + 2 D^2 L int64 out.  The scan reads
// and writes consecutive int64 per consecutive lane and does its chunked work in LDS; the table
// part gives every thread one (link, boundary) entry, so a wave reads consecutive activation
// sizes and writes 64 consecutive int64 results (512-byte coalesced segments).
#include "pp_common.h"

#define SCAN_THREADS 256

// One workgroup scans both arrays.  The inputs are read lane-interleaved (consecutive lanes,
// consecutive int64: coalesced) into LDS, every thread then scans a contiguous chunk there,
// the chunk totals are scanned with wave shuffles and one exchange between the four waves,
// and the results leave LDS lane-interleaved again.  A value that reaches 2^62 (also by
// wrap-around: each addend is below 2^62, so a running sum cannot skip the interval
// [2^62, 2^64)) raises the overflow fault.
__device__ __forceinline__ void prefix_scan(
    int L, const long long *__restrict__ fwd, const long long *__restrict__ bwd,
    const long long *__restrict__ actf, const long long *__restrict__ actb,
    long long *__restrict__ PF, long long *__restrict__ PB, int32_t *status) {
    __shared__ unsigned long long sF[PP_MAX_LAYERS], sB[PP_MAX_LAYERS];
    __shared__ unsigned long long wF[SCAN_THREADS / 64], wB[SCAN_THREADS / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int fault = 0;
    for (int l = tid; l < L; l += SCAN_THREADS) {
        const long long f = fwd[l], b = bwd[l];
        if (f < 0 || b < 0) fault |= PP_FAULT_NEGATIVE;
        if (f >= PP_CAP62 || b >= PP_CAP62) fault |= PP_FAULT_OVERFLOW;
        if (l + 1 < L && (actf[l] < 0 || (actb && actb[l] < 0))) fault |= PP_FAULT_NEGATIVE;
        sF[l] = (unsigned long long)f;
        sB[l] = (unsigned long long)b;
    }
    __syncthreads();
    const int chunk = (L + SCAN_THREADS - 1) / SCAN_THREADS;
    const int lo = tid * chunk, hi = min(L, lo + chunk);
    unsigned long long tf = 0, tb = 0;
    for (int l = lo; l < hi; ++l) { tf += sF[l]; tb += sB[l]; }
    // inclusive scan of the chunk totals: within the wave, then across the four waves
    unsigned long long inf = tf, inb = tb;
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long of = __shfl_up(inf, d), ob = __shfl_up(inb, d);
        if (lane >= d) { inf += of; inb += ob; }
    }
    if (lane == 63) { wF[wave] = inf; wB[wave] = inb; }
    __syncthreads();
    unsigned long long rf = inf - tf, rb = inb - tb;  // exclusive: the sum before this chunk
    for (int v = 0; v < wave; ++v) { rf += wF[v]; rb += wB[v]; }
    // a partial total that wrapped shows up here or in some later chunk's running value
    if (rf + tf >= (unsigned long long)PP_CAP62 || rb + tb >= (unsigned long long)PP_CAP62)
        fault |= PP_FAULT_OVERFLOW;
    for (int l = lo; l < hi; ++l) {
        rf += sF[l];
        rb += sB[l];
        if (rf >= (unsigned long long)PP_CAP62 || rb >= (unsigned long long)PP_CAP62)
            fault |= PP_FAULT_OVERFLOW;
        sF[l] = rf;
        sB[l] = rb;
    }
    __syncthreads();
    if (tid == 0) { PF[0] = 0; PB[0] = 0; }
    for (int l = tid; l < L; l += SCAN_THREADS) {
        PF[l + 1] = (long long)sF[l];
        PB[l + 1] = (long long)sB[l];
    }
    if (fault) pp_raise(status, fault);
}

__device__ __forceinline__ long long ceil_div_u(long long a, long long b) {
    unsigned long long q = (unsigned long long)a / (unsigned long long)b;
    return (long long)(q + ((unsigned long long)a - q * (unsigned long long)b != 0));
}

// one thread per table entry i = link * L + k, link = u*D+v; `block` counts the table's blocks
__device__ __forceinline__ void transfer_tables(
    size_t block, int L, int D, const long long *__restrict__ actf, const long long *__restrict__ actb,
    const long long *__restrict__ bw, long long *__restrict__ XF, long long *__restrict__ XB,
    int32_t *status) {
    const size_t i = block * blockDim.x + threadIdx.x;
    if (i >= (size_t)D * D * L) return;
    const int link = (int)(i / (size_t)L);
    const int k = (int)(i - (size_t)link * L);
    const int u = link / D, v = link - u * D;
    long long xf = 0, xb = 0;
    int fault = 0;
    if (u != v) {
        const long long buv = bw[(size_t)u * D + v], bvu = bw[(size_t)v * D + u];
        if (buv <= 0 || bvu <= 0) {
            fault |= PP_FAULT_BANDWIDTH;
        } else if (k + 1 < L) {
            const long long af = actf[k], ab = actb ? actb[k] : af;
            if (af >= 0) xf = ceil_div_u(af, buv);
            if (ab >= 0) xb = ceil_div_u(ab, bvu);
            if (xf >= PP_CAP62 || xb >= PP_CAP62) fault |= PP_FAULT_OVERFLOW;
        }
    }
    XF[i] = xf;
    XB[i] = xb;
    if (fault) pp_raise(status, fault);
}

// Workgroup 0 scans; the others fill the tables, which do not depend on the scan: one launch.
__global__ __launch_bounds__(SCAN_THREADS) void k_prefix_costs(
    int L, int D, const long long *__restrict__ fwd, const long long *__restrict__ bwd,
    const long long *__restrict__ actf, const long long *__restrict__ actb,
    const long long *__restrict__ bw, long long *__restrict__ PF, long long *__restrict__ PB,
    long long *__restrict__ XF, long long *__restrict__ XB, int32_t *status) {
    if (blockIdx.x == 0) prefix_scan(L, fwd, bwd, actf, actb, PF, PB, status);
    else transfer_tables((size_t)blockIdx.x - 1, L, D, actf, actb, bw, XF, XB, status);
}

extern "C" int pp_prefix_costs(int L, int D, const int64_t *fwd_us, const int64_t *bwd_us,
                               const int64_t *act_fwd_bytes, const int64_t *act_bwd_bytes,
                               const int64_t *bw, int64_t *PF, int64_t *PB, int64_t *XF,
                               int64_t *XB, int32_t *status, void *stream) {
    if (L < 1 || L > PP_MAX_LAYERS || D < 1 || D > PP_MAX_DEVICES) return PP_ERR_INVALID_ARG;
    if (!fwd_us || !bwd_us || !act_fwd_bytes || !bw || !PF || !PB || !XF || !XB)
        return PP_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const size_t total = (size_t)D * D * L;
    hipLaunchKernelGGL(k_prefix_costs, dim3((unsigned)(1 + (total + SCAN_THREADS - 1) / SCAN_THREADS)),
                       dim3(SCAN_THREADS), 0, st, L, D, (const long long *)fwd_us,
                       (const long long *)bwd_us, (const long long *)act_fwd_bytes,
                       (const long long *)act_bwd_bytes, (const long long *)bw, (long long *)PF,
                       (long long *)PB, (long long *)XF, (long long *)XB, status);
    if (hipGetLastError() != hipSuccess) return PP_ERR_HIP;
    return PP_OK;
}
