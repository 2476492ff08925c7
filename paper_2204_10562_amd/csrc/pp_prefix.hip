// pp_prefix_costs: prefix sums of the per-layer times and the transfer-time tables.
//
// Stage compute time is a difference of prefix sums of p^f_l + p^b_l (Lemma 1, definition
// of C); transfer time over a link is size / bandwidth (Sec. III-B, c^f and c^b with one GPU
// per stage), rounded up to whole microseconds per direction.
//
// Both parts are bandwidth-trivial: 4L int64 in, 2(L+1) + 2 D^2 L int64 out.  The table
// part gives every thread one (link, boundary) entry, so a wave reads consecutive
// activation sizes and writes 64 consecutive int64 results (512-byte coalesced segments).
#include "pp_common.h"

#define SCAN_THREADS 256

// One workgroup scans both arrays.  Each thread owns a contiguous chunk; chunk totals are
// scanned through LDS; a value that reaches 2^62 (also by wrap-around: each addend is below
// 2^62, so a running sum cannot skip the interval [2^62, 2^64)) raises the overflow fault.
__device__ __forceinline__ void prefix_scan(
    int L, const long long *__restrict__ fwd, const long long *__restrict__ bwd,
    const long long *__restrict__ actf, const long long *__restrict__ actb,
    long long *__restrict__ PF, long long *__restrict__ PB, int32_t *status) {
    __shared__ unsigned long long totF[SCAN_THREADS], totB[SCAN_THREADS];
    const int tid = threadIdx.x;
    const int chunk = (L + SCAN_THREADS - 1) / SCAN_THREADS;
    const int lo = tid * chunk, hi = min(L, lo + chunk);
    int fault = 0;
    unsigned long long sf = 0, sb = 0;
    for (int l = lo; l < hi; ++l) {
        long long f = fwd[l], b = bwd[l];
        if (f < 0 || b < 0) fault |= PP_FAULT_NEGATIVE;
        if (f >= PP_CAP62 || b >= PP_CAP62) fault |= PP_FAULT_OVERFLOW;
        if (l + 1 < L && (actf[l] < 0 || (actb && actb[l] < 0))) fault |= PP_FAULT_NEGATIVE;
        sf += (unsigned long long)f;
        sb += (unsigned long long)b;
    }
    totF[tid] = sf;
    totB[tid] = sb;
    __syncthreads();
    // inclusive Hillis-Steele scan of the chunk totals
    for (int d = 1; d < SCAN_THREADS; d <<= 1) {
        unsigned long long af = 0, ab = 0;
        if (tid >= d) { af = totF[tid - d]; ab = totB[tid - d]; }
        __syncthreads();
        totF[tid] += af;
        totB[tid] += ab;
        __syncthreads();
    }
    unsigned long long rf = tid ? totF[tid - 1] : 0, rb = tid ? totB[tid - 1] : 0;
    if (tid == 0) { PF[0] = 0; PB[0] = 0; }
    for (int l = lo; l < hi; ++l) {
        rf += (unsigned long long)fwd[l];
        rb += (unsigned long long)bwd[l];
        if (rf >= (unsigned long long)PP_CAP62 || rb >= (unsigned long long)PP_CAP62)
            fault |= PP_FAULT_OVERFLOW;
        PF[l + 1] = (long long)rf;
        PB[l + 1] = (long long)rb;
    }
    // a partial total that wrapped shows up in some later chunk's running value or here
    if (totF[tid] >= (unsigned long long)PP_CAP62 || totB[tid] >= (unsigned long long)PP_CAP62)
        fault |= PP_FAULT_OVERFLOW;
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
