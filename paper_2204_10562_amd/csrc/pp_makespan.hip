// pp_schedule_makespan: per-iteration time of a plan under the pipeline execution scheduler
// (Alg. 1, Sec. IV-A), and the candidate arg-min of the SPP listing (Alg. 3).
//
// The scheduler's two phases collapse into a max-plus recurrence.  Its ordering phase moves
// every microbatch one block per sweep, so block j serves microbatch m = t - j + 1 in sweep
// t; each of the R = 2S-1 serial resources (stages, and one channel per stage pair for both
// directions) serves its items in (sweep, block) order, and an item starts when its
// microbatch has left block j-1 (which happened in sweep t-1) and the resource is idle:
//     fin_t[j] = max(fin_{t-1}[j-1], idle(resource of j)) + dur[j],
// where a resource's idle time is the latest finish of its two blocks j and 2R-j (finish
// times on one resource never decrease).  Within a sweep the forward block of a resource
// precedes its backward block.  All blocks of a sweep depend only on the sweep before (the
// anti-diagonal t = m + j - 1 of the (block, microbatch) grid), so one lane can carry one
// candidate with all lanes running the same uniform loop.
#include "pp_common.h"

// One lane per candidate; the lane's state (block durations, last finish per block) lives
// in its own LDS column [row][lane], so there are no bank conflicts and no barriers.
// blockDim.x = lanes in use (64, or fewer when 2 * (4S-3) rows of 64 would not fit in LDS).
__global__ __launch_bounds__(64) void k_makespan_lds(
    int L, int D, int S, long long N, int M, const long long *__restrict__ PF,
    const long long *__restrict__ PB, const long long *__restrict__ XF,
    const long long *__restrict__ XB, const int *__restrict__ orderings,
    const int *__restrict__ bounds, long long *__restrict__ T_out, int32_t *status) {
    extern __shared__ long long sm[];
    const int lane = threadIdx.x, W = blockDim.x;
    const int R = 2 * S - 1, J = 2 * R - 1;
    // rows 0..J-1: duration of block j = row+1; rows J..2J-1: its latest finish time
    long long *dur = sm + lane;
    long long *fin = sm + (size_t)J * W + lane;
    const long long c = (long long)blockIdx.x * W + lane;
    const bool live = c < N;
    int fault = 0;

    if (live) {
        // ordering must be distinct devices below D
        if (orderings) {
            for (int n = 0; n < S; ++n) {
                int d = orderings[c * S + n];
                bool bad = d < 0 || d >= D;
                for (int q = 0; q < n; ++q) bad |= (orderings[c * S + q] == d);
                if (bad) fault |= PP_FAULT_ORDERING;
            }
        }
        int prev = 0;
        for (int n = 0; n < S; ++n) {
            int e = bounds[c * S + n];
            if (e <= prev || e > L) fault |= PP_FAULT_BOUNDS;
            prev = e;
        }
        if (prev != L) fault |= PP_FAULT_BOUNDS;
    }
    long long worst = 0;
    {
        unsigned long long rem = (unsigned long long)(live ? c : 0);
        unsigned used = 0;
        int e_prev = 0, o_prev = 0;
        for (int n = 0; n < S; ++n) {
            long long F = 0, Bk = 0, cf = 0, cb = 0;
            int o_n = 0;
            if (live && !fault) {
                o_n = orderings ? orderings[c * S + n] : pp_unrank_next(D, n, rem, used);
                int e = bounds[c * S + n];
                F = PF[e] - PF[e_prev];
                Bk = PB[e] - PB[e_prev];
                if (n) {
                    size_t at = ((size_t)o_prev * D + o_n) * L + (size_t)(e_prev - 1);
                    cf = XF[at];
                    cb = XB[at];
                }
                e_prev = e;
                o_prev = o_n;
            }
            worst = max(worst, max(F + Bk, cf + cb));
            const int r = 2 * n + 1;  // stage n is resource 2n+1, channel n is resource 2n
            if (n == S - 1) {
                dur[(size_t)(R - 1) * W] = F + Bk;  // merged forward+backward block
            } else {
                dur[(size_t)(r - 1) * W] = F;
                dur[(size_t)((2 * R - r) - 1) * W] = Bk;
            }
            if (n) {
                dur[(size_t)((r - 1) - 1) * W] = cf;
                dur[(size_t)((2 * R - (r - 1)) - 1) * W] = cb;
            }
        }
    }
    // the schedule is no longer than (M + 4S - 4) * C (Lemma 1)
    if (live && !fault && worst > (PP_CAP62 - 1) / ((long long)M + 4 * S - 4))
        fault |= PP_FAULT_OVERFLOW;

    for (int j = 1; j <= J; ++j) fin[(size_t)(j - 1) * W] = 0;

    const int sweeps = M + 2 * R - 2;
    for (int t = 1; t <= sweeps; ++t) {
        const int jlo = max(1, t - M + 1), jhi = min(J, t);
        const long long finR_prev = fin[(size_t)(R - 1) * W];
        // forward blocks (and the merged block R), descending so that fin[j-1] is still the
        // previous sweep's value
        for (int j = min(jhi, R); j >= jlo; --j) {
            long long idle = max(fin[(size_t)(j - 1) * W], fin[(size_t)((2 * R - j) - 1) * W]);
            long long ready = j > 1 ? fin[(size_t)((j - 1) - 1) * W] : 0;
            fin[(size_t)(j - 1) * W] = max(idle, ready) + dur[(size_t)(j - 1) * W];
        }
        // backward blocks: the resource may just have been used by this sweep's forward block
        for (int j = jhi; j >= max(jlo, R + 1); --j) {
            long long idle = max(fin[(size_t)(j - 1) * W], fin[(size_t)((2 * R - j) - 1) * W]);
            long long ready = j == R + 1 ? finR_prev : fin[(size_t)((j - 1) - 1) * W];
            fin[(size_t)(j - 1) * W] = max(idle, ready) + dur[(size_t)(j - 1) * W];
        }
    }
    if (live) {
        T_out[c] = fault ? PP_INF64 : fin[(size_t)(J - 1) * W];
        if (fault) pp_raise(status, fault);
    }
}

int pp_launch_makespan(int L, int D, int S, int64_t N, int M, const int64_t *PF, const int64_t *PB,
                       const int64_t *XF, const int64_t *XB, const int32_t *orderings,
                       const int32_t *bounds, int64_t *T_out, int32_t *status, hipStream_t st) {
    const int J = 4 * S - 3;
    int W = 64;  // lanes per workgroup: as many as keep 2J rows of int64 within 64 KiB of LDS
    while ((size_t)2 * J * W * 8 > 64 * 1024) W >>= 1;
    size_t lds = (size_t)2 * J * W * 8;
    unsigned grid = (unsigned)((N + W - 1) / W);
    hipLaunchKernelGGL(k_makespan_lds, dim3(grid), dim3(W), lds, st, L, D, S, (long long)N, M,
                       (const long long *)PF, (const long long *)PB, (const long long *)XF,
                       (const long long *)XB, orderings, bounds, (long long *)T_out, status);
    if (hipGetLastError() != hipSuccess) return PP_ERR_HIP;
    return PP_OK;
}

// ---------------------------------------------------------------- candidate arg-min

struct tc_pair { long long T, c; };

__device__ __forceinline__ tc_pair tc_min(tc_pair a, tc_pair b) {
    return (b.T < a.T || (b.T == a.T && b.c < a.c)) ? b : a;
}

__device__ tc_pair block_tc_min(tc_pair v, tc_pair *sh) {
    for (int off = 32; off; off >>= 1) {
        tc_pair o;
        o.T = __shfl_xor(v.T, off);
        o.c = __shfl_xor(v.c, off);
        v = tc_min(v, o);
    }
    const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    if ((threadIdx.x & 63) == 0) sh[wave] = v;
    __syncthreads();
    if (threadIdx.x == 0)
        for (int w = 1; w < nw; ++w) v = tc_min(v, sh[w]);
    return v;  // valid in thread 0
}

__global__ __launch_bounds__(256) void k_argmin_partial(long long N, const long long *__restrict__ T,
                                                        tc_pair *__restrict__ part) {
    __shared__ tc_pair sh[4];
    tc_pair v = {PP_INF64, INT64_MAX};
    for (long long c = (long long)blockIdx.x * blockDim.x + threadIdx.x; c < N;
         c += (long long)gridDim.x * blockDim.x) {
        tc_pair o = {T[c], c};
        v = tc_min(v, o);
    }
    v = block_tc_min(v, sh);
    if (threadIdx.x == 0) part[blockIdx.x] = v;
}

__global__ __launch_bounds__(256) void k_argmin_final(int parts, int D, int S,
                                                      const tc_pair *__restrict__ part,
                                                      const long long *__restrict__ C,
                                                      const int *__restrict__ bounds,
                                                      const int *__restrict__ orderings,
                                                      pp_result *out) {
    __shared__ tc_pair sh[4];
    tc_pair v = {PP_INF64, INT64_MAX};
    for (int i = threadIdx.x; i < parts; i += blockDim.x) v = tc_min(v, part[i]);
    v = block_tc_min(v, sh);
    if (threadIdx.x == 0) {
        const bool none = v.T == PP_INF64;
        out->best_index = none ? -1 : v.c;
        out->T = v.T;
        out->C = none ? PP_INF64 : C[v.c];
        out->S = S;
        unsigned long long rem = (unsigned long long)(none ? 0 : v.c);
        unsigned used = 0;
        for (int n = 0; n < PP_MAX_STAGES; ++n) {
            int b = 0, o = 0;
            if (n < S && !none) {
                b = bounds[v.c * S + n];
                o = orderings ? orderings[v.c * S + n] : pp_unrank_next(D, n, rem, used);
            }
            out->bounds[n] = b;
            out->order[n] = o;
        }
    }
}

int pp_launch_argmin(int D, int S, int64_t N, const int64_t *T, const int64_t *C,
                     const int32_t *bounds, const int32_t *orderings, void *part, pp_result *out,
                     hipStream_t st) {
    int parts = (int)((N + 255) / 256);
    if (parts > PP_ARGMIN_PARTS) parts = PP_ARGMIN_PARTS;
    hipLaunchKernelGGL(k_argmin_partial, dim3(parts), dim3(256), 0, st, (long long)N,
                       (const long long *)T, (tc_pair *)part);
    if (hipGetLastError() != hipSuccess) return PP_ERR_HIP;
    hipLaunchKernelGGL(k_argmin_final, dim3(1), dim3(256), 0, st, parts, D, S,
                       (const tc_pair *)part, (const long long *)C, bounds, orderings, out);
    if (hipGetLastError() != hipSuccess) return PP_ERR_HIP;
    return PP_OK;
}
