// pp_partition_dp: min-max partition of L layers into S contiguous stages, one candidate
// device ordering per workgroup.
//
// Recursion for W(l, xi, r, i) of Sec. IV-B / the PRM listing with one replica per stage:
//   W[0][l] = P[l];  W[n][l] = min_{n<=k<l} max(W[n-1][k], X_n[k], P[l] - P[k]),
// lowest minimising k kept, plan read back from (S-1, L).
//
// Two representations.  When every time is below 2^(31-K) - 1 (K = bits of a split index) a
// cell is a 32-bit key (time << K) | k: the max of two keys whose low bits both equal k keeps
// k, so a plain integer min over k yields the smallest time and, among equal times, the
// lowest k - the required tie-break - at three integer operations per (cell, split) pair.
// Otherwise cells are int64 with an explicit strict-less update.  Which one applies depends
// on the data, which the host cannot see without synchronising, so both kernels are enqueued
// and the one whose turn it is not returns at once.
#include <type_traits>

#include "pp_common.h"

// ---------------------------------------------------------------- pack

// P as int32 and the header's running maximum, seeded with P[L].
__global__ __launch_bounds__(256) void k_pack_p(int L, const long long *__restrict__ PF,
                                                const long long *__restrict__ PB,
                                                pp_ws_header *hdr, int *__restrict__ p32) {
    for (int l = threadIdx.x; l <= L; l += blockDim.x) p32[l] = (int)(PF[l] + PB[l]);
    if (threadIdx.x == 0) {
        long long pl = PF[L] + PB[L];
        hdr->vmax = pl < 0 ? ~0ull : (unsigned long long)pl;
    }
}

// x32[link*L + k] = XF + XB at cut position k (k layers before the cut), k = 1..L-1;
// entry 0 is 0.  Also folds the largest entry into hdr->vmax.
__global__ __launch_bounds__(256) void k_pack_x(int L, size_t total,
                                                const long long *__restrict__ XF,
                                                const long long *__restrict__ XB,
                                                pp_ws_header *hdr, int *__restrict__ x32) {
    unsigned long long m = 0;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (size_t)gridDim.x * blockDim.x) {
        int k = (int)(i % (size_t)L);
        long long x = 0;
        if (k >= 1) x = XF[i - 1] + XB[i - 1];
        x32[i] = (int)x;
        unsigned long long ux = x < 0 ? ~0ull : (unsigned long long)x;
        m = ux > m ? ux : m;
    }
    for (int off = 32; off; off >>= 1) {
        unsigned long long o = __shfl_xor(m, off);
        m = o > m ? o : m;
    }
    if ((threadIdx.x & 63) == 0 && m) atomicMax(&hdr->vmax, m);
}

int pp_launch_pack(int L, int D, const int64_t *PF, const int64_t *PB, const int64_t *XF,
                   const int64_t *XB, void *ws, const pp_ws_layout &lay, hipStream_t st) {
    char *base = (char *)ws;
    pp_ws_header *hdr = (pp_ws_header *)(base + lay.hdr);
    int *p32 = (int *)(base + lay.p32);
    int *x32 = (int *)(base + lay.x32);
    hipLaunchKernelGGL(k_pack_p, dim3(1), dim3(256), 0, st, L, (const long long *)PF,
                       (const long long *)PB, hdr, p32);
    if (hipGetLastError() != hipSuccess) return PP_ERR_HIP;
    size_t total = (size_t)D * D * L;
    int grid = (int)((total + 255) / 256);
    if (grid > 2048) grid = 2048;
    hipLaunchKernelGGL(k_pack_x, dim3(grid), dim3(256), 0, st, L, total, (const long long *)XF,
                       (const long long *)XB, hdr, x32);
    if (hipGetLastError() != hipSuccess) return PP_ERR_HIP;
    return PP_OK;
}

// ---------------------------------------------------------------- generic kernel

struct dp_args {
    int L, D, S, K;
    long long N;
    unsigned long long fit_limit;  // keys are usable iff hdr->vmax < fit_limit
    const long long *PF, *PB, *XF, *XB;
    const int *orderings;
    const pp_ws_header *hdr;
    const int *p32, *x32;
    unsigned short *arg;  // [gridDim.x][S][L+1] backtrack tables, one per resident workgroup
    long long *C_out;
    int *bounds_out;
    int32_t *status;
};

// Loads candidate c's ordering into s_o[0..S-1]; returns false (uniformly) if it is not a
// list of distinct devices below D.  Must be called by the whole workgroup.
__device__ bool load_ordering(const dp_args &a, long long c, int *s_o, int *s_ok) {
    const int tid = threadIdx.x;
    if (tid == 0) *s_ok = 1;
    if (a.orderings) {
        for (int n = tid; n < a.S; n += blockDim.x) s_o[n] = a.orderings[c * a.S + n];
    } else if (tid == 0) {
        unsigned long long rem = (unsigned long long)c;
        unsigned used = 0;
        for (int n = 0; n < a.S; ++n) s_o[n] = pp_unrank_next(a.D, n, rem, used);
    }
    __syncthreads();
    if (a.orderings) {
        for (int n = tid; n < a.S; n += blockDim.x) {
            int d = s_o[n];
            bool bad = d < 0 || d >= a.D;
            for (int q = 0; q < n; ++q) bad |= (s_o[q] == d);
            if (bad) *s_ok = 0;
        }
    }
    __syncthreads();
    return *s_ok != 0;
}

template <bool WIDE>
__global__ __launch_bounds__(256) void k_dp_generic(dp_args a) {
    const bool fits = a.hdr->vmax < a.fit_limit;
    if (fits == WIDE) return;

    using V = typename std::conditional<WIDE, long long, int>::type;
    const V INF = WIDE ? (V)PP_INF64 : (V)PP_INF32;
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int s_o[PP_MAX_STAGES];
    __shared__ int s_ok;
    const int L = a.L, S = a.S, K = a.K, tid = threadIdx.x, B = blockDim.x;
    const int kmask = (1 << K) - 1;
    V *sP = (V *)smem;      // WIDE: P[l];  keys: (P[l] << K) - l
    V *sW = sP + (L + 1);   // row n-1, then row n: W[.][l] (keys: time << K in the high bits)
    V *sG = sW + (L + 1);   // g[k] = max(W[n-1][k], X_n[k])  (keys: | k)
    unsigned short *arg = a.arg + (size_t)blockIdx.x * S * (L + 1);

    for (int l = tid; l <= L; l += B) {
        if (WIDE) sP[l] = (V)(a.PF[l] + a.PB[l]);
        else sP[l] = (V)((a.p32[l] << K) - l);
    }

    for (long long c = blockIdx.x; c < a.N; c += gridDim.x) {
        __syncthreads();
        if (!load_ordering(a, c, s_o, &s_ok)) {
            if (tid == 0) { pp_raise(a.status, PP_FAULT_ORDERING); a.C_out[c] = PP_INF64; }
            for (int n = tid; n < S; n += B) a.bounds_out[c * S + n] = 0;
            continue;
        }
        // one stage holding the first l layers
        for (int l = tid; l <= L; l += B) sW[l] = l ? (WIDE ? sP[l] : sP[l] + l) : INF;

        for (int n = 1; n < S; ++n) {
            __syncthreads();
            const size_t link = ((size_t)s_o[n - 1] * a.D + s_o[n]) * L;
            for (int k = n + tid; k < L; k += B) {
                if (WIDE) {
                    V x = (V)(a.XF[link + k - 1] + a.XB[link + k - 1]);
                    sG[k] = sW[k] > x ? sW[k] : x;
                } else {
                    int xk = (a.x32[link + k] << K) | k;
                    int wk = ((int)sW[k] & ~kmask) | k;
                    sG[k] = (V)(wk > xk ? wk : xk);
                }
            }
            __syncthreads();
            // only W[S-1][L] is needed of the last row
            const int lfirst = (n == S - 1) ? L : n + 1;
            for (int l = lfirst + tid; l <= L; l += B) {
                if (WIDE) {
                    const V Pl = sP[l];
                    V best = INF;
                    int bk = 0;
                    for (int k = n; k < l; ++k) {
                        V d = Pl - sP[k];
                        V t = sG[k] > d ? sG[k] : d;
                        if (t < best) { best = t; bk = k; }
                    }
                    sW[l] = best;
                    arg[n * (L + 1) + l] = (unsigned short)bk;
                } else {
                    const int Pl = (int)sP[l] + l;
                    int best = PP_INF32;
                    for (int k = n; k < l; ++k) {
                        int d = Pl - (int)sP[k];
                        int t = (int)sG[k] > d ? (int)sG[k] : d;
                        best = t < best ? t : best;
                    }
                    sW[l] = (V)best;
                    arg[n * (L + 1) + l] = (unsigned short)(best & kmask);
                }
            }
        }
        __threadfence();
        __syncthreads();
        if (tid == 0) {
            a.C_out[c] = WIDE ? (long long)sW[L] : (long long)((int)sW[L] >> K);
            int e = L;
            for (int n = S - 1; n >= 1; --n) {
                a.bounds_out[c * S + n] = e;
                e = arg[n * (L + 1) + e];
            }
            a.bounds_out[c * S] = e;
        }
    }
}

int pp_launch_dp(int L, int D, int S, int64_t N, const int64_t *PF, const int64_t *PB,
                 const int64_t *XF, const int64_t *XB, const int32_t *orderings, int64_t *C_out,
                 int32_t *bounds_out, void *ws, const pp_ws_layout &lay, int32_t *status,
                 hipStream_t st) {
    char *base = (char *)ws;
    dp_args a;
    a.L = L; a.D = D; a.S = S; a.K = pp_index_bits(L); a.N = N;
    a.fit_limit = (1ull << (31 - a.K)) - 1;
    a.PF = (const long long *)PF; a.PB = (const long long *)PB;
    a.XF = (const long long *)XF; a.XB = (const long long *)XB;
    a.orderings = orderings;
    a.hdr = (const pp_ws_header *)(base + lay.hdr);
    a.p32 = (const int *)(base + lay.p32);
    a.x32 = (const int *)(base + lay.x32);
    a.arg = (unsigned short *)(base + lay.arg);
    a.C_out = (long long *)C_out;
    a.bounds_out = bounds_out;
    a.status = status;
    int block = (L + 63) / 64 * 64;
    if (block > 256) block = 256;
    int grid = lay.slots;
    hipLaunchKernelGGL(k_dp_generic<false>, dim3(grid), dim3(block), (size_t)3 * (L + 1) * 4, st, a);
    if (hipGetLastError() != hipSuccess) return PP_ERR_HIP;
    hipLaunchKernelGGL(k_dp_generic<true>, dim3(grid), dim3(block), (size_t)3 * (L + 1) * 8, st, a);
    if (hipGetLastError() != hipSuccess) return PP_ERR_HIP;
    return PP_OK;
}
