// Generic partition DP: any L, 32-bit keys or int64 values.  Shared by the stand-alone
// generic kernel and by the tiled kernel's fallback for times that do not fit 32-bit keys.
//
// Recursion for W(l, xi, r, i) of Sec. IV-B / the PRM listing with one replica per stage:
//   W[0][l] = P[l];  W[n][l] = min_{n<=k<l} max(W[n-1][k], X_n[k], P[l] - P[k]),
// lowest minimising k kept, plan read back from (S-1, L).
#pragma once

#include <type_traits>

#include "pp_common.h"

struct dp_args {
    int L, D, S, K;
    long long N;
    unsigned long long fit_limit;  // keys are usable iff hdr->vmax < fit_limit
    const long long *PF, *PB, *XF, *XB;
    const int *ord;  // [N][S] explicit orderings
    int validate;    // the list came from the caller: check every row
    pp_ws_header *hdr;
    const int *p32, *x32;
    const long long *bfl;  // the partition DP with no channel cost (values, then splits), see pp_dp_flat.h
    size_t lds_bytes;      // dynamic LDS of the launch
    // > 0: when the closed form applies and the finish times of a schedule of defer_mmax
    // microbatches fit 32 bits, leave the plans to the makespan kernel that follows
    int defer_mmax;
    unsigned short *arg;  // [nblocks][S][L+1] backtrack tables, one per working workgroup
    int nblocks;          // workgroups that take part (the rest of the grid returns)
    // stages == 0: C_out [N], bounds_out [N][S]: the plan with S stages.
    // stages == 1: the plan for every stage count xi = 1..S on the first xi devices (row xi-1
    // of the same table, read at cell L): C_out [N][S], bounds_out [N][S(S+1)/2] with the xi
    // bounds of stage count xi at offset xi(xi-1)/2.
    int stages;
    long long *C_out;
    int *bounds_out;
    int32_t *status;
};

// Kernel for 128 < L with 32-bit keys (pp_dp_big.hip): persistent waves, as many as fit the
// GPU (cus compute units) but at most max_waves (the backtrack tables the workspace holds).
// list: what pp_launch_share_prepare leaves in the workspace (representatives, every
// candidate's key, room for saved rows), or NULL.
struct pp_share_list {
    const int *reps, *keys, *start;
    int *rows;
    long long row_slots;  // rows of (128 ceil(L / 128) + 4) keys that fit the area
};
int pp_launch_dp_big(const dp_args &g, int max_waves, int cus, const pp_share_list *list,
                     hipStream_t st);
// The waves pp_launch_dp_big will use for this shape, and how many of them can walk the list of
// representatives (each needs room for S - 2 saved rows).
int pp_dp_big_waves(int L, int D, int S, int max_waves, int cus);
static inline int pp_dp_big_run_waves(int waves, int S, long long row_slots) {
    long long nw = row_slots / (S > 3 ? S - 2 : 1);
    nw = nw < waves ? nw : waves;
    return (int)(nw > 1 ? nw : 1);
}

// Loads candidate c's ordering into s_o[0..S-1]; returns false (uniformly) if it is not a
// list of distinct devices below D.  Must be called by the whole workgroup.
__device__ inline bool load_ordering(const dp_args &a, long long c, int *s_o, int *s_ok) {
    const int tid = threadIdx.x;
    if (tid == 0) *s_ok = 1;
    for (int n = tid; n < a.S; n += blockDim.x) s_o[n] = a.ord[c * a.S + n];
    __syncthreads();
    if (a.validate) {
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

// One workgroup per candidate (workgroup b walks candidates b, b + nblocks, ...), cells
// spread over the threads, rows in LDS (smem: 3 * (L+1) values of 4 or 8 bytes), backtrack
// table in the workgroup's slice of a.arg.  Must be entered by whole workgroups.
template <bool WIDE>
__device__ void dp_generic_body(const dp_args &a, unsigned char *smem) {
    if ((int)blockIdx.x >= a.nblocks) return;
    using V = typename std::conditional<WIDE, long long, int>::type;
    const V INF = WIDE ? (V)PP_INF64 : (V)PP_INF32;
    __shared__ int s_o[PP_MAX_STAGES];
    __shared__ int s_ok;
    __shared__ long long s_top[PP_MAX_STAGES];  // W[n][L] of every row (stage-count search)
    const int tri = a.S * (a.S + 1) / 2;
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

    unsigned long long pairs = 0, nrows = 0;  // work done by this workgroup (kept by thread 0)
    for (long long c = blockIdx.x; c < a.N; c += a.nblocks) {
        __syncthreads();
        if (!load_ordering(a, c, s_o, &s_ok)) {
            if (tid == 0) pp_raise(a.status, PP_FAULT_ORDERING);
            if (a.stages) {
                for (int n = tid; n < S; n += B) a.C_out[c * S + n] = PP_INF64;
                for (int n = tid; n < tri; n += B) a.bounds_out[c * tri + n] = 0;
            } else {
                if (tid == 0) a.C_out[c] = PP_INF64;
                for (int n = tid; n < S; n += B) a.bounds_out[c * S + n] = 0;
            }
            continue;
        }
        // one stage holding the first l layers
        for (int l = tid; l <= L; l += B) {
            sW[l] = l ? (WIDE ? sP[l] : sP[l] + l) : INF;
            if (l == L) s_top[0] = (long long)sW[l];
        }

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
                    if (l == L) s_top[n] = (long long)best;
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
                    if (l == L) s_top[n] = (long long)best;
                }
            }
        }
        // the backtrack table was written by the whole workgroup and is read by a few of its
        // threads: a workgroup-scope fence is enough (and much cheaper than a device-scope one)
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
        __syncthreads();
        if (a.stages) {
            // thread xi-1 reads back the plan with xi stages from (xi-1, L)
            for (int t = tid; t < S; t += B) {
                a.C_out[c * S + t] = WIDE ? s_top[t] : (long long)((int)s_top[t] >> K);
                int *bo = a.bounds_out + c * tri + t * (t + 1) / 2;
                int e = L;
                for (int n = t; n >= 1; --n) {
                    bo[n] = e;
                    e = arg[n * (L + 1) + e];
                }
                bo[0] = e;
            }
        } else if (tid == 0) {
            a.C_out[c] = WIDE ? (long long)sW[L] : (long long)((int)sW[L] >> K);
            int e = L;
            for (int n = S - 1; n >= 1; --n) {
                a.bounds_out[c * S + n] = e;
                e = arg[n * (L + 1) + e];
            }
            a.bounds_out[c * S] = e;
        }
        if (tid == 0) {
            for (int n = 1; n < S - 1; ++n) pairs += (unsigned long long)(L - n) * (L - n + 1) / 2;
            if (S > 1) pairs += (unsigned long long)(L - S + 1);
            nrows += S - 1;
        }
    }
    if (tid == 0) pp_count_work(a.hdr, pairs, nrows, blockIdx.x);
}

