// Partition DP for L <= 128: one wavefront per candidate, cells and splits tiled over the
// 64 lanes, everything that does not depend on the candidate kept in registers.
//
// Recursion for W(l, xi, r, i) of Sec. IV-B / the PRM listing with one replica per stage:
//   W[n][l] = min_{n<=k<l} max(g_n[k], P[l] - P[k]),   g_n[k] = max(W[n-1][k], X_n[k]).
//
// Lane (a, b), a = lane/8, b = lane%8, owns cells l = 8i + a + 1 and splits k = 8j + b
// (i, j = 0..NT-1, NT = ceil(L/8)).  A cell is a 32-bit key (time << K) | k, so that max
// keeps the split index and a plain min over k returns the smallest time with the lowest k.
// The term ((P[l] - P[k]) << K) | k does not depend on the candidate or the row: every lane
// computes its NT(NT+1)/2 values once (invalid pairs k >= l hold the infinite key) and keeps
// them in registers for the lifetime of the wave.  A row then costs, per (cell, split) pair,
// one max and half a three-operand min, plus a 3-step DPP min over the 8 lanes that share a
// cell and 2 operations per split to build g.  Rows live in LDS (their low key bits are the
// backtrack table), one private slice per wave, so there are no barriers.
//
// Row n of a candidate depends only on the first n+1 devices of its ordering.  A wave walks
// a contiguous chunk of candidates and recomputes only the rows from the first position in
// which the ordering differs from the previous candidate's; with all D! orderings in
// lexicographic order most rows are shared.
#include "pp_common.h"
#include "pp_dp_tile.h"

#define DPP_QUAD_XOR1 0xB1   // quad_perm:[1,0,3,2]
#define DPP_QUAD_XOR2 0x4E   // quad_perm:[2,3,0,1]
#define DPP_HALF_MIRROR 0x141  // row_half_mirror: lane b <-> 7-b within each 8 lanes

__device__ __forceinline__ int imin(int a, int b) { return a < b ? a : b; }
__device__ __forceinline__ int imax(int a, int b) { return a > b ? a : b; }

template <int CTRL>
__device__ __forceinline__ int dpp_min(int v) {
    int o = __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, true);
    return imin(v, o);
}

// min over the 8 lanes that share a = lane/8 (all of them get the result)
__device__ __forceinline__ int min_over_b(int v) {
    v = dpp_min<DPP_QUAD_XOR1>(v);
    v = dpp_min<DPP_QUAD_XOR2>(v);
    v = dpp_min<DPP_HALF_MIRROR>(v);
    return v;
}

template <int NT>
__global__ __launch_bounds__(DPT_THREADS) void k_dp_tile(dp_tile_args a) {
    if (!(a.hdr->vmax < a.fit_limit)) return;  // the int64 kernel takes over

    extern __shared__ int lds[];
    constexpr int RS = 8 * NT + 4;  // row stride in dwords: index k (0 = infinite) .. 8NT
    const int lane = threadIdx.x & 63;
    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int la = lane >> 3, lb = lane & 7;
    const int S = a.S, K = a.K, L = a.L, D = a.D;
    const int kmask = (1 << K) - 1;
    int *rows = lds + wib * S * RS;

    // candidate-independent part: Dp[i][j] = ((P[l] - P[k]) << K) | k, or infinite if k >= l
    int Dp[NT * (NT + 1) / 2];
    {
        int Pl[NT], Pk[NT];
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            Pl[i] = a.p32[8 * i + la + 1] << K;
            Pk[i] = (a.p32[8 * i + lb] << K) - (8 * i + lb);
        }
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
            for (int j = 0; j <= i; ++j)
            {
                int d = (j < i || lb <= la) ? Pl[i] - Pk[j] : PP_INF32;
                asm volatile("" : "+v"(d));  // keep the masked value, not the mask, in the loop
                Dp[i * (i + 1) / 2 + j] = d;
            }
        // row 0: one stage holding the first l layers (same for every candidate)
        if (lb == 0) {
#pragma unroll
            for (int i = 0; i < NT; ++i) rows[8 * i + la + 1] = Pl[i];
        }
        // index 0 (no layers before the split) is infeasible in every row
        for (int n = lane; n < S; n += 64) rows[n * RS] = PP_INF32;
    }

    const long long wave = (long long)blockIdx.x * (blockDim.x >> 6) + wib;
    const long long c0 = wave * a.chunk;
    const long long c1 = c0 + a.chunk < a.N ? c0 + a.chunk : a.N;
    if (c0 >= c1) return;
    const unsigned long long smask = S >= 64 ? ~0ull : ((1ull << S) - 1);

    // Lane n carries device o[n] of the candidate (v_o) and the link index o[n-1]*D + o[n]
    // that row n needs (v_link).  `first` is the first row to recompute: rows below it are
    // still valid from the previous candidate of this wave.
    int v_prev = 0;
    bool have_prev = false;
    int v_o = lane < S ? a.ord[c0 * S + lane] : 0;

    // Looks at candidate ordering v (previous one in v_prev): returns the first row to
    // compute, or -1 if the ordering is not a list of distinct devices below D.
    auto inspect = [&](int v) -> int {
        int p = 0;
        if (have_prev) {
            unsigned long long diff = __ballot(v != v_prev) & smask;
            p = diff ? __builtin_ctzll(diff) : S;
        }
        if (a.validate) {
            bool bad = lane < S && (v < 0 || v >= D);
            for (int q = 0; q + 1 < S; ++q) {
                int oq = __builtin_amdgcn_readlane(v, q);
                bad |= (lane > q && lane < S && oq == v);
            }
            if (__ballot(bad)) return -1;
        }
        return p > 1 ? p : 1;
    };
    auto links = [&](int v) -> int {
        int up = __shfl_up(v, 1);
        return up * D + v;
    };
    auto fetch_x = [&](int (&x)[NT], int link) {
        const int *xp = a.xkt + ((size_t)link * 8 + lb) * NT;
#pragma unroll
        for (int j = 0; j < NT; ++j) x[j] = xp[j];
    };

    int first = inspect(v_o);
    int v_link = first >= 0 ? links(v_o) : 0;
    int xk[NT];
    if (first >= 1 && first < S) fetch_x(xk, __builtin_amdgcn_readlane(v_link, first));

    for (long long c = c0; c < c1; ++c) {
        // ordering of the next candidate, needed only after this one's rows
        const bool more = c + 1 < c1;
        int v_on = (more && lane < S) ? a.ord[(c + 1) * S + lane] : 0;

        if (first >= 0) {
            for (int n = first; n < S; ++n) {
                // next row's channel keys are fetched while this row is computed
                int xn[NT];
                if (n + 1 < S) fetch_x(xn, __builtin_amdgcn_readlane(v_link, n + 1));
                const int *prow = rows + (n - 1) * RS;
                int *nrow = rows + n * RS;
                int g[NT];
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    int w = prow[8 * j + lb];
                    // previous row's time with this split's index in the low bits, then the channel
                    int wk = (w & ~kmask) | (xk[j] & kmask);
                    g[j] = imax(wk, xk[j]);
                }
                if (n < S - 1) {
                    int acc[NT];
#pragma unroll
                    for (int i = 0; i < NT; ++i) {
                        int v = PP_INF32;
#pragma unroll
                        for (int j = 0; j <= i; ++j) v = imin(v, imax(g[j], Dp[i * (i + 1) / 2 + j]));
                        acc[i] = v;
                    }
#pragma unroll
                    for (int i = 0; i < NT; ++i) {
                        acc[i] = min_over_b(acc[i]);
                        asm volatile("" : "+v"(acc[i]));
                    }
                    if (lb == 0) {
#pragma unroll
                        for (int i = 0; i < NT; ++i) nrow[8 * i + la + 1] = acc[i];
                    }
                } else {
                    // only W[S-1][L] is needed of the last row; L lies in tile NT-1
                    constexpr int i = NT - 1;
                    int v = PP_INF32;
#pragma unroll
                    for (int j = 0; j <= i; ++j) v = imin(v, imax(g[j], Dp[i * (i + 1) / 2 + j]));
                    v = min_over_b(v);
                    asm volatile("" : "+v"(v));
                    if (lb == 0) nrow[8 * i + la + 1] = v;
                }
                __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int j = 0; j < NT; ++j) xk[j] = xn[j];
            }
        }

        // look at the next candidate and start fetching its first row's channel keys, so
        // that the fetch overlaps this candidate's read-back below
        const bool ok = first >= 0;
        int first_n = 0, v_link_n = 0;
        if (more) {
            if (ok) { v_prev = v_o; have_prev = true; } else { have_prev = false; }
            first_n = inspect(v_on);
            if (first_n >= 0) {
                v_link_n = links(v_on);
                if (first_n < S) fetch_x(xk, __builtin_amdgcn_readlane(v_link_n, first_n));
            }
        }

        if (ok) {
            // bottleneck and plan: every lane follows the same chain, lane n keeps bound n
            int e = L, mine = 0;
            const int top = rows[(S - 1) * RS + L];
            for (int m = S - 1; m >= 1; --m) {
                if (lane == m) mine = e;
                e = rows[m * RS + e] & kmask;
            }
            if (lane == 0) { mine = e; a.C_out[c] = (long long)(top >> K); }
            if (lane < S) a.bounds_out[c * S + lane] = mine;
        } else {
            if (lane == 0) { pp_raise(a.status, PP_FAULT_ORDERING); a.C_out[c] = PP_INF64; }
            if (lane < S) a.bounds_out[c * S + lane] = 0;
        }
        v_o = v_on;
        first = first_n;
        v_link = v_link_n;
    }
}

template <int NT>
static int launch_nt(const dp_tile_args &a, int grid, int wpb, size_t lds, hipStream_t st) {
    hipLaunchKernelGGL(k_dp_tile<NT>, dim3(grid), dim3(64 * wpb), lds, st, a);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_HIP;
}

int pp_launch_dp_tile(const dp_tile_args &a, int nt, int grid, int wpb, hipStream_t st) {
    const size_t lds = (size_t)wpb * a.S * (8 * nt + 4) * 4;
    switch (nt) {
#define CASE(n) case n: return launch_nt<n>(a, grid, wpb, lds, st);
        CASE(1) CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7) CASE(8)
        CASE(9) CASE(10) CASE(11) CASE(12) CASE(13) CASE(14) CASE(15) CASE(16)
#undef CASE
    }
    return PP_ERR_INVALID_ARG;
}
