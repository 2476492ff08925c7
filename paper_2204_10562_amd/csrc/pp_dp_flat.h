// Partition DP in closed form when no link's channel time depends on the cut position
// (equal activation sizes at every layer boundary, as in transformer stacks).
//
// Recursion for W(l, xi, r, i) of Sec. IV-B / the PRM listing with one replica per stage:
//   W[n][l] = min_{n<=k<l} max(W[n-1][k], x_n, P[l] - P[k]),   x_n = X on link o[n-1] -> o[n].
// With x_n constant in k, max with it commutes with the minimum, so by induction
//   W[n][l] = max(m_n, B[n][l]),   m_n = max(x_1..x_n),
// where B is the same recursion with every x taken as 0: one table per problem, built by the
// pack kernel, not one per candidate.  B[n][.] and hence W[n][.] are non-decreasing in l (a
// stage can always be split in two at no cost when channels are free), and P[l] - P[k] falls as
// k grows.  The splits that attain v = W[n][l] are therefore those with W[n-1][k] <= v (a
// prefix of the range) and P[l] - P[k] <= v (a suffix); the lowest of them - the one the
// listing's strict-improvement update keeps - is the first k >= n with P[k] >= P[l] - v.
// A plan is then read back without any row of its own:
//   e = L;  for n = S-1 .. 1:  v = max(m_n, B[n][e]);  e = max(n, lower_bound(P, P[e] - v)),
// and where the channels do not bind (m_n <= B[n][e]) the new e is A[n][e], the split of the
// channel-free table, which the pack kernel stores beside B.  One lane per candidate, all in
// int64 (no key representation, so no limit on the size of the times).
#pragma once

#include "pp_common.h"
#include "pp_dp_generic.h"

// LDS per working wave: a column of prefix maxima (int64) and one of devices, later bounds
// (int32), per lane.
__host__ __device__ static inline size_t pp_flat_col_bytes(int S) { return (size_t)S * 64 * 12; }
__host__ __device__ static inline int pp_flat_steps(int L) {
    int s = 1;
    while ((1 << s) < L + 1) ++s;
    return s;
}
// LDS for the tables, laid out as the pack kernel leaves them in the workspace: B [S][L+1]
// int64 (row 0 = P), then A [S][L+1] int32; rounded up to whole 16-byte pieces.
__host__ __device__ static inline size_t pp_flat_table_bytes(int L, int S) {
    return ((size_t)S * (L + 1) * 12 + 15) & ~(size_t)15;
}
// LDS a launch of `wpb` waves per workgroup should provide so that the closed-form body runs
// with everything staged (it works with less, down to one column: it then leaves waves idle
// and reads the tables from global memory).
static inline size_t pp_flat_lds_wanted(int L, int D, int S, int wpb) {
    size_t want = (size_t)wpb * pp_flat_col_bytes(S) + pp_flat_table_bytes(L, S);
    if (D <= 32) want += (size_t)D * D * 8;
    while (want > 64 * 1024 && wpb > 1) {
        --wpb;
        want -= pp_flat_col_bytes(S);
    }
    if (want > 64 * 1024) want = pp_flat_col_bytes(S);  // tables stay in global memory
    return want;
}

// Sum of a 32-bit value over the 64 lanes (uniform result): four DPP steps inside each row of
// 16 lanes, then the four row sums through scalar registers.
__device__ __forceinline__ unsigned flat_wave_sum(unsigned v) {
    v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, true);   // quad_perm:[1,0,3,2]
    v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, true);   // quad_perm:[2,3,0,1]
    v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, true);  // row_half_mirror
    v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xf, 0xf, true);  // row_mirror
    return (unsigned)__builtin_amdgcn_readlane((int)v, 0) + (unsigned)__builtin_amdgcn_readlane((int)v, 16) +
           (unsigned)__builtin_amdgcn_readlane((int)v, 32) + (unsigned)__builtin_amdgcn_readlane((int)v, 48);
}

// What the body works on: the tables either all staged in LDS (TABLES; the per-link channel
// times too if X is not NULL) or all in global memory.
struct flat_view {
    const long long *P, *B;  // P = row 0 of B
    const int *A;
    const long long *X;      // [D*D] channel time of every link in LDS, or NULL
    long long *mcol;         // this lane's column of prefix maxima: m_n at mcol[n * 64]
    int *ocol;               // this lane's column of devices, later of bounds
    int steps;
    long long c, lanes;      // first candidate of this lane and the stride to its next one
};

template <bool TABLES>
__device__ __forceinline__ void dp_flat_run(const dp_args &a, const flat_view &f, bool row_fetched) {
    const int L = a.L, S = a.S, D = a.D, nP = L + 1, lane = threadIdx.x & 63;
    const long long *P = f.P, *B = f.B;
    const int *A = f.A;
    long long *mcol = f.mcol;
    int *ocol = f.ocol;
    const int tri = S * (S + 1) / 2;
    unsigned probes = 0;
    // first index r in 0..L with P[r] >= t (P[L] >= t holds for every target used here)
    auto lower_bound = [&](long long t) -> int {
        int pos = 0;
        for (int s = 1 << (f.steps - 1); s; s >>= 1) {
            const int idx = pos + s - 1;
            const long long val = P[idx <= L ? idx : L];
            // (beyond L the array would hold infinity: every target is at most P[L])
            pos += val < t ? s : 0;
        }
        probes += (unsigned)f.steps;
        return pos < L ? pos : L;
    };
    auto fetch_row = [&](long long cc) {
        const int *o = a.ord + cc * S;
        for (int n0 = 0; n0 < S; n0 += 8) {
            int v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = n0 + u < S ? o[n0 + u] : 0;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (n0 + u < S) ocol[(n0 + u) * 64] = v[u];
        }
    };

    for (long long c = f.c; c < a.N; c += f.lanes) {
        if (!row_fetched) fetch_row(c);
        row_fetched = false;
        // prefix maxima of the channel times along the ordering (and the checks of a caller's row)
        bool bad = false;
        unsigned long long seen = 0;
        long long run = 0;
        int prev = 0;
        for (int n = 0; n < S; ++n) {
            const int d = ocol[n * 64];
            if (a.validate) {
                if (d < 0 || d >= D) { bad = true; break; }
                if (D <= 64) {
                    bad |= (seen >> d) & 1ull;
                    seen |= 1ull << d;
                } else {
                    for (int q = 0; q < n; ++q) bad |= (ocol[q * 64] == d);
                }
                if (bad) break;
            }
            if (n >= 1) {
                long long x = 0;
                if (TABLES && f.X) x = f.X[prev * D + d];
                else if (L > 1) { const size_t at = ((size_t)prev * D + d) * L; x = a.XF[at] + a.XB[at]; }
                run = x > run ? x : run;
            }
            mcol[n * 64] = run;
            prev = d;
        }
        if (bad) {
            pp_raise(a.status, PP_FAULT_ORDERING);
            if (a.stages) {
                for (int n = 0; n < S; ++n) a.C_out[c * S + n] = PP_INF64;
                for (int n = 0; n < tri; ++n) a.bounds_out[c * tri + n] = 0;
            } else {
                a.C_out[c] = PP_INF64;
                for (int n = 0; n < S; ++n) a.bounds_out[c * S + n] = 0;
            }
            continue;
        }
        // xi = number of stages of the plan read back: S only, or every count 1..S
        for (int xi = a.stages ? 1 : S; xi <= S; ++xi) {
            int *bo = a.bounds_out + (a.stages ? c * tri + xi * (xi - 1) / 2 : c * S);
            int e = L;
            for (int n = xi - 1; n >= 1; --n) {
                ocol[n * 64] = e;  // the devices are no longer needed: the column takes the bounds
                const long long mn = mcol[n * 64], bn = B[(size_t)n * nP + e];
                const int an = A[(size_t)n * nP + e];
                if (n == xi - 1) a.C_out[a.stages ? c * S + xi - 1 : c] = mn > bn ? mn : bn;
                int r = an;
                if (mn > bn) {  // the channels bind: the longest last stage that fits in m_n
                    r = lower_bound(P[e] - mn);
                    r = r > n ? r : n;
                }
                e = r;
                ++probes;
            }
            ocol[0] = e;
            if (xi == 1) a.C_out[a.stages ? c * S : c] = P[L];
            // the row goes out in pieces of 16 bytes where it can
            if ((xi & 3) == 0 && (((size_t)bo & 15) == 0)) {
                for (int n = 0; n < xi; n += 4)
                    *(int4 *)(bo + n) = make_int4(ocol[n * 64], ocol[(n + 1) * 64], ocol[(n + 2) * 64], ocol[(n + 3) * 64]);
            } else {
                for (int n = 0; n < xi; ++n) bo[n] = ocol[n * 64];
            }
        }
    }
    const unsigned total = flat_wave_sum(probes);
    if (lane == 0) pp_count_work(a.hdr, total, 0, blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6));
}

// The same for S <= 8 with the candidate's devices, prefix maxima and bounds in registers and
// every loop over stages unrolled: the channel times of all links of the row are looked up
// side by side instead of one after the other.  row[] holds the devices of the lane's first
// candidate (if it has one).
template <bool TABLES>
__device__ __forceinline__ void dp_flat_run8(const dp_args &a, const flat_view &f, int (&row)[8], bool row_fetched) {
    const int L = a.L, S = a.S, D = a.D, nP = L + 1, lane = threadIdx.x & 63;
    const long long *P = f.P, *B = f.B;
    const int *A = f.A;
    const int tri = S * (S + 1) / 2;
    unsigned probes = 0;
    auto lower_bound = [&](long long t) -> int {
        int pos = 0;
        for (int s = 1 << (f.steps - 1); s; s >>= 1) {
            const int idx = pos + s - 1;
            const long long val = P[idx <= L ? idx : L];
            pos += val < t ? s : 0;
        }
        probes += (unsigned)f.steps;
        return pos < L ? pos : L;
    };
    for (long long c = f.c; c < a.N; c += f.lanes) {
        if (!row_fetched) {
#pragma unroll
            for (int u = 0; u < 8; ++u) row[u] = u < S ? a.ord[c * S + u] : 0;
        }
        row_fetched = false;
        bool bad = false;
        if (a.validate) {
#pragma unroll
            for (int n = 0; n < 8; ++n) {
                if (n >= S) break;
                bad |= row[n] < 0 || row[n] >= D;
#pragma unroll
                for (int q = 0; q < n; ++q) bad |= row[q] == row[n];
            }
        }
        if (bad) {
            pp_raise(a.status, PP_FAULT_ORDERING);
            if (a.stages) {
                for (int n = 0; n < S; ++n) a.C_out[c * S + n] = PP_INF64;
                for (int n = 0; n < tri; ++n) a.bounds_out[c * tri + n] = 0;
            } else {
                a.C_out[c] = PP_INF64;
                for (int n = 0; n < S; ++n) a.bounds_out[c * S + n] = 0;
            }
            continue;
        }
        // channel time of link n-1 -> n, all looked up before any is used, then the prefix maxima
        long long m[8];
        m[0] = 0;
#pragma unroll
        for (int n = 1; n < 8; ++n) {
            long long x = 0;
            if (n < S) {
                const int link = row[n - 1] * D + row[n];
                if (TABLES && f.X) x = f.X[link];
                else if (L > 1) x = a.XF[(size_t)link * L] + a.XB[(size_t)link * L];
            }
            m[n] = x;
        }
#pragma unroll
        for (int n = 1; n < 8; ++n) m[n] = m[n] > m[n - 1] ? m[n] : m[n - 1];
        for (int xi = a.stages ? 1 : S; xi <= S; ++xi) {
            int *bo = a.bounds_out + (a.stages ? c * tri + xi * (xi - 1) / 2 : c * S);
            int e = L;
            int b[8];
#pragma unroll
            for (int n = 7; n >= 1; --n) {
                b[n] = e;
                if (n <= xi - 1) {
                    const long long mn = m[n], bn = B[(size_t)n * nP + e];
                    const int an = A[(size_t)n * nP + e];
                    if (n == xi - 1) a.C_out[a.stages ? c * S + xi - 1 : c] = mn > bn ? mn : bn;
                    int r = an;
                    if (mn > bn) {  // the channels bind: the longest last stage that fits in m_n
                        r = lower_bound(P[e] - mn);
                        r = r > n ? r : n;
                    }
                    e = r;
                    ++probes;
                }
            }
            b[0] = e;
            if (xi == 1) a.C_out[a.stages ? c * S : c] = P[L];
            if (xi == 8 && (((size_t)bo & 15) == 0)) {
                *(int4 *)bo = make_int4(b[0], b[1], b[2], b[3]);
                *(int4 *)(bo + 4) = make_int4(b[4], b[5], b[6], b[7]);
            } else {
#pragma unroll
                for (int n = 0; n < 8; ++n)
                    if (n < xi) bo[n] = b[n];
            }
        }
    }
    const unsigned total = flat_wave_sum(probes);
    if (lane == 0) pp_count_work(a.hdr, total, 0, blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6));
}

// True (uniformly) if the plans of this call are built by the makespan kernel that follows
// (same test as there: pp_makespan.hip, fused_gather).  All lanes of a full wave must call.
__device__ __forceinline__ bool dp_flat_deferred(const dp_args &a) {
    if (!a.defer_mmax) return false;
    // (lane b looks at the largest time of pack block b: all below the limit = their maximum is)
    const unsigned long long limit = 0x7fffffffull / (unsigned long long)(a.defer_mmax + 4 * a.S - 4);
    return !__ballot(a.hdr->pmax[threadIdx.x & (PP_PACK_BLOCKS - 1)] > limit);
}

// Must be entered by whole workgroups of full waves; lds_bytes = dynamic LDS of the launch
// (at least pp_flat_col_bytes(S)).
__device__ inline void dp_flat_body(const dp_args &a, unsigned char *smem, size_t lds_bytes) {
    const int L = a.L, S = a.S, D = a.D, tid = threadIdx.x, lane = tid & 63;
    const int nP = L + 1, wpb = blockDim.x >> 6, wib = tid >> 6;
    const int steps = pp_flat_steps(L);
    const size_t col = pp_flat_col_bytes(S), tab = pp_flat_table_bytes(L, S);
    int ncols = (int)(lds_bytes / col);
    ncols = ncols < wpb ? ncols : wpb;
    size_t rest = lds_bytes - (size_t)ncols * col;
    // give up columns (down to one) if that lets the tables in
    while (ncols > 1 && rest < tab) { --ncols; rest += col; }
    const bool tables = rest >= tab;
    const bool xtab = tables && D <= 32 && rest - tab >= (size_t)D * D * 8;

    const long long *gB = a.bfl;
    const int *gA = (const int *)(a.bfl + (size_t)S * nP);
    long long *mcols = (long long *)smem;                     // [ncols][S][64]
    int *ocols = (int *)(smem + (size_t)ncols * S * 64 * 8);  // [ncols][S][64]
    long long *sB = (long long *)(smem + (size_t)ncols * col);
    int *sA = (int *)(sB + (size_t)S * nP);
    long long *sX = (long long *)((unsigned char *)sB + tab);
    flat_view f;
    f.steps = steps;
    f.mcol = mcols + (size_t)wib * S * 64 + lane;
    f.ocol = ocols + (size_t)wib * S * 64 + lane;
    f.lanes = (long long)gridDim.x * ncols * 64;
    f.c = ((long long)blockIdx.x * ncols + wib) * 64 + lane;
    const bool worker = wib < ncols;
    if ((long long)blockIdx.x * ncols * 64 >= a.N) return;  // (the whole workgroup: no candidate)

    // Everything this workgroup needs from global memory is requested before anything is
    // waited for, so that the prologue costs one trip to memory: the per-link channel times,
    // the first 8 devices of this lane's first candidate, the two tables (contiguous in the
    // workspace, copied in 16-byte pieces, 4 per thread and pass).
    long long xf = 0, xb = 0;
    if (xtab && tid < D * D && L > 1) { xf = a.XF[(size_t)tid * L]; xb = a.XB[(size_t)tid * L]; }
    int row[8];
    const bool fetched = worker && f.c < a.N;
#pragma unroll
    for (int u = 0; u < 8; ++u) row[u] = (fetched && u < S) ? a.ord[f.c * S + u] : 0;
    if (tables) {
        const int4 *src = (const int4 *)gB;  // the workspace region is 256-byte aligned and padded
        int4 *dst = (int4 *)sB;
        const int n16 = (int)(tab / 16), B4 = blockDim.x;
        for (int i = tid; i < n16; i += 4 * B4) {
            int4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = i + u * B4 < n16 ? src[i + u * B4] : make_int4(0, 0, 0, 0);
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (i + u * B4 < n16) dst[i + u * B4] = v[u];
        }
        if (xtab)
            for (int i = tid; i < D * D; i += blockDim.x) {
                if (i >= blockDim.x && L > 1) { xf = a.XF[(size_t)i * L]; xb = a.XB[(size_t)i * L]; }
                sX[i] = xf + xb;
            }
    }
    if (fetched) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (u < S) f.ocol[u * 64] = row[u];
        for (int n = 8; n < S; ++n) f.ocol[n * 64] = a.ord[f.c * S + n];
    }
    __syncthreads();
    if (!worker) return;
    if (tables && S <= 8) {
        f.P = sB; f.B = sB; f.A = sA; f.X = xtab ? sX : NULL;
        dp_flat_run8<true>(a, f, row, fetched);
    } else if (tables) {
        f.P = sB; f.B = sB; f.A = sA; f.X = xtab ? sX : NULL;
        dp_flat_run<true>(a, f, fetched);
    } else {
        f.P = gB; f.B = gB; f.A = gA; f.X = NULL;
        dp_flat_run<false>(a, f, fetched);
    }
}
