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
//   e = L;  for n = S-1 .. 1:  v = max(m_n, B[n][e]);  e = max(n, lower_bound(P, P[e] - v)).
// One lane per candidate, O(S log L) steps each, all in int64 (no key representation, so no
// limit on the size of the times).
#include "pp_common.h"
#include "pp_dp_generic.h"

struct dp_flat_args {
    dp_args g;
    int steps;       // ceil(log2(L + 1)): halving steps of the search over P[0..L]
    int tables_lds;  // P (padded to 2^steps entries) and B are staged in LDS
};

// LDS: [waves][S][64] prefix maxima m_n, one column per lane; then, if tables_lds, P padded
// with infinity to 2^steps entries and B [S][L+1].
__global__ __launch_bounds__(256) void k_dp_flat(dp_flat_args b) {
    extern __shared__ __align__(16) long long fsm[];
    const dp_args &a = b.g;
    if (!pp_is_flat(a.hdr)) return;  // the general kernel does the work
    const int L = a.L, S = a.S, D = a.D, tid = threadIdx.x, lane = tid & 63;
    const int nP = L + 1, wpb = blockDim.x >> 6;
    long long *mcol = fsm + (size_t)(tid >> 6) * S * 64 + lane;  // m_n at mcol[n * 64]
    const long long *P = a.bfl, *B = a.bfl;
    if (b.tables_lds) {
        long long *sP = fsm + (size_t)wpb * S * 64, *sB = sP + ((size_t)1 << b.steps);
        for (int i = tid; i < (1 << b.steps); i += blockDim.x) sP[i] = i <= L ? a.bfl[i] : PP_INF64;
        for (int i = tid; i < S * nP; i += blockDim.x) sB[i] = a.bfl[i];
        __syncthreads();
        P = sP;
        B = sB;
    }
    const bool padded = b.tables_lds != 0;
    const int tri = S * (S + 1) / 2;
    unsigned long long probes = 0;

    // first index r in 0..L with P[r] >= t (P[L] >= t always holds for the targets used here)
    auto lower_bound = [&](long long t) -> int {
        int pos = 0;
        for (int s = 1 << (b.steps - 1); s; s >>= 1) {
            const int idx = pos + s - 1;
            const long long val = (padded || idx <= L) ? P[idx] : PP_INF64;
            pos += val < t ? s : 0;
        }
        probes += (unsigned)b.steps;
        return pos < L ? pos : L;
    };

    const long long stride = (long long)gridDim.x * blockDim.x;
    for (long long c = (long long)blockIdx.x * blockDim.x + tid; c < a.N; c += stride) {
        const int *o = a.ord + c * S;
        // prefix maxima of the channel times along the ordering (and the checks of a caller's row)
        bool bad = false;
        unsigned long long seen = 0;
        long long run = 0;
        int prev = 0;
        for (int n = 0; n < S; ++n) {
            const int d = o[n];
            if (a.validate) {
                if (d < 0 || d >= D) { bad = true; break; }
                if (D <= 64) {
                    bad |= (seen >> d) & 1ull;
                    seen |= 1ull << d;
                } else {
                    for (int q = 0; q < n; ++q) bad |= (o[q] == d);
                }
                if (bad) break;
            }
            if (n >= 1) {
                const size_t at = ((size_t)prev * D + d) * L;  // the entry of the first cut position
                const long long x = a.XF[at] + a.XB[at];
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
            for (int n = xi - 1; n >= 0; --n) {
                bo[n] = e;
                if (n == 0) break;
                const long long mn = mcol[n * 64], bn = B[(size_t)n * nP + e];
                const long long v = mn > bn ? mn : bn;
                if (n == xi - 1) a.C_out[a.stages ? c * S + xi - 1 : c] = v;
                const int r = lower_bound(P[e] - v);
                e = r > n ? r : n;
            }
            if (xi == 1) a.C_out[a.stages ? c * S : c] = P[L];
        }
    }
    for (int off = 32; off; off >>= 1) probes += __shfl_xor(probes, off);
    if (lane == 0) pp_count_work(a.hdr, probes, 0, blockIdx.x * wpb + (tid >> 6));
}

int pp_launch_dp_flat(const dp_args &g, hipStream_t st) {
    dp_flat_args b;
    b.g = g;
    b.steps = 1;
    while ((1 << b.steps) < g.L + 1) ++b.steps;
    // the columns of prefix maxima take S * 512 bytes per wave: four waves per workgroup up to
    // 16 stages, one beyond (S <= 64: 32 KiB)
    const int wpb = g.S <= 16 ? 4 : 1;
    size_t lds = (size_t)wpb * g.S * 64 * 8;
    const size_t tables = (((size_t)1 << b.steps) + (size_t)g.S * (g.L + 1)) * 8;
    b.tables_lds = lds + tables <= 64 * 1024;
    if (b.tables_lds) lds += tables;
    long long blocks = (g.N + 64 * wpb - 1) / (64 * wpb);
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(k_dp_flat, dim3((unsigned)blocks), dim3(64 * wpb), lds, st, b);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_HIP;
}
