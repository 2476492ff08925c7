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
#include "pp_dp_tile.h"

// ---------------------------------------------------------------- pack

struct pack_args {
    int L, D, S, K, nt;
    long long N;
    size_t total;  // D*D*L
    const long long *PF, *PB, *XF, *XB;
    pp_ws_header *hdr;
    int *p32, *x32, *xkt, *ord;  // ord != NULL: write all D! orderings in lexicographic order
};

// P as int32, padded with P[L] up to a whole tile.
__device__ void pack_p(const pack_args &a, int tid, int nthreads) {
    for (int l = tid; l <= a.L + 16; l += nthreads) {
        int q = l < a.L ? l : a.L;
        a.p32[l] = (int)(a.PF[q] + a.PB[q]);
    }
}

// x32[link*L + k] = XF + XB at cut position k (k layers before the cut), k = 1..L-1; entry 0
// is 0.  Returns this thread's largest entry.
__device__ unsigned long long pack_x(const pack_args &a, size_t first, size_t stride) {
    unsigned long long m = 0;
    for (size_t i = first; i < a.total; i += stride) {
        int k = (int)(i % (size_t)a.L);
        long long x = 0;
        if (k >= 1) x = a.XF[i - 1] + a.XB[i - 1];
        a.x32[i] = (int)x;
        unsigned long long ux = x < 0 ? ~0ull : (unsigned long long)x;
        m = ux > m ? ux : m;
    }
    return m;
}

// Tile layout of the same table as keys, for the register-tiled kernel:
// xkt[(link*8 + b)*nt + j] = (x << K) | k for k = 8j + b, infinite for k == 0 or k >= L.
__device__ void pack_xkt(const pack_args &a, size_t first, size_t stride) {
    if (!a.nt) return;
    const size_t per_link = (size_t)8 * a.nt, n = (size_t)a.D * a.D * per_link;
    for (size_t i = first; i < n; i += stride) {
        size_t link = i / per_link;
        int r = (int)(i - link * per_link);
        int b = r / a.nt, j = r - b * a.nt, k = 8 * j + b;
        int key = PP_INF32;
        if (k >= 1 && k < a.L) {
            long long x = a.XF[link * a.L + k - 1] + a.XB[link * a.L + k - 1];
            key = (int)(((unsigned)x << a.K) | (unsigned)k);
        }
        a.xkt[i] = key;
    }
}

__device__ unsigned long long wave_max(unsigned long long m) {
    for (int off = 32; off; off >>= 1) {
        unsigned long long o = __shfl_xor(m, off);
        m = o > m ? o : m;
    }
    return m;
}

__device__ void unrank_rows(const pack_args &a, long long first, long long stride) {
    for (long long c = first; c < a.N; c += stride) {
        unsigned long long rem = (unsigned long long)c;
        unsigned used = 0;
        for (int n = 0; n < a.S; ++n) a.ord[c * a.S + n] = pp_unrank_next(a.D, n, rem, used);
    }
}

// Small tables: block 0 packs everything and writes the header without atomics; the other
// blocks (if any) write the explicit ordering list.
__global__ __launch_bounds__(256) void k_prep_small(pack_args a) {
    __shared__ unsigned long long sh[4];
    const int tid = threadIdx.x;
    if (blockIdx.x == 0) {
        pack_p(a, tid, 256);
        unsigned long long m = wave_max(pack_x(a, tid, 256));
        pack_xkt(a, tid, 256);
        if ((tid & 63) == 0) sh[tid >> 6] = m;
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < 4; ++w) m = sh[w] > m ? sh[w] : m;
            long long pl = a.PF[a.L] + a.PB[a.L];
            unsigned long long up = pl < 0 ? ~0ull : (unsigned long long)pl;
            a.hdr->vmax = up > m ? up : m;
        }
    } else if (a.ord) {
        unrank_rows(a, (long long)(blockIdx.x - 1) * 256 + tid, (long long)(gridDim.x - 1) * 256);
    }
}

// Large tables: header seeded by one kernel, entries folded in with atomicMax by the next.
__global__ __launch_bounds__(256) void k_pack_p(pack_args a) {
    pack_p(a, threadIdx.x, 256);
    if (threadIdx.x == 0) {
        long long pl = a.PF[a.L] + a.PB[a.L];
        a.hdr->vmax = pl < 0 ? ~0ull : (unsigned long long)pl;
    }
}

__global__ __launch_bounds__(256) void k_pack_x(pack_args a) {
    const size_t first = (size_t)blockIdx.x * 256 + threadIdx.x, stride = (size_t)gridDim.x * 256;
    unsigned long long m = wave_max(pack_x(a, first, stride));
    pack_xkt(a, first, stride);
    if ((threadIdx.x & 63) == 0 && m) atomicMax(&a.hdr->vmax, m);
    if (a.ord) unrank_rows(a, (long long)first, (long long)stride);
}

int pp_launch_pack(int L, int D, int S, int64_t N, const int64_t *PF, const int64_t *PB,
                   const int64_t *XF, const int64_t *XB, const int32_t *orderings, void *ws,
                   const pp_ws_layout &lay, const int32_t **ord, hipStream_t st) {
    char *base = (char *)ws;
    pack_args a;
    a.L = L; a.D = D; a.S = S; a.K = pp_index_bits(L); a.nt = lay.nt; a.N = N;
    a.total = (size_t)D * D * L;
    a.PF = (const long long *)PF; a.PB = (const long long *)PB;
    a.XF = (const long long *)XF; a.XB = (const long long *)XB;
    a.hdr = (pp_ws_header *)(base + lay.hdr);
    a.p32 = (int *)(base + lay.p32);
    a.x32 = (int *)(base + lay.x32);
    a.xkt = (int *)(base + lay.xkt);
    a.ord = orderings ? NULL : (int *)(base + lay.ord);
    *ord = orderings ? orderings : (const int32_t *)(base + lay.ord);
    if (a.total <= (size_t)1 << 16) {
        int grid = 1;
        if (a.ord) grid += (int)((N + 255) / 256 < 1024 ? (N + 255) / 256 : 1024);
        hipLaunchKernelGGL(k_prep_small, dim3(grid), dim3(256), 0, st, a);
        return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_HIP;
    }
    hipLaunchKernelGGL(k_pack_p, dim3(1), dim3(256), 0, st, a);
    if (hipGetLastError() != hipSuccess) return PP_ERR_HIP;
    size_t work = a.total > (size_t)N ? a.total : (size_t)N;
    int grid = (int)((work + 255) / 256 < 2048 ? (work + 255) / 256 : 2048);
    hipLaunchKernelGGL(k_pack_x, dim3(grid), dim3(256), 0, st, a);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_HIP;
}

// ---------------------------------------------------------------- generic kernel

struct dp_args {
    int L, D, S, K;
    long long N;
    unsigned long long fit_limit;  // keys are usable iff hdr->vmax < fit_limit
    const long long *PF, *PB, *XF, *XB;
    const int *ord;  // [N][S] explicit orderings
    int validate;    // the list came from the caller: check every row
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

// Consecutive candidates one wave of the tiled kernel walks.  For all D! orderings in
// lexicographic order a chunk of k! candidates shares its first D-k devices, so rows
// 1..D-k-1 are computed once per chunk and row n >= D-k once per distinct prefix; pick the k
// that minimises (rounds of chunks over the resident waves) x (rows per chunk).
static long long choose_chunk(int64_t N, int S, int D, bool lex, long long wave_slots) {
    if (!lex) return (long long)((N + wave_slots - 1) / wave_slots);
    long long best_chunk = 1;
    double best_cost = 1e300;
    long long f = 1;
    for (int k = 0; k < D; ++k) {
        if (k) f *= k;
        if (f > N) break;
        double rows = 0.1 * (double)f;  // last row: one cell per candidate
        for (int n = 1; n <= D - 2; ++n) {
            double nodes = 1;  // row n is shared by the whole chunk when n <= D-k-1
            if (n >= D - k) {
                nodes = (double)f;
                for (int q = 2; q <= D - 1 - n; ++q) nodes /= q;
            }
            rows += nodes;
        }
        long long nch = (long long)(N / f);
        double rounds = (double)((nch + wave_slots - 1) / wave_slots);
        double cost = rounds * rows;
        if (cost < best_cost) { best_cost = cost; best_chunk = f; }
    }
    (void)S;
    return best_chunk;
}

int pp_launch_dp(int L, int D, int S, int64_t N, const int64_t *PF, const int64_t *PB,
                 const int64_t *XF, const int64_t *XB, const int32_t *lex_ord,
                 const int32_t *user_ord, int64_t *C_out, int32_t *bounds_out, void *ws,
                 const pp_ws_layout &lay, int32_t *status, hipStream_t st) {
    char *base = (char *)ws;
    dp_args a;
    a.L = L; a.D = D; a.S = S; a.K = pp_index_bits(L); a.N = N;
    a.fit_limit = (1ull << (31 - a.K)) - 1;
    a.PF = (const long long *)PF; a.PB = (const long long *)PB;
    a.XF = (const long long *)XF; a.XB = (const long long *)XB;
    a.ord = lex_ord ? lex_ord : user_ord;
    a.validate = user_ord != NULL;
    a.hdr = (const pp_ws_header *)(base + lay.hdr);
    a.p32 = (const int *)(base + lay.p32);
    a.x32 = (const int *)(base + lay.x32);
    a.arg = (unsigned short *)(base + lay.arg);
    a.C_out = (long long *)C_out;
    a.bounds_out = bounds_out;
    a.status = status;
    int block = (L + 63) / 64 * 64;
    if (block > 256) block = 256;
    const int grid = lay.slots;

    if (lay.nt) {
        // 32-bit keys, L <= 128: register-tiled kernel, one wave per candidate
        dp_tile_args t;
        t.L = L; t.D = D; t.S = S; t.K = a.K; t.N = N;
        t.fit_limit = a.fit_limit;
        t.validate = a.validate;
        t.hdr = a.hdr; t.p32 = a.p32;
        t.xkt = (const int *)(base + lay.xkt);
        t.ord = a.ord;
        t.C_out = a.C_out; t.bounds_out = bounds_out; t.status = status;
        int cus = 256;
        int dev = 0;
        if (hipGetDevice(&dev) == hipSuccess)
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        const size_t lds_wave = (size_t)S * (8 * lay.nt + 4) * 4;
        int wpb = 4;  // waves per workgroup, limited by 64 KiB of LDS
        while (wpb > 1 && lds_wave * wpb > 64 * 1024) wpb >>= 1;
        if (lds_wave * wpb > 64 * 1024) return PP_ERR_INVALID_ARG;  // cannot happen: S*132*4 <= 33 KiB
        const int waves_per_simd = lay.nt >= 15 ? 2 : (lay.nt >= 13 ? 3 : 4);
        const long long slots = (long long)cus * 4 * waves_per_simd;
        t.chunk = choose_chunk(N, S, D, lex_ord != NULL, slots);
        const long long nchunks = (N + t.chunk - 1) / t.chunk;
        int rc = pp_launch_dp_tile(t, lay.nt, (int)((nchunks + wpb - 1) / wpb), wpb, st);
        if (rc) return rc;
    } else {
        hipLaunchKernelGGL(k_dp_generic<false>, dim3(grid), dim3(block), (size_t)3 * (L + 1) * 4, st, a);
        if (hipGetLastError() != hipSuccess) return PP_ERR_HIP;
    }
    hipLaunchKernelGGL(k_dp_generic<true>, dim3(grid), dim3(block), (size_t)3 * (L + 1) * 8, st, a);
    if (hipGetLastError() != hipSuccess) return PP_ERR_HIP;
    return PP_OK;
}
