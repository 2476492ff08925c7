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
// Otherwise cells are int64 with an explicit strict-less update.  And when no link's channel
// time depends on the cut position the whole program has a closed form (pp_dp_flat.h).  Which
// of the three applies depends on the data, which the host cannot see without synchronising:
// the pack kernel leaves what is needed to tell in the workspace header, and the one kernel
// enqueued after it branches on that.
#include "pp_common.h"
#include "pp_dp_generic.h"
#include "pp_dp_tile.h"

// ---------------------------------------------------------------- pack

struct pack_args {
    int L, D, S, K, nt;
    long long N;
    size_t total;  // D*D*L
    const long long *PF, *PB, *XF, *XB;
    pp_ws_header *hdr;
    int *p32, *x32, *xkt, *xct, *ord;  // ord != NULL: write all D! orderings in lexicographic order
    long long *bfl;                    // [S][L+1] partition DP without channel costs
};

// x32[link*L + k] = XF + XB at cut position k (k layers before the cut), k = 1..L-1; entry 0
// is 0.  Returns this thread's largest entry; clears `flat` if an entry differs from the one
// at the previous cut position of the same link.
__device__ unsigned long long pack_x(const pack_args &a, size_t first, size_t stride, bool &flat) {
    unsigned long long m = 0;
    for (size_t i = first; i < a.total; i += stride) {
        int k = a.total <= 0xffffffffu ? (int)((unsigned)i % (unsigned)a.L) : (int)(i % (size_t)a.L);
        long long x = 0;
        if (k >= 1) x = a.XF[i - 1] + a.XB[i - 1];
        if (k >= 2) flat &= (x == a.XF[i - 2] + a.XB[i - 2]);
        a.x32[i] = (int)x;
        unsigned long long ux = x < 0 ? ~0ull : (unsigned long long)x;
        m = ux > m ? ux : m;
    }
    return m;
}

// Tile layout of the same table as keys, for the register-tiled kernel:
// xkt[(link*8 + b)*nt + j] = (x << K) | k for k = 8j + b, infinite for k == 0 or k >= L.
__device__ void pack_xkt(const pack_args &a, unsigned first, unsigned stride) {
    if (!a.nt) return;
    const unsigned per_link = 8u * a.nt, n = (unsigned)a.D * a.D * per_link;  // D*D*128 < 2^32
    for (unsigned i = first; i < n; i += stride) {
        unsigned link = i / per_link;
        int r = (int)(i - link * per_link);
        int b = r / a.nt, j = r - b * a.nt, k = 8 * j + b;
        int key = PP_INF32;
        if (k >= 1 && k < a.L) {
            long long x = a.XF[(size_t)link * a.L + k - 1] + a.XB[(size_t)link * a.L + k - 1];
            key = (int)(((unsigned)x << a.K) | (unsigned)k);
        }
        a.xkt[i] = key;
    }
}

// The same keys once more in the layout of the cells a lane holds after a row's reduction
// (lane (a, b) holds the cells l = 8 (h H + r) + a + 1, h = b / 4, r = 0..H-1, H = ceil(nt / 2)):
// xct[((link*8 + a)*2 + h)*H + r] = (x << K) | l, infinite for l >= L or a tile beyond nt.
__device__ void pack_xct(const pack_args &a, unsigned first, unsigned stride) {
    if (!a.nt) return;
    const unsigned H = (unsigned)(a.nt + 1) / 2, per_link = 16u * H, n = (unsigned)a.D * a.D * per_link;
    for (unsigned i = first; i < n; i += stride) {
        unsigned link = i / per_link, r0 = i - link * per_link;
        unsigned la = r0 / (2 * H), h = (r0 / H) & 1u, r = r0 % H;
        int tile = (int)(h * H + r), l = 8 * tile + (int)la + 1;
        int key = PP_INF32;
        if (tile < a.nt && l < a.L) {
            long long x = a.XF[(size_t)link * a.L + l - 1] + a.XB[(size_t)link * a.L + l - 1];
            key = (int)(((unsigned)x << a.K) | (unsigned)l);
        }
        a.xct[i] = key;
    }
}

// Row c of the explicit list = the ordering of lexicographic rank c.  Its factorial-number
// digits come out least significant first by dividing by 1, 2, 3, ...: digit n (counted from
// the front) = (c / (D-1-n)!) mod (D-n); digit n selects the digit-th smallest unused device.
// 32-bit arithmetic when D! fits (D <= 12).
__device__ void unrank_rows(const pack_args &a, long long first, long long stride) {
    const int D = a.D;
    for (long long c = first; c < a.N; c += stride) {
        unsigned long long digits = 0;  // 5 bits per digit: digits 0..11 here, 12..19 in digits_hi
        unsigned long long digits_hi = 0;
        if (D <= 12) {
            unsigned rem = (unsigned)c;
#pragma unroll
            for (int i = 1; i <= 12; ++i) {  // i = D - n; unrolled: divisions by constants
                if (i > D) break;
                unsigned q = rem / (unsigned)i;
                unsigned long long dg = rem - q * (unsigned)i;
                rem = q;
                digits |= dg << (5 * (D - i));
            }
        } else {
            unsigned long long rem = (unsigned long long)c;
            for (int i = 1; i <= D; ++i) {
                unsigned long long q = rem / (unsigned long long)i;
                unsigned long long dg = rem - q * (unsigned long long)i;
                rem = q;
                int n = D - i;
                if (n < 12) digits |= dg << (5 * n);
                else digits_hi |= dg << (5 * (n - 12));
            }
        }
        unsigned used = 0;
        int row[4];
        const bool vec = (D & 3) == 0;  // rows are 16-byte aligned pieces: store four devices at a time
        for (int n = 0; n < D; ++n) {
            int digit = (int)(((n < 12 ? digits >> (5 * n) : digits_hi >> (5 * (n - 12)))) & 31);
            // digit-th zero bit of `used`
            unsigned freeb = ~used;
            for (int k = 0; k < digit; ++k) freeb &= freeb - 1;
            int dev = __builtin_ctz(freeb);
            used |= 1u << dev;
            if (vec) {
                row[n & 3] = dev;
                if ((n & 3) == 3) *(int4 *)(a.ord + c * D + n - 3) = make_int4(row[0], row[1], row[2], row[3]);
            } else {
                a.ord[c * D + n] = dev;
            }
        }
    }
}

// The partition DP with every channel cost taken as zero, which does not depend on the
// candidate: B[0][l] = P[l], B[n][l] = min_{n<=k<l} max(B[n-1][k], P[l] - P[k]) (infinite for
// l <= n), and A[n][l] = the lowest minimising k.  pp_dp_flat.h builds every candidate's plan
// from these two tables when no link's channel time depends on the cut position.  Rows are
// non-decreasing in l and P[l] - P[k] falls as k grows, so a cell is decided at the first
// split k* where the two cross (binary search): left of it the difference is the larger term,
// from it on the previous row.  If the difference just left of the crossing is no larger than
// the row value at it, the minimum sits there, at the lowest split with that same prefix sum
// (zero-length layers make equal neighbours); otherwise at k*.
// One workgroup; sh holds P and two rows.  a.bfl: B [S][L+1] int64, then A [S][L+1] int32.
__device__ void flat_table(const pack_args &a, long long *sh) {
    const int L = a.L, S = a.S, tid = threadIdx.x;
    // The tables are read only when no link's channel time depends on the cut position.  If
    // some link's times at the first two cut positions already differ, that is not so (the
    // pack blocks will find the same), and the work below can be left out.  Only for long
    // models: for L <= 128 the table is cheap and this launch is on the path of a step of a few
    // tens of microseconds, where the test's own barriers cost more than it can save.
    // (this thread's first entry of P is requested here, so that it travels with the loads of the test)
    const long long p_first = tid <= L ? a.PF[tid] + a.PB[tid] : 0;
    if (L > PP_TILE_MAX_L) {
        __shared__ int s_differs;
        if (tid == 0) s_differs = 0;
        __syncthreads();
        bool differs = false;
        for (int link = tid; link < a.D * a.D; link += 256) {
            if (link / a.D == link % a.D) continue;
            const size_t at = (size_t)link * L;
            differs |= a.XF[at] + a.XB[at] != a.XF[at + 1] + a.XB[at + 1];
        }
        if (differs) s_differs = 1;
        __syncthreads();
        if (s_differs) return;
    }
    long long *P = sh, *cur = sh + (L + 1), *nxt = cur + (L + 1);
    int *A = (int *)(a.bfl + (size_t)S * (L + 1));
    for (int l = tid; l <= L; l += 256) {
        const long long p = l == tid ? p_first : a.PF[l] + a.PB[l];
        P[l] = p;
        cur[l] = p;
        a.bfl[l] = p;
        A[l] = 0;
    }
    __syncthreads();
    for (int n = 1; n < S; ++n) {
        for (int l = tid; l <= L; l += 256) {
            long long best = PP_INF64;
            int arg = 0;
            if (l >= n + 1) {
                const long long Pl = P[l];
                int lo = n, hi = l;  // first split k in [n, l) with row[k] >= P[l] - P[k], or l
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (cur[mid] >= Pl - P[mid]) hi = mid;
                    else lo = mid + 1;
                }
                arg = lo;
                if (lo <= l - 1) best = cur[lo];
                if (lo - 1 >= n) {
                    const long long d = Pl - P[lo - 1];
                    if (d <= best) {
                        best = d;
                        int k = lo - 1;
                        while (k > n && P[k - 1] == P[k]) --k;
                        arg = k;
                    }
                }
            }
            nxt[l] = best;
            a.bfl[(size_t)n * (L + 1) + l] = best;
            A[(size_t)n * (L + 1) + l] = arg;
        }
        // The next row reads this one from LDS only, so the barrier waits for the LDS writes and
        // lets the stores to global memory drain behind it (__syncthreads would wait for them
        // too: a trip to memory per row).
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        long long *t = cur; cur = nxt; nxt = t;
    }
}

// Blocks 0..PP_PACK_BLOCKS-1 pack a slice of the tables each and record the largest time of
// their slice in the header (no atomics, nothing to initialise); further blocks, if any, write
// the explicit list of all D! orderings.  Block PP_PACK_BLOCKS builds the channel-free DP table.
__global__ __launch_bounds__(256) void k_prep(pack_args a) {
    extern __shared__ __align__(16) long long dyn[];
    __shared__ unsigned long long sh[4];
    __shared__ int shf[4];
    const int tid = threadIdx.x;
    if (blockIdx.x < PP_PACK_BLOCKS) {
        const unsigned first = blockIdx.x * 256 + tid, stride = PP_PACK_BLOCKS * 256;
        unsigned long long m = 0;
        if (blockIdx.x == 0) {
            // P as int32, padded with P[L] up to a whole tile
            for (int l = tid; l <= a.L + 16; l += 256) {
                int q = l < a.L ? l : a.L;
                a.p32[l] = (int)(a.PF[q] + a.PB[q]);
            }
            long long pl = a.PF[a.L] + a.PB[a.L];
            m = pl < 0 ? ~0ull : (unsigned long long)pl;
            if (tid < 64) { a.hdr->work[tid].pairs = 0; a.hdr->work[tid].rows = 0; }
        }
        bool flat = true;
        unsigned long long mx = pack_x(a, first, stride, flat);
        m = mx > m ? mx : m;
        pack_xkt(a, first, stride);
        pack_xct(a, first, stride);
        for (int off = 32; off; off >>= 1) {
            unsigned long long o = __shfl_xor(m, off);
            m = o > m ? o : m;
        }
        const int wflat = __ballot(!flat) == 0;
        if ((tid & 63) == 0) { sh[tid >> 6] = m; shf[tid >> 6] = wflat; }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < 4; ++w) m = sh[w] > m ? sh[w] : m;
            a.hdr->pmax[blockIdx.x] = m;
            a.hdr->flat[blockIdx.x] = (unsigned)(shf[0] & shf[1] & shf[2] & shf[3]);
        }
    } else if (blockIdx.x == PP_PACK_BLOCKS) {
        flat_table(a, dyn);
    } else {
        unrank_rows(a, (long long)(blockIdx.x - PP_PACK_BLOCKS - 1) * 256 + tid,
                    (long long)(gridDim.x - PP_PACK_BLOCKS - 1) * 256);
    }
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
    a.xct = (int *)(base + lay.xct);
    a.bfl = (long long *)(base + lay.bfl);
    a.ord = orderings ? NULL : (int *)(base + lay.ord);
    *ord = orderings ? orderings : (const int32_t *)(base + lay.ord);
    int grid = PP_PACK_BLOCKS + 1;
    if (a.ord) grid += (int)((N + 255) / 256 < 1024 ? (N + 255) / 256 : 1024);
    hipLaunchKernelGGL(k_prep, dim3(grid), dim3(256), (size_t)3 * (L + 1) * 8, st, a);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_HIP;
}

// ---------------------------------------------------------------- launch policy

// Consecutive candidates one wave of the tiled kernel walks.
//
// Caller's list: split it evenly over the resident waves.  All D! orderings in
// lexicographic order: consecutive candidates share ordering prefixes and with them DP rows,
// so a wave that walks c candidates computes about c * r + (D - 2 - r) full rows, where
// r = sum_{m=1}^{D-2} 1/m! is the average number of rows that change from one ordering to
// the next; a chunk of k! candidates aligned to a multiple of k! shares its first D-k
// devices and needs exactly (D-k-1) + sum_{n>=D-k} k!/(D-1-n)! rows.  The kernel is bound by
// instruction issue, so a SIMD that holds w waves takes about w times as long as one that
// holds a single wave would at full rate, except that a lone wave cannot hide its own LDS
// and issue latencies and runs about 1.4 times slower per row.  Pick the size that minimises
// (waves on the busiest SIMD) x (rows per wave) under that model.
static long long choose_chunk(int64_t N, int D, bool lex, long long simds, int waves_per_simd) {
    const long long slots = simds * waves_per_simd;
    const long long even = (long long)((N + slots - 1) / slots);
    if (!lex || D < 3) return even;
    double r = 0, term = 1;
    for (int m = 1; m <= D - 2; ++m) { term /= m; r += term; }
    auto cost = [&](long long c, double rows) {
        long long nwaves = (long long)((N + c - 1) / c);
        long long per_simd = (nwaves + simds - 1) / simds;
        if (per_simd > waves_per_simd)  // later waves start as earlier ones finish
            return rows * (double)nwaves / (double)simds;
        return rows * (per_simd <= 1 ? 1.4 : (double)per_simd);
    };
    long long best = even;
    double best_cost = cost(even, even * r + (D - 2 - r) + 0.1 * even);
    long long f = 1;
    for (int k = 1; k < D; ++k) {
        f *= k;
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
        double c = cost(f, rows);
        if (c < best_cost) { best_cost = c; best = f; }
    }
    return best;
}

int pp_launch_dp(int L, int D, int S, int64_t N, const int64_t *PF, const int64_t *PB,
                 const int64_t *XF, const int64_t *XB, const int32_t *lex_ord,
                 const int32_t *user_ord, int stages, int defer_mmax, int keep_list,
                 int64_t *C_out, int32_t *bounds_out, void *ws, const pp_ws_layout &lay,
                 int32_t *status, hipStream_t st) {
    if (keep_list && !lay.sh_table) return PP_ERR_INVALID_ARG;
    char *base = (char *)ws;
    dp_args a;
    a.stages = stages;
    a.L = L; a.D = D; a.S = S; a.K = pp_index_bits(L); a.N = N;
    a.fit_limit = (1ull << (31 - a.K)) - 1;
    a.PF = (const long long *)PF; a.PB = (const long long *)PB;
    a.XF = (const long long *)XF; a.XB = (const long long *)XB;
    a.ord = lex_ord ? lex_ord : user_ord;
    a.validate = user_ord != NULL;
    a.hdr = (pp_ws_header *)(base + lay.hdr);
    a.p32 = (const int *)(base + lay.p32);
    a.x32 = (const int *)(base + lay.x32);
    a.arg = (unsigned short *)(base + lay.arg);
    a.C_out = (long long *)C_out;
    a.bounds_out = bounds_out;
    a.status = status;
    a.nblocks = lay.slots;
    a.bfl = (const long long *)(base + lay.bfl);
    a.defer_mmax = defer_mmax;

    if (lay.nt) {
        // L <= 128: register-tiled kernel, one wave per candidate (falls back to the generic
        // int64 body inside the same launch when the times do not fit 32-bit keys)
        dp_tile_args t;
        t.L = L; t.D = D; t.S = S; t.K = a.K; t.N = N;
        t.validate = a.validate;
        t.xkt = (const int *)(base + lay.xkt);
        t.xct = (const int *)(base + lay.xct);
        int cus = 256;
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            cus = 256;
        const size_t lds_wave = pp_dp_tile_lds_per_wave(S, lay.nt);
        int wpb = 4;  // waves per workgroup, limited by 64 KiB of LDS
        while (wpb > 1 && lds_wave * wpb > 64 * 1024) wpb >>= 1;
        if (lds_wave * wpb > 64 * 1024) return PP_ERR_INVALID_ARG;  // cannot happen for S <= 64
        const int waves_per_simd = lay.nt >= 14 ? 2 : (lay.nt >= 12 ? 3 : 4);
        t.chunk = choose_chunk(N, D, lex_ord != NULL, (long long)cus * 4, waves_per_simd);
        {
            // Priority levels end when a tenth, a quarter and half of the chunk are left: the
            // two waves of a SIMD drift apart while they are on the same level and are pulled
            // together at each boundary, so the levels get shorter towards the end (measured at
            // GPT size against equal quarters: 65.8 against 67.1 us).
            const long long frac[3] = {10, 4, 2};
            for (int k = 0; k < 3; ++k) {
                long long v = t.chunk / frac[k];
                t.prio_left[k] = (int)(v > 0x3fffffff ? 0x3fffffff : v);
            }
        }
        const long long nchunks = (N + t.chunk - 1) / t.chunk;
        const int grid = (int)((nchunks + wpb - 1) / wpb);
        if (a.nblocks > grid) a.nblocks = grid;
        t.g = a;
        return pp_launch_dp_tile(t, lay.nt, grid, wpb, st);
    }
    // L > 128: super-tiled kernel, one persistent wave per candidate slot
    int cus = 256;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        cus = 256;
    long long waves = lay.slots < N ? lay.slots : N;
    if (!lay.sh_table) return pp_launch_dp_big(a, (int)waves, cus, NULL, st);
    // candidates whose links have the same channel times share one DP: the kernel walks the
    // representatives the preparation finds, and their results are copied to the others
    const int run_waves = pp_dp_big_run_waves(pp_dp_big_waves(L, D, S, (int)waves, cus), S, lay.sh_row_slots);
    int rc = pp_launch_share_prepare(L, D, S, N, XF, XB, a.ord, a.validate, keep_list, run_waves, ws, lay, st);
    if (rc) return rc;
    pp_share_list list;
    list.reps = (const int *)(base + lay.sh_reps);
    list.keys = (const int *)(base + lay.sh_keys);
    list.start = (const int *)(base + lay.sh_start);
    list.rows = (int *)(base + lay.sh_rows);
    list.row_slots = lay.sh_row_slots;
    rc = pp_launch_dp_big(a, (int)waves, cus, &list, st);
    if (rc || keep_list) return rc;
    return pp_launch_share_scatter(N, stages ? S : 1, stages ? S * (S + 1) / 2 : S, 0, 1, C_out,
                                   bounds_out, NULL, ws, lay, st);
}
