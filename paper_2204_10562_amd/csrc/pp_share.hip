// One partition DP for all candidates that are the same problem.
//
// Row n of the recursion for W(l, xi, r, i) (Sec. IV-B with one replica per stage) sees a
// candidate's devices only through X_n[k], the time link (o[n-1], o[n]) needs for the
// activations at cut position k.  Real clusters have few distinct bandwidths (Sec. III-A: PCIe
// or NVLink inside a server, RDMA or TCP between servers; the testbeds of Sec. V-A have one of
// each), so many links carry the same row X[.], and two candidates whose links have equal rows
// position by position get the same table, bottleneck and plan.  This file finds those groups
// on the device:
//   1. k_share_hash     a hash of every link's forward and backward row (one wave per link),
//                       and the table of representatives set to "none";
//   2. k_share_classes  link i joins the class of the lowest link with the same hash whose rows
//                       are equal entry by entry (one wave per link);
//   3. k_share_keys     classes numbered 0..nc-1; a candidate's key is its sequence of S-1
//                       class numbers read as a number in base nc (first link most
//                       significant), and the lowest candidate of every key is kept with an
//                       atomic min (only if nc^(S-1) fits the table);
//   4. k_share_count, k_share_reps   the table compacted, in the order of the keys, into the
//                       list of representatives;
//   5. k_share_cost, k_share_bounds  the list cut into runs of about equal work, one per wave
//                       of the DP kernel.
// The DP kernel walks the list - neighbours in it share their first links and with them the
// first rows of the table - and k_share_scatter hands every representative's results to the
// candidates of its key.  Candidates with a bad ordering are representatives of themselves
// (kept after the sorted ones), so the DP kernel reports them as it always does.
//
// When the keys do not fit the table (every link its own class) there is still something to
// share: row n depends on the first n + 1 devices only, and a long sampled list holds each
// choice of the first few devices many times.  The same kernels then sort the candidates by
// their first k devices (D^k <= table entries; a counting sort: histogram in k_share_keys,
// bucket offsets in k_share_count / k_share_reps, placement in k_share_place), the list holds
// all N candidates, and the DP kernel reuses the first k - 1 rows between neighbours.  All decisions are taken on the device; when
// the keys do not fit the table the kernels return at once and the DP runs over all candidates.
#include "pp_common.h"

struct share_args {
    int L, D, S, validate;
    long long N;
    const long long *XF, *XB;
    const int *ord;
    pp_ws_header *hdr;
    unsigned long long *lhash;  // [D*D]
    int *lrep;                  // [D*D] lowest link with equal rows (-1 on the diagonal)
    int *table;                 // [PP_SHARE_TABLE] lowest candidate of every key
    int *keys;                  // [N] key of every candidate (-1: bad ordering)
    int *reps;                  // [N] representatives (see pp_share_at)
    int *cnt;                   // [PP_SHARE_TABLE / 256] keys in use per 256 table entries
    int *start;                 // [run_waves + 1] first list entry of every run
    int run_waves;
    // arg-min partials to preset (pairs of int64), or NULL
    long long *part;
    long long n_part;
    // scatter
    int nC, nB, nT, tw, vec;
    long long *C_out, *T_out;
    int *bounds_out;
};

#define SHARE_NONE 0x7fffffff
#define SHARE_FILL_BLOCKS 256

// (a finaliser in the style of splitmix64: multiply, fold the high bits down, twice)
__device__ __forceinline__ unsigned long long share_mix(unsigned long long z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__global__ __launch_bounds__(256) void k_share_hash(share_args a) {
    const int nl = a.D * a.D, hash_blocks = (nl + 3) / 4;
    const int tid = threadIdx.x, lane = tid & 63;
    if ((int)blockIdx.x >= hash_blocks) {
        // the table of representatives: every key empty
        const int b = blockIdx.x - hash_blocks;
        int4 *t4 = (int4 *)a.table;
        const int4 none = make_int4(SHARE_NONE, SHARE_NONE, SHARE_NONE, SHARE_NONE);
        for (int i = b * 256 + tid; i < PP_SHARE_TABLE / 4; i += SHARE_FILL_BLOCKS * 256) t4[i] = none;
        return;
    }
    if (blockIdx.x == 0 && tid == 0) {
        a.hdr->share_active = 0;
        a.hdr->share_nc = 0;
        a.hdr->share_tsize = 0;
        a.hdr->share_nreps = 0;
        a.hdr->share_nsorted = 0;
        a.hdr->share_nbad = 0;
        a.hdr->share_sorted = 0;
        a.hdr->share_kdev = 0;
        a.hdr->share_nchunks = 0;
    }
    const int i = blockIdx.x * 4 + (tid >> 6);
    if (i >= nl) return;
    const int u = i / a.D, v = i - u * a.D;
    unsigned long long h = 0;
    if (u != v) {
        // the entries a plan can read: cut positions 1..L-1, stored at 0..L-2
        const long long *xf = a.XF + (size_t)i * a.L, *xb = a.XB + (size_t)i * a.L;
        for (int k = lane; k < a.L - 1; k += 64)
            h += share_mix(share_mix((unsigned long long)xf[k] + 0x9E3779B97F4A7C15ull * (unsigned)(k + 1)) ^
                           (unsigned long long)xb[k]);
        for (int off = 32; off; off >>= 1) h += __shfl_xor(h, off);
    }
    if (lane == 0) a.lhash[i] = h;
}

__global__ __launch_bounds__(256) void k_share_classes(share_args a) {
    const int nl = a.D * a.D, D = a.D, L = a.L;
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= nl) return;
    if (i / D == i % D) {
        if (lane == 0) a.lrep[i] = -1;
        return;
    }
    const unsigned long long h = a.lhash[i];
    int rep = i;
    for (int base = 0; base < i && rep == i; base += 64) {
        const int j = base + lane;
        const bool m = j < i && j / D != j % D && a.lhash[j] == h;
        unsigned long long mask = __ballot(m);
        while (mask) {
            const int j0 = base + __builtin_ctzll(mask);
            mask &= mask - 1;
            bool diff = false;
            const long long *xi = a.XF + (size_t)i * L, *xj = a.XF + (size_t)j0 * L;
            const long long *yi = a.XB + (size_t)i * L, *yj = a.XB + (size_t)j0 * L;
            for (int k = lane; k < L - 1; k += 64) diff |= xi[k] != xj[k] || yi[k] != yj[k];
            if (!__ballot(diff)) {
                // the lowest link with these rows: it is its own representative
                rep = j0;
                break;
            }
        }
    }
    if (lane == 0) a.lrep[i] = rep;
}

__global__ __launch_bounds__(256) void k_share_keys(share_args a) {
    __shared__ int s_cls[PP_SHARE_MAX_D * PP_SHARE_MAX_D];
    __shared__ int s_cnt[256];
    const int nl = a.D * a.D, D = a.D, S = a.S, tid = threadIdx.x;
    // class numbers: the rank of a link's representative among the representatives
    const int per = (nl + 255) / 256, lo = tid * per, hi = lo + per < nl ? lo + per : nl;
    int cnt = 0;
    for (int i = lo; i < hi; ++i) cnt += a.lrep[i] == i;
    s_cnt[tid] = cnt;
    __syncthreads();
    int before = 0, nc = 0;
    for (int t = 0; t < 256; ++t) {
        const int v = s_cnt[t];
        before += t < tid ? v : 0;
        nc += v;
    }
    for (int i = lo; i < hi; ++i)
        if (a.lrep[i] == i) s_cls[i] = before++;
    __syncthreads();
    int mine[(PP_SHARE_MAX_D * PP_SHARE_MAX_D + 255) / 256];
    for (int i = lo; i < hi; ++i) {
        const int r = a.lrep[i];
        mine[i - lo] = r >= 0 ? s_cls[r] : 0;
    }
    __syncthreads();
    for (int i = lo; i < hi; ++i) s_cls[i] = mine[i - lo];
    __syncthreads();
    // keys are S-1 digits in base nc
    unsigned tsize = 1;
    for (int n = 1; n < S; ++n) {
        const unsigned long long t = (unsigned long long)tsize * (unsigned)nc;
        tsize = t <= PP_SHARE_TABLE ? (unsigned)t : 0;
    }
    if (nc == 0) tsize = S > 1 ? 0 : 1;
    // otherwise: buckets of the first kdev devices (at least two, or there is no row to share)
    int kdev = 0;
    unsigned nbuck = 1;
    if (!tsize) {
        while (kdev < S && (unsigned long long)nbuck * (unsigned)D <= PP_SHARE_TABLE) { nbuck *= (unsigned)D; ++kdev; }
        if (kdev < 2 || S < 3) kdev = 0;
    }
    if (blockIdx.x == 0 && tid == 0) {
        a.hdr->share_nc = (unsigned)nc;
        a.hdr->share_tsize = tsize ? tsize : (kdev ? nbuck : 0);
        a.hdr->share_active = tsize != 0;
        a.hdr->share_sorted = kdev != 0;
        a.hdr->share_kdev = (unsigned)kdev;
    }
    const bool vec = (S & 3) == 0 && ((uintptr_t)a.ord & 15) == 0;
    if (!tsize) {
        if (!kdev) return;
        // histogram of the buckets (the table starts at SHARE_NONE everywhere: counts are taken
        // relative to that, in unsigned arithmetic)
        for (long long c = (long long)blockIdx.x * 256 + tid; c < a.N; c += (long long)gridDim.x * 256) {
            const int *row = a.ord + c * S;
            unsigned key = 0;
            for (int n = 0; n < kdev; ++n) {
                int d = row[n];
                d = (d < 0 || d >= D) ? 0 : d;  // (a bad row is found by the DP kernel; any bucket will do)
                key = key * (unsigned)D + (unsigned)d;
            }
            a.keys[c] = (int)key;
            atomicAdd((unsigned *)&a.table[key], 1u);
        }
        return;
    }
    for (long long c = (long long)blockIdx.x * 256 + tid; c < a.N; c += (long long)gridDim.x * 256) {
        const int *row = a.ord + c * S;
        unsigned long long used = 0;
        unsigned key = 0;
        bool bad = false;
        int prev = 0;
        auto step = [&](int n, int d) {
            if (a.validate) {
                if (d < 0 || d >= D) { bad = true; d = 0; }
                bad |= (used >> d) & 1;
                used |= 1ull << d;
            }
            if (n) key = key * (unsigned)nc + (unsigned)s_cls[prev * D + d];
            prev = d;
        };
        if (vec) {
            // (a row is S devices of 4 bytes: 16 bytes at a time where rows are so aligned)
            for (int n = 0; n < S; n += 4) {
                const int4 v = *(const int4 *)(row + n);
                step(n, v.x); step(n + 1, v.y); step(n + 2, v.z); step(n + 3, v.w);
            }
        } else {
            for (int n = 0; n < S; ++n) step(n, row[n]);
        }
        if (bad) {
            a.keys[c] = -1;
            a.reps[a.N - 1 - atomicAdd(&a.hdr->share_nbad, 1u)] = (int)c;
        } else {
            a.keys[c] = (int)key;
            // (most candidates of a common key arrive after a lower one: a look first spares
            // the atomic, which would queue behind all others on the same address)
            if (__hip_atomic_load(&a.table[key], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) > (int)c)
                atomicMin(&a.table[key], (int)c);
        }
    }
}

// Keys in use in every block of 256 table entries.
__global__ __launch_bounds__(256) void k_share_count(share_args a) {
    __shared__ int sh[4];
    const unsigned tsize = a.hdr->share_tsize;
    const unsigned key = blockIdx.x * 256u + threadIdx.x;
    int n;
    if (a.hdr->share_sorted) {
        // candidates in the bucket
        n = key < tsize ? (int)((unsigned)a.table[key] - (unsigned)SHARE_NONE) : 0;
        for (int off = 32; off; off >>= 1) n += __shfl_xor(n, off);
    } else {
        const bool has = key < tsize && a.table[key] != SHARE_NONE;
        n = __builtin_popcountll(__ballot(has));
    }
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = n;
    __syncthreads();
    if (threadIdx.x == 0) a.cnt[blockIdx.x] = sh[0] + sh[1] + sh[2] + sh[3];
}

__global__ __launch_bounds__(256) void k_share_reps(share_args a) {
    __shared__ int sh[4], shw[4];
    const int tid = threadIdx.x, lane = tid & 63, wib = tid >> 6;
    // (T, candidate) = "none" in every slot of the arg-min's partials: the makespan kernel that
    // walks the list writes only the slots of the waves that have a representative
    for (long long i = (long long)blockIdx.x * 256 + tid; i < a.n_part; i += (long long)gridDim.x * 256) {
        a.part[2 * i] = PP_INF64;
        a.part[2 * i + 1] = INT64_MAX;
    }
    const unsigned tsize = a.hdr->share_tsize;
    if (blockIdx.x * 256u >= tsize && blockIdx.x) return;
    // keys in use before this block's (block 0: in all blocks, for the header)
    const int upto = blockIdx.x ? (int)blockIdx.x : PP_SHARE_TABLE / 256;
    int sum = 0;
    for (int i = tid; i < upto; i += 256) sum += a.cnt[i];
    for (int off = 32; off; off >>= 1) sum += __shfl_xor(sum, off);
    if (lane == 0) sh[wib] = sum;
    __syncthreads();
    const int before = sh[0] + sh[1] + sh[2] + sh[3];
    if (blockIdx.x == 0) {
        if (tid == 0) {
            a.hdr->share_nsorted = (unsigned)before;
            a.hdr->share_nreps = (unsigned)before + a.hdr->share_nbad;
        }
    }
    const int base = blockIdx.x ? before : 0;
    const unsigned key = blockIdx.x * 256u + tid;
    if (a.hdr->share_sorted) {
        // every bucket's first position in the list (k_share_place hands the positions out)
        if (blockIdx.x == 0 && tid == 0) a.hdr->share_nsorted = a.hdr->share_nreps = (unsigned)a.N;
        const int n = key < tsize ? (int)((unsigned)a.table[key] - (unsigned)SHARE_NONE) : 0;
        int incl = n;
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(incl, off);
            incl += lane >= off ? o : 0;
        }
        if (lane == 63) shw[wib] = incl;
        __syncthreads();
        int at = base + incl - n;
        for (int w = 0; w < wib; ++w) at += shw[w];
        if (key < tsize) a.table[key] = at;
        return;
    }
    const int c = key < tsize ? a.table[key] : SHARE_NONE;
    const bool has = c != SHARE_NONE;
    const unsigned long long mask = __ballot(has);
    if (lane == 0) shw[wib] = __builtin_popcountll(mask);
    __syncthreads();
    int at = base + __builtin_popcountll(mask & ((1ull << lane) - 1));
    for (int w = 0; w < wib; ++w) at += shw[w];
    if (has) a.reps[at] = c;
}

// Work of representative r of the sorted list when it follows r - 1 in a run: the rows its key
// does not share with its predecessor's (at least the last one), plus one row's worth for what
// a candidate costs besides its rows.  A run's first entry computes all S - 1 rows.
__device__ __forceinline__ int share_cost(const share_args &a, long long r) {
    const int S = a.S;
    if (r == 0 || S < 3) return S;
    const unsigned key = (unsigned)a.keys[a.reps[r]], prev = (unsigned)a.keys[a.reps[r - 1]];
    const unsigned nc = a.hdr->share_nc;
    unsigned pw = a.hdr->share_tsize / nc;  // weight of the first digit
    int p = 0;
    for (int n = 1; n < S - 1 && key / pw == prev / pw; ++n) { ++p; pw /= nc; }
    return S - p;
}

// Sum of share_cost over every 256 entries of the sorted list (cnt is free again by now).
__global__ __launch_bounds__(256) void k_share_cost(share_args a) {
    __shared__ int sh[4];
    if (!a.hdr->share_active) return;
    const long long r = (long long)blockIdx.x * 256 + threadIdx.x;
    int c = r < (long long)a.hdr->share_nsorted ? share_cost(a, r) : 0;
    for (int off = 32; off; off >>= 1) c += __shfl_xor(c, off);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) a.cnt[blockIdx.x] = sh[0] + sh[1] + sh[2] + sh[3];
}

// Cuts the sorted list into runs of about total / run_waves work each (never less than S + 1, so
// that the running sum crosses at most one boundary per entry): start[w] = first entry of run w.
__global__ __launch_bounds__(256) void k_share_bounds(share_args a) {
    __shared__ long long sh[4], s_excl[256];
    if (!a.hdr->share_active) return;
    const int tid = threadIdx.x, lane = tid & 63, wib = tid >> 6;
    const long long ns = a.hdr->share_nsorted;
    if (ns == 0) {
        if (blockIdx.x == 0 && tid == 0) { a.hdr->share_nchunks = 0; a.start[0] = 0; }
        return;
    }
    if ((long long)blockIdx.x * 256 >= ns) return;
    // work before this block, and in all
    const int nblk = (int)((ns + 255) / 256);
    long long before = 0, total = 0;
    for (int i = tid; i < nblk; i += 256) {
        const int v = a.cnt[i];
        total += v;
        before += i < (int)blockIdx.x ? v : 0;
    }
    for (int off = 32; off; off >>= 1) { before += __shfl_xor(before, off); total += __shfl_xor(total, off); }
    if (lane == 0) { sh[wib] = before; s_excl[wib] = total; }
    __syncthreads();
    before = sh[0] + sh[1] + sh[2] + sh[3];
    total = s_excl[0] + s_excl[1] + s_excl[2] + s_excl[3];
    __syncthreads();
    long long quota = (total + a.run_waves - 1) / a.run_waves;
    quota = quota > a.S + 1 ? quota : a.S + 1;
    const long long r = (long long)blockIdx.x * 256 + tid;
    const int c = r < ns ? share_cost(a, r) : 0;
    long long incl = c;
    for (int off = 1; off < 64; off <<= 1) {
        const long long o = __shfl_up(incl, off);
        incl += lane >= off ? o : 0;
    }
    if (lane == 63) sh[wib] = incl;
    __syncthreads();
    long long excl = before + incl - c;
    for (int w = 0; w < wib; ++w) excl += sh[w];
    s_excl[tid] = excl;
    __syncthreads();
    if (r >= ns) return;
    const long long id = excl / quota;
    long long id_prev = -1;
    if (tid) id_prev = s_excl[tid - 1] / quota;
    else if (r) id_prev = (excl - share_cost(a, r - 1)) / quota;
    if (id != id_prev) a.start[id] = (int)r;
    if (r == ns - 1) {
        a.start[id + 1] = (int)ns;
        a.hdr->share_nchunks = (unsigned)(id + 1);
    }
}

// Counting sort, last step: every candidate takes the next free position of its bucket.
__global__ __launch_bounds__(256) void k_share_place(share_args a) {
    if (!a.hdr->share_sorted) return;
    for (long long c = (long long)blockIdx.x * 256 + threadIdx.x; c < a.N; c += (long long)gridDim.x * 256)
        a.reps[atomicAdd(&a.table[a.keys[c]], 1)] = (int)c;
}

// Every candidate that is not the representative of its key takes the representative's
// results.
__global__ __launch_bounds__(256) void k_share_scatter(share_args a) {
    if (!a.hdr->share_active) return;
    for (long long c = (long long)blockIdx.x * 256 + threadIdx.x; c < a.N; c += (long long)gridDim.x * 256) {
        const int key = a.keys[c];
        if (key < 0) continue;
        const long long r = a.table[key];
        if (r == c) continue;
        for (int i = 0; i < a.nC; ++i) a.C_out[c * a.nC + i] = a.C_out[r * a.nC + i];
        for (int q = 0; q < a.nT; ++q)
            for (int i = 0; i < a.tw; ++i) a.T_out[(q * a.N + c) * a.tw + i] = a.T_out[(q * a.N + r) * a.tw + i];
        if (a.vec) {
            const int4 *src = (const int4 *)(a.bounds_out + r * a.nB);
            int4 *dst = (int4 *)(a.bounds_out + c * a.nB);
            for (int i = 0; i < a.nB / 4; ++i) dst[i] = src[i];
        } else {
            for (int i = 0; i < a.nB; ++i) a.bounds_out[c * a.nB + i] = a.bounds_out[r * a.nB + i];
        }
    }
}

static share_args share_base(void *ws, const pp_ws_layout &lay) {
    char *base = (char *)ws;
    share_args a = {};
    a.hdr = (pp_ws_header *)(base + lay.hdr);
    a.lhash = (unsigned long long *)(base + lay.sh_hash);
    a.lrep = (int *)(base + lay.sh_rep);
    a.table = (int *)(base + lay.sh_table);
    a.keys = (int *)(base + lay.sh_keys);
    a.reps = (int *)(base + lay.sh_reps);
    a.cnt = (int *)(base + lay.sh_cnt);
    a.start = (int *)(base + lay.sh_start);
    return a;
}

static long long share_grid(int64_t N) {
    const long long g = (N + 255) / 256;
    return g < 4096 ? g : 4096;
}

int pp_launch_share_prepare(int L, int D, int S, int64_t N, const int64_t *XF, const int64_t *XB,
                            const int32_t *ord, int validate, int fill_part, int run_waves, void *ws,
                            const pp_ws_layout &lay, hipStream_t st) {
    if (!lay.sh_table || run_waves < 1 || run_waves > PP_DP_SLOTS) return PP_ERR_INVALID_ARG;
    share_args a = share_base(ws, lay);
    if (fill_part) {
        a.part = (long long *)((char *)ws + lay.part);
        a.n_part = (long long)((N + 63) / 64) * PP_MAX_M_LIST;
    }
    a.L = L; a.D = D; a.S = S; a.N = N; a.validate = validate;
    a.XF = (const long long *)XF; a.XB = (const long long *)XB;
    a.ord = ord;
    a.run_waves = run_waves;
    const int link_blocks = (D * D + 3) / 4;
    hipLaunchKernelGGL(k_share_hash, dim3(link_blocks + SHARE_FILL_BLOCKS), dim3(256), 0, st, a);
    hipLaunchKernelGGL(k_share_classes, dim3(link_blocks), dim3(256), 0, st, a);
    hipLaunchKernelGGL(k_share_keys, dim3((unsigned)share_grid(N)), dim3(256), 0, st, a);
    hipLaunchKernelGGL(k_share_count, dim3(PP_SHARE_TABLE / 256), dim3(256), 0, st, a);
    hipLaunchKernelGGL(k_share_reps, dim3(PP_SHARE_TABLE / 256), dim3(256), 0, st, a);
    hipLaunchKernelGGL(k_share_place, dim3((unsigned)share_grid(N)), dim3(256), 0, st, a);
    hipLaunchKernelGGL(k_share_cost, dim3((unsigned)share_grid(N)), dim3(256), 0, st, a);
    hipLaunchKernelGGL(k_share_bounds, dim3((unsigned)share_grid(N)), dim3(256), 0, st, a);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_HIP;
}

int pp_launch_share_scatter(int64_t N, int nC, int nB, int nT, int tw, int64_t *C_out,
                            int32_t *bounds_out, int64_t *T_out, void *ws, const pp_ws_layout &lay,
                            hipStream_t st) {
    if (!lay.sh_table) return PP_ERR_INVALID_ARG;
    share_args a = share_base(ws, lay);
    a.N = N; a.nC = nC; a.nB = nB; a.nT = nT; a.tw = tw;
    a.C_out = (long long *)C_out;
    a.T_out = (long long *)T_out;
    a.bounds_out = bounds_out;
    a.vec = nB > 0 && (nB % 4 == 0) && (((uintptr_t)bounds_out & 15) == 0);
    hipLaunchKernelGGL(k_share_scatter, dim3((unsigned)share_grid(N)), dim3(256), 0, st, a);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_HIP;
}
