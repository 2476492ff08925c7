// Partition DP for 128 < L <= 2048 with 32-bit keys: one wavefront per candidate, the cells of
// a row in super-rows of 128, the (cell, split) plane in blocks of 32 x 32 that the 64 lanes
// cover as 4 x 4 tiles of 8 x 8.
//
// Recursion for W(l, xi, r, i) of Sec. IV-B / the PRM listing with one replica per stage:
//   W[n][l] = min_{n<=k<l} max(g_n[k], P[l] - P[k]),   g_n[k] = max(W[n-1][k], X_n[k]).
//
// Same key representation and lane layout as the kernel for L <= 128 (lane (a, b) owns cells
// 128I + 8i + a + 1 and splits 128J + 8j + b; a cell is (time << K) | k, so max keeps the
// split index and min returns the smallest time with the lowest split), but the difference
// term ((P[l] - P[k]) << K) | k is too large to keep in registers for the whole plane, so it
// is formed on the fly: subtract, max and half a three-operand min per pair.  The cells are
// taken in groups of 32 (four tiles); a group visits the blocks of 32 splits on or below the
// diagonal, from the diagonal leftwards, and stops as soon as the difference term alone rules
// out everything further left for its cells; the last super-row has NTL <= 16 cell tiles,
// fixed at compile time, so a model of 300 layers does not pay for 384.
//
// Per wave in LDS: two rows of keys (the row being read, rewritten in place as g, and the row
// being produced).  Split indices go to a per-wave table in global memory while the next row's
// g is built (one coalesced pass), and the plan is read back from there with cache-bypassing
// loads.  Waves are persistent and walk candidates wave, wave + nwaves, ...; where groups of
// candidates are the same problem (pp_share.hip) a wave instead takes a run of consecutive
// entries of the sorted list of representatives, keeps every row it computes in the workspace
// and starts each representative at the first row its predecessor does not share.
#include "pp_common.h"
#include "pp_dp_flat.h"
#include "pp_dp_generic.h"

#define DPP_QUAD_XOR1 0xB1     // quad_perm:[1,0,3,2]
#define DPP_QUAD_XOR2 0x4E     // quad_perm:[2,3,0,1]
#define DPP_HALF_MIRROR 0x141  // row_half_mirror: lane b <-> 7-b within each 8 lanes

struct dp_big_args {
    int NI;      // super-rows: ceil(L / 128)
    int waves;   // working waves (each owns one backtrack table)
    size_t arg_stride;  // entries of one wave's backtrack table: S * Lp
    // non-NULL: if the workspace header says so, walk this list of representatives (one per
    // group of candidates with the same DP, see pp_share.hip) instead of all candidates: every
    // wave a run of neighbours, which share their first links and so their first rows (keys:
    // the key of every candidate; rows: room for row_slots saved rows of Lp + 4 keys)
    const int *reps, *keys, *start;
    int *rows;
    long long row_slots;  // rows of Lp + 4 keys the area `rows` holds
    dp_args g;
};

__device__ __forceinline__ int bmin(int a, int b) { return a < b ? a : b; }
__device__ __forceinline__ int bmax(int a, int b) { return a > b ? a : b; }

template <int CTRL>
__device__ __forceinline__ int big_dpp_min(int v) {
    int o = __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, true);
    return bmin(v, o);
}

__device__ __forceinline__ int big_min_over_b(int v) {
    v = big_dpp_min<DPP_QUAD_XOR1>(v);
    v = big_dpp_min<DPP_QUAD_XOR2>(v);
    v = big_dpp_min<DPP_HALF_MIRROR>(v);
    return v;
}

__device__ __forceinline__ void big_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// The g row and the table (P[k] << K) - k at the 4 split tiles of one block, as lane (a, b)
// needs them: splits 8 j + b.
struct big_splits {
    int g[4], pk[4];
};

__device__ __forceinline__ void big_load(big_splits &s, const int *G, const int *Pk, int lb) {
#pragma unroll
    for (int j = 0; j < 4; ++j) { s.g[j] = G[8 * j + lb]; s.pk[j] = Pk[8 * j + lb]; }
}

// One block: NI4 (<= 4) cell tiles against 4 split tiles.  DIAG: the split tiles are the cell
// tiles' own: tiles above the diagonal are skipped, those on it are valid for lanes with b <= a.
template <int NI4, bool DIAG>
__device__ __forceinline__ void big_block(int (&acc)[4], const int (&Pl)[4], const big_splits &s,
                                          int la, int lb) {
#pragma unroll
    for (int i = 0; i < NI4; ++i) {
        int v = acc[i];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (DIAG && j > i) continue;
            int d = Pl[i] - s.pk[j];
            if (DIAG && j == i) d = lb <= la ? d : PP_INF32;
            v = bmin(v, bmax(s.g[j], d));
        }
        acc[i] = v;
    }
}

// (cell, split) pairs with cell in [a, b], split in [klo, cell - 1] (at most L^2 / 2 < 2^22)
__device__ __forceinline__ unsigned big_pairs(int a, int b, int klo) {
    if (a <= klo) a = klo + 1;
    if (b < a) return 0;
    const unsigned lo = (unsigned)(a - klo), hi = (unsigned)(b - klo);
    return (lo + hi) * (hi - lo + 1) / 2;
}

// A group of NI4 cell tiles (cells c0+1 .. c0+8 NI4, c0 a multiple of 32) of row n: the block on
// the diagonal, then the blocks of 32 splits to its left from the nearest on, then the
// reduction over the 8 lanes that share a cell, then the cells go to the next row.
// P[l] - P[k] grows as k falls, so once the smallest difference of the next block (first cell
// of the group against the block's last split) exceeds every value a lane still holds for a
// cell of the group, neither that block nor any further left can lower or tie one of them:
// the scan stops there.  The test costs a scalar subtraction, two maxima and one compare:
// pend holds (P[32 s + 31] << K) in lane s.  Returns the pairs evaluated (for the work counter).
template <int NI4>
__device__ __forceinline__ unsigned big_cell_group(int c0, int n, int L, const int *G,
                                                             const int *sPk, int *nxt, int la,
                                                             int lb, int pend) {
    int acc[4], Pl[4];
#pragma unroll
    for (int i = 0; i < NI4; ++i) {
        const int l = c0 + 8 * i + la + 1;
        Pl[i] = sPk[l] + l;  // P[l] << K
        acc[i] = PP_INF32;
    }
    big_splits s;
    big_load(s, G + c0, sPk + c0, lb);
    big_block<NI4, true>(acc, Pl, s, la, lb);
    const int first = __builtin_amdgcn_readlane(Pl[0], 0);  // lane 0 holds cell c0 + 1
    const int sg_lo = n >> 5;  // blocks wholly below split n hold nothing feasible
    int sg = (c0 >> 5) - 1;
    for (; sg >= sg_lo; --sg) {
        // ((P[c0 + 1] - P[32 sg + 31]) << K) is the smallest difference key of block sg: it can
        // still lower or tie a cell of the group only if some lane holds a key that is not below it
        // (fetching the next block's splits ahead of this test was measured: no gain)
        const int dkey = first - __builtin_amdgcn_readlane(pend, sg);
        int m = acc[0];
#pragma unroll
        for (int i = 1; i < NI4; ++i) m = bmax(m, acc[i]);
        if (!__ballot(m >= dkey)) break;
        big_load(s, G + 32 * sg, sPk + 32 * sg, lb);
        big_block<NI4, false>(acc, Pl, s, la, lb);
    }
#pragma unroll
    for (int i = 0; i < NI4; ++i) {
        acc[i] = big_min_over_b(acc[i]);
        asm volatile("" : "+v"(acc[i]));
    }
    if (lb == 0) {
#pragma unroll
        for (int i = 0; i < NI4; ++i) nxt[c0 + 8 * i + la + 1] = acc[i];
    }
    const int a0 = c0 + 1 > n + 1 ? c0 + 1 : n + 1, b0 = c0 + 8 * NI4 < L ? c0 + 8 * NI4 : L;
    const int klo = 32 * (sg + 1) > n ? 32 * (sg + 1) : n;
    return big_pairs(a0, b0, klo);
}

// One super-row of NTI cell tiles of row n, in groups of four.
template <int NTI>
__device__ __forceinline__ unsigned big_super_row(int I, int n, int L, const int *G,
                                                            const int *sPk, int *nxt, int la,
                                                            int lb, int pend) {
    unsigned pairs = 0;
    constexpr int REST = (NTI & 3) ? (NTI & 3) : 4;
#pragma unroll
    for (int cg = 0; cg < (NTI + 3) / 4; ++cg) {
        const int c0 = 128 * I + 32 * cg;
        if (NTI - 4 * cg >= 4) pairs += big_cell_group<4>(c0, n, L, G, sPk, nxt, la, lb, pend);
        else pairs += big_cell_group<REST>(c0, n, L, G, sPk, nxt, la, lb, pend);
    }
    return pairs;
}

template <int NTL>
__global__ __launch_bounds__(256) void k_dp_big(dp_big_args b) {
    extern __shared__ __align__(16) unsigned char smem[];
    const dp_args &a = b.g;
    if (pp_is_flat(a.hdr)) {
        // no channel time depends on the cut position: closed form, here or in the makespan kernel
        if (!dp_flat_deferred(a)) dp_flat_body(a, smem, a.lds_bytes);
        return;
    }
    if (!(pp_vmax(a.hdr) < a.fit_limit)) {
        dp_generic_body<true>(a, smem);  // times too large for 32-bit keys
        return;
    }
    const int lane = threadIdx.x & 63;
    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wpb = blockDim.x >> 6;
    const int la = lane >> 3, lb = lane & 7;
    const int S = a.S, K = a.K, L = a.L, D = a.D, NI = b.NI;
    const int Lp = 128 * NI, RS = Lp + 4;
    const int kmask = (1 << K) - 1;
    int *sPk = (int *)smem;                       // (P[k] << K) - k, k = 0..Lp (P padded with P[L])
    int *bufA = sPk + RS + (size_t)wib * 2 * RS;  // this wave's two rows
    int *bufB = bufA + RS;
    const long long wave = (long long)blockIdx.x * wpb + wib;

    for (int k = threadIdx.x; k <= Lp; k += blockDim.x) sPk[k] = (a.p32[k < L ? k : L] << K) - k;
    __syncthreads();
    if (wave >= b.waves) return;
    // lane s: (P[32 s + 31] << K), the last split of block s (for the early exit's test)
    const int pend = 32 * lane + 31 <= Lp ? sPk[32 * lane + 31] + 32 * lane + 31 : 0;
    unsigned short *arg = a.arg + (size_t)wave * b.arg_stride;
    unsigned long long pairs = 0, nrows = 0;
    const int tri = S * (S + 1) / 2;

    // Which candidates this wave takes: every waves-th one, or a run of consecutive entries of a
    // list the preparation left (pp_share.hip): the sorted representatives where candidates
    // share their DP, or all candidates sorted by their first devices.  Neighbours in a list
    // share their first rows; the wave keeps the rows that can be shared (all of them, or the
    // first kdev - 1) in its slice of the workspace.
    const bool listed = b.reps != NULL && a.hdr->share_active != 0;
    const bool sorted = b.reps != NULL && !listed && a.hdr->share_sorted != 0;
    // main part: entries r_begin, r_begin + r_step, ... (n_main of them); then, where candidates
    // share their DP, this wave's share of the candidates with a bad ordering that follow the
    // sorted representatives in the list (n_tail entries t_begin, t_begin + waves, ...)
    long long r_begin = wave, r_step = b.waves, nsorted = 0, t_begin = 0, n_tail = 0;
    long long n_main = wave < a.N ? (a.N - wave + b.waves - 1) / b.waves : 0;
    unsigned pw = 1;  // lane n = 1..S-1: (classes)^(S-1-n), the weight of the key's digit n
    int keep_rows = 0;  // rows 1..keep_rows are saved
    if (listed) {
        // runs of about equal work, cut by the preparation
        const long long total = a.hdr->share_nreps, nch = a.hdr->share_nchunks;
        nsorted = a.hdr->share_nsorted;
        keep_rows = S - 2 > 0 ? S - 2 : 0;
        r_begin = wave < nch ? b.start[wave] : 0;
        n_main = wave < nch ? b.start[wave + 1] - r_begin : 0;
        r_step = 1;
        t_begin = nsorted + wave;
        n_tail = t_begin < total ? (total - t_begin + b.waves - 1) / b.waves : 0;
        const unsigned nc = a.hdr->share_nc;
        for (int n = lane + 1; n < S; ++n) pw *= nc;
    } else if (sorted) {
        nsorted = a.N;
        keep_rows = (int)a.hdr->share_kdev - 1;
        keep_rows = keep_rows < S - 2 ? keep_rows : S - 2;
        keep_rows = keep_rows > 0 ? keep_rows : 0;
        long long nw = b.row_slots / (keep_rows > 0 ? keep_rows : 1);  // waves whose rows fit the area
        nw = nw < b.waves ? nw : b.waves;
        nw = nw > 1 ? nw : 1;
        const long long chunk = (a.N + nw - 1) / nw;
        r_begin = wave * chunk;
        n_main = r_begin < a.N ? (r_begin + chunk < a.N ? chunk : a.N - r_begin) : 0;
        r_step = 1;
    }
    const long long n_items = n_main + n_tail;
    auto entry = [&](long long i) { return i < n_main ? r_begin + i * r_step : t_begin + (i - n_main) * b.waves; };
    // (row n >= 1 of this wave's slice at save + (n - 1) RS)
    int *save = b.rows + (size_t)((listed || sorted) && n_main ? wave : 0) * keep_rows * RS;
    int prev_key = -1, prev_o = -1;
    int v_tops = 0;  // lane n keeps W[n][L] (with its split index) for the stage-count search
    int *cur = bufA, *nxt = bufB;
    // A candidate's index, key and devices come from memory through a chain of loads (list
    // entry, then key and ordering): they are fetched one candidate ahead.
    auto fetch = [&](long long i, long long &c, int &key, int &v_o) {
        c = 0; key = -1; v_o = 0;
        if (i >= n_items) return;
        const long long r = entry(i);
        c = (listed || sorted) ? pp_share_at(a.hdr, b.reps, a.N, r) : r;
        if (listed && r < nsorted) key = b.keys[c];
        v_o = lane < S ? a.ord[c * S + lane] : 0;
    };
    long long c_next;
    int key_next, v_o_next;
    fetch(0, c_next, key_next, v_o_next);
    for (long long i = 0; i < n_items; ++i) {
        const long long r = entry(i);
        const long long c = c_next;
        const int v_o = v_o_next;
        // rows 1..p of the previous candidate are this one's too: its key has the same first p
        // digits (equal links give equal rows), or its first p + 1 devices are the same
        int p = 0;
        const int key = key_next;
        fetch(i + 1, c_next, key_next, v_o_next);
        if (listed && r < nsorted) {
            if (prev_key >= 0) {
                const bool differ = lane >= 1 && lane < S && (unsigned)key / pw != (unsigned)prev_key / pw;
                const unsigned long long m = __ballot(differ);
                p = m ? __builtin_ctzll(m) - 1 : S - 2;
                p = p < S - 2 ? p : S - 2;
                p = p > 0 ? p : 0;
            }
        }
        prev_key = key;
        // ordering: lane n holds device o[n]
        bool bad = false;
        if (a.validate) {
            bad = lane < S && (v_o < 0 || v_o >= D);
            for (int q = 0; q + 1 < S; ++q) {
                int oq = __builtin_amdgcn_readlane(v_o, q);
                bad |= (lane > q && lane < S && oq == v_o);
            }
        }
        if (__ballot(bad)) {
            if (lane == 0) pp_raise(a.status, PP_FAULT_ORDERING);
            if (a.stages) {
                if (lane < S) a.C_out[c * S + lane] = PP_INF64;
                for (int n = lane; n < tri; n += 64) a.bounds_out[c * tri + n] = 0;
            } else {
                if (lane == 0) a.C_out[c] = PP_INF64;
                if (lane < S) a.bounds_out[c * S + lane] = 0;
            }
            prev_key = -1;  // (the next candidate starts from row 0)
            prev_o = -1;
            continue;
        }
        if (sorted) {
            // (prev_o: the previous candidate's device in this lane, -1 if there is none)
            const unsigned long long m = __ballot(lane < S && v_o != prev_o);
            p = m ? __builtin_ctzll(m) - 1 : S - 2;
            p = p < keep_rows ? p : keep_rows;
            p = p > 0 ? p : 0;
            prev_o = v_o;
        }
        const int v_link = __shfl_up(v_o, 1) * D + v_o;

        int top = 0;
        if (p == 0) {
            // row 0: one stage holding the first l layers
            for (int l = lane; l <= Lp; l += 64) cur[l] = l ? sPk[l] + l : PP_INF32;
            big_lds_sync();
            top = cur[L];  // S == 1: C = P[L]
            v_tops = top;
        } else {
            // row p as this wave left it (stored by other lanes of the wave: wait for the
            // stores, then read past the L1 cache)
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
            const int *from = save + (size_t)(p - 1) * RS;
            for (int l = lane; l <= Lp; l += 64)
                cur[l] = __hip_atomic_load(from + l, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            big_lds_sync();
        }

        for (int n = p + 1; n < S; ++n) {
            const int *xrow = a.x32 + (size_t)__builtin_amdgcn_readlane(v_link, n) * L;
            // Rewrite the previous row in place as g; on the way its split indices (the low
            // key bits) go to the backtrack table.
            unsigned short *arow = arg + (size_t)(n - 1) * Lp;
            // (the link's times are requested eight steps at a time, ahead of the stores they
            // could otherwise not be moved across: one trip per 512 splits instead of eight)
            for (int k0 = lane; k0 < Lp; k0 += 512) {
                int xv[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int k = k0 + 64 * u;
                    xv[u] = (k >= 1 && k < L) ? xrow[k] : 0;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int k = k0 + 64 * u;
                    if (k < Lp) {
                        const int w = cur[k];
                        if (n >= 2) arow[k] = (unsigned short)(w & kmask);
                        int xk = PP_INF32;
                        if (k >= 1 && k < L) xk = (xv[u] << K) | k;
                        int wk = (w & ~kmask) | (xk & kmask);
                        cur[k] = bmax(wk, xk);
                    }
                }
            }
            big_lds_sync();
            if (n < S - 1) {
                for (int I = 0; I < NI; ++I)
                    pairs += I + 1 < NI ? big_super_row<16>(I, n, L, cur, sPk, nxt, la, lb, pend)
                                        : big_super_row<NTL>(I, n, L, cur, sPk, nxt, la, lb, pend);
                if (lane == 0) nxt[0] = PP_INF32;
                big_lds_sync();
                int *t = cur; cur = nxt; nxt = t;
                const int top_n = cur[L];
                if (lane == n) v_tops = top_n;
                if (n <= keep_rows) {
                    // kept for the next candidate of the run
                    int *to = save + (size_t)(n - 1) * RS;
                    for (int l = lane; l <= Lp; l += 64) to[l] = cur[l];
                }
            } else {
                // only W[S-1][L] is needed of the last row
                const int PL = sPk[L] + L;
                int v = PP_INF32;
                for (int k = lane; k < L; k += 64) v = bmin(v, bmax(cur[k], PL - sPk[k]));
                for (int off = 32; off; off >>= 1) v = bmin(v, __shfl_xor(v, off));
                top = v;
                if (lane == n) v_tops = v;
                pairs += (unsigned long long)(L - n);
            }
            ++nrows;
        }

        // plan: every lane follows the same chain through the backtrack table, lane n keeps
        // bound n.  The table was written by other lanes of this wave: wait for the stores,
        // then read past the L1 cache (which may hold lines of an earlier candidate).
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
        if (a.stages) {
            // lane xi-1 follows its own chain from (xi-1, L): the plan with xi stages
            if (lane < S) {
                a.C_out[c * S + lane] = (long long)(v_tops >> K);
                int *bo = a.bounds_out + c * tri + lane * (lane + 1) / 2;
                int e = L;
                for (int m = lane; m >= 1; --m) {
                    bo[m] = e;
                    if (m == lane) {
                        e = v_tops & kmask;
                        e = e < Lp ? e : Lp - 1;  // stays inside the table whatever the data
                    } else {
                        const size_t at = (size_t)m * Lp + e;
                        const unsigned *word = (const unsigned *)(arg + (at & ~(size_t)1));
                        unsigned w2 = __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        e = (int)((at & 1) ? (w2 >> 16) : (w2 & 0xffffu));
                    }
                }
                bo[0] = e;
            }
            continue;
        }
        int e = L, mine = 0;
        for (int m = S - 1; m >= 1; --m) {
            if (lane == m) mine = e;
            if (m == S - 1) {
                e = top & kmask;
            } else {
                const size_t at = (size_t)m * Lp + e;
                const unsigned *word = (const unsigned *)(arg + (at & ~(size_t)1));
                unsigned w2 = __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                e = (int)((at & 1) ? (w2 >> 16) : (w2 & 0xffffu));
            }
        }
        if (lane == 0) { mine = e; a.C_out[c] = (long long)(top >> K); }
        if (lane < S) a.bounds_out[c * S + lane] = mine;
    }
    if (lane == 0) pp_count_work(a.hdr, pairs, nrows, (unsigned)wave);
}

template <int NTL>
static int launch_big(const dp_big_args &b, int grid, int wpb, size_t lds, hipStream_t st) {
    hipLaunchKernelGGL(k_dp_big<NTL>, dim3(grid), dim3(64 * wpb), lds, st, b);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_HIP;
}

// LDS of a workgroup and waves per workgroup for this shape (0 if it does not fit).
static size_t big_lds(int L, int D, int S, int &wpb) {
    const int Lp = 128 * ((L + 127) / 128), RS = Lp + 4;
    wpb = 4;  // waves per workgroup: table + two rows per wave within 64 KiB of LDS
    while (wpb > 1 && (size_t)(1 + 2 * wpb) * RS * 4 > 64 * 1024) wpb >>= 1;
    size_t lds = (size_t)(1 + 2 * wpb) * RS * 4;
    const size_t generic = (size_t)3 * (L + 1) * 8;  // the int64 fallback's rows
    if (lds < generic) lds = generic;
    const size_t flat = pp_flat_lds_wanted(L, D, S, wpb);  // the closed-form body's tables
    if (lds < flat) lds = flat;
    return lds > 64 * 1024 ? 0 : lds;
}

int pp_dp_big_waves(int L, int D, int S, int max_waves, int cus) {
    int wpb;
    const size_t lds = big_lds(L, D, S, wpb);
    if (!lds) return 1;
    // resident waves: 4 per SIMD by registers, and what 160 KiB of LDS per CU allow
    long long per_cu = (long long)(160 * 1024 / lds) * wpb;
    if (per_cu > 16) per_cu = 16;
    if (per_cu < 1) per_cu = 1;
    long long waves = per_cu * cus;
    if (waves > max_waves) waves = max_waves;
    return (int)(waves < 1 ? 1 : waves);
}

int pp_launch_dp_big(const dp_args &g, int max_waves, int cus, const pp_share_list *list,
                     hipStream_t st) {
    dp_big_args b;
    b.g = g;
    b.reps = list ? list->reps : NULL;
    b.keys = list ? list->keys : NULL;
    b.start = list ? list->start : NULL;
    b.rows = list ? list->rows : NULL;
    b.row_slots = list ? list->row_slots : 0;
    b.NI = (g.L + 127) / 128;
    const int Lp = 128 * b.NI, RS = Lp + 4;
    b.arg_stride = (size_t)g.S * Lp;
    const int ntl = (g.L - 128 * (b.NI - 1) + 7) / 8;
    int wpb;
    const size_t lds = big_lds(g.L, g.D, g.S, wpb);
    if (!lds) return PP_ERR_INVALID_ARG;
    b.g.lds_bytes = lds;
    const long long waves = pp_dp_big_waves(g.L, g.D, g.S, max_waves, cus);
    b.waves = (int)waves;
    const int grid = (int)((waves + wpb - 1) / wpb);
    b.g.nblocks = g.nblocks < grid ? g.nblocks : grid;
    switch (ntl) {
#define CASE(n) case n: return launch_big<n>(b, grid, wpb, lds, st);
        CASE(1) CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7) CASE(8)
        CASE(9) CASE(10) CASE(11) CASE(12) CASE(13) CASE(14) CASE(15) CASE(16)
#undef CASE
    }
    return PP_ERR_INVALID_ARG;
}
