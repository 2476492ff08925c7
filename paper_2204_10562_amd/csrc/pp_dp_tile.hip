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
// one max and half a three-operand min, plus a DPP min over the 8 lanes that share a cell
// (2 operations per tile) and 2 operations per split to build g.  The rows of the current
// candidate live in LDS, one private slice per wave, so there are no barriers.  The single
// cell of the last row that is needed is worked out at the end of row S-2, from registers.
//
// Row n of a candidate depends only on the first n+1 devices of its ordering.  A wave walks
// a contiguous chunk of candidates and recomputes only the rows from the first position in
// which the ordering differs from the previous candidate's; with all D! orderings in
// lexicographic order most rows are shared.
//
// Reading a plan back is a chain of S-1 dependent lookups, far longer than the arithmetic of
// a candidate that recomputes one or two rows.  So every computed row also leaves its split
// indices (one byte per cell) in an arena in LDS, every finished candidate records which
// arena rows make up its path, and the plans of up to 64 finished candidates are read back
// together, one candidate per lane.
#include "pp_common.h"
#include "pp_dp_flat.h"
#include "pp_dp_tile.h"

#define DPP_QUAD_XOR1 0xB1     // quad_perm:[1,0,3,2]
#define DPP_QUAD_XOR2 0x4E     // quad_perm:[2,3,0,1]
#define DPP_HALF_MIRROR 0x141  // row_half_mirror: lane b <-> 7-b within each 8 lanes
#define DPP_ROW_ROR8 0x128     // row_ror:8: lane <-> lane + 8 within each 16 lanes

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

// Min over the 8 lanes that share a = lane/8 for NT values at once.  The first step pairs
// lane b with lane 7-b and lets the lanes b < 4 reduce value i and the lanes b >= 4 value
// i + H (H = ceil(NT/2)) into the same register, so the two remaining steps run on half as
// many registers.  Afterwards v[i], i < H, holds the minimum of value i on lanes b < 4 and of
// value i + H (if there is one) on lanes b >= 4.
// The compiler does not see that the statements below are DPP operations, so the wait states
// DPP needs after a write of its source register are given explicitly: the empty statements
// pin every producer before the first s_nop, and every step is separated from the next.
template <int NT>
__device__ __forceinline__ void min_over_b_halves(int (&v)[NT]) {
    constexpr int H = (NT + 1) / 2;
#pragma unroll
    for (int i = 0; i < NT; ++i) asm volatile("" : "+v"(v[i]));
    asm volatile("s_nop 1");
#pragma unroll
    for (int i = 0; i < H; ++i) {
        asm volatile("v_min_i32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0x5"
                     : "+v"(v[i]));
        if (i + H < NT)
            asm volatile("v_min_i32_dpp %0, %1, %1 row_half_mirror row_mask:0xf bank_mask:0xa"
                         : "+v"(v[i])
                         : "v"(v[i + H]));
    }
    asm volatile("s_nop 1");
#pragma unroll
    for (int i = 0; i < H; ++i)
        asm volatile("v_min_i32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf"
                     : "+v"(v[i]));
    asm volatile("s_nop 1");
#pragma unroll
    for (int i = 0; i < H; ++i)
        asm volatile("v_min_i32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf"
                     : "+v"(v[i]));
    asm volatile("s_nop 1");
#pragma unroll
    for (int i = 0; i < H; ++i) asm volatile("" : "+v"(v[i]));
}

__device__ __forceinline__ void lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <int NT>
__global__ __launch_bounds__(256) void k_dp_tile(dp_tile_args a) {
    extern __shared__ __align__(16) unsigned char smem[];
    if (pp_is_flat(a.g.hdr)) {
        // no channel time depends on the cut position: closed form, here or in the makespan kernel
        if (!dp_flat_deferred(a.g)) dp_flat_body(a.g, smem, a.g.lds_bytes);
        return;
    }
    if (!(pp_vmax(a.g.hdr) < a.g.fit_limit)) {
        dp_generic_body<true>(a.g, smem);  // times too large for 32-bit keys
        return;
    }

    constexpr int RS = 8 * NT + 4;  // key row stride in dwords: index k (0 = infinite) .. 8NT
    constexpr int RB = 8 * NT + 4;  // arena row stride in bytes: split index of cell l at [l]
    const int lane = threadIdx.x & 63;
    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int la = lane >> 3, lb = lane & 7;
    const int S = a.S, K = a.K, L = a.L, D = a.D;
    const int kmask = (1 << K) - 1;
    unsigned char *mine = smem + (size_t)wib * pp_dp_tile_lds_per_wave(S, NT);
    int *rows = (int *)mine;
    unsigned char *arena = mine + (size_t)S * RS * 4;
    unsigned char *slots = arena + (size_t)DPT_ARENA_ROWS * RB;  // [pending][S] arena row of row n
    int *tops = (int *)(slots + (size_t)DPT_PENDING * S);        // [pending][S] key of cell (n, L)
    const bool stages = a.g.stages != 0;
    const int tri = S * (S + 1) / 2;
    long long *C_out = a.g.C_out;
    int *bounds_out = a.g.bounds_out;
    const int *ord = a.g.ord;

    const long long wave = (long long)blockIdx.x * (blockDim.x >> 6) + wib;
    const long long c0 = wave * a.chunk;
    const long long c1 = c0 + a.chunk < a.N ? c0 + a.chunk : a.N;
    if (c0 >= c1) return;

    // candidate-independent part: Dp[i][j] = ((P[l] - P[k]) << K) | k, or infinite if k >= l
    int Dp[NT * (NT + 1) / 2];
    int Pl[NT], Pk[NT];
    {
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            Pl[i] = a.g.p32[8 * i + la + 1] << K;
            Pk[i] = (a.g.p32[8 * i + lb] << K) - (8 * i + lb);
        }
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
            for (int j = 0; j <= i; ++j) {
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
        lds_sync();
    }

    // FUSE: cell (S-1, L), the only cell of the last row that is needed, is computed at the
    // end of row S-2 from that row's cells while they are still in registers: after the
    // reduction a lane holds the cells l = 8 (h H + r) + a + 1 (h = b / 4, r = 0..H-1), and
    // DL[r] = ((P[L] - P[l]) << K) | l (infinite for l >= L) is the difference key of cell L
    // against the split after l layers.
    constexpr bool FUSE = true;
    constexpr int HC = (NT + 1) / 2;
    int DL[FUSE ? HC : 1];
    if (FUSE) {
        const int plk = a.g.p32[L];
#pragma unroll
        for (int r = 0; r < HC; ++r) {
            const int tile = (lb >> 2) * HC + r, l = 8 * tile + la + 1;
            int d = ((plk - a.g.p32[l]) << K) | l;
            d = (tile < NT && l < L) ? d : PP_INF32;
            asm volatile("" : "+v"(d));
            DL[r] = d;
        }
    }

    // the difference key of block (i, j)
    auto dkey = [&](int i, int j) __attribute__((always_inline)) -> int {
        return Dp[i * (i + 1) / 2 + j];
    };
    const unsigned long long smask = S >= 64 ? ~0ull : ((1ull << S) - 1);
    const int top_lane = ((L - 1) & 7) * 8;  // a lane that owns cell L (in tile NT-1)
    constexpr int H = (NT + 1) / 2;
    // where this lane stores the cells it holds after a row's reduction (b = 0 or 4 only)
    const int wofs = la + 1 + (lb >> 2) * 8 * H;

    // finished candidates pend0 .. pend0+pending-1 wait for their plans to be written out;
    // lane q keeps the key of cell (S-1, L) of pending candidate q (-1: its ordering was bad)
    long long pend0 = c0;
    int pending = 0, v_top = 0;
    unsigned long long pairs = 0, nrows = 0;  // work done by this wave
    int arena_used = 0;
    bool fresh = true;  // the arena was emptied: the next candidate must recompute every row
    int v_cur = 0;  // lane n: arena row holding the split indices of row n of the current path
    // lane n: key of cell (n, L) of the current path, i.e. the result for n+1 stages
    int v_tops = __builtin_amdgcn_readlane(Pl[NT - 1], top_lane);

    // Writes out C and the plans of all pending candidates, one per lane.
    auto flush = [&]() {
        lds_sync();
        const bool live = lane < pending;
        const long long cq = pend0 + lane;
        const bool bad = live && v_top < 0;
        if (__ballot(bad) && lane == 0) pp_raise(a.g.status, PP_FAULT_ORDERING);
        // xi = number of stages of the plan read back: S only, or every count 1..S
        for (int xi = stages ? 1 : S; xi <= S; ++xi) {
            int top = v_top;
            if (xi < S && live && !bad) top = tops[lane * S + xi - 1];
            const long long cat = stages ? cq * S + xi - 1 : cq;
            if (live) C_out[cat] = bad ? PP_INF64 : (long long)(top >> K);
            int *bo = bounds_out + (stages ? cq * tri + xi * (xi - 1) / 2 : cq * S);
            int e = L;
            for (int n = xi - 1; n >= 0; --n) {
                if (live) bo[n] = bad ? 0 : e;
                if (n == 0) break;
                // split index stored with cell (n, e): the key itself for the plan's last row
                int nxt = top & kmask;
                if (n < xi - 1 && live && !bad) nxt = arena[(int)slots[lane * S + n] * RB + e] & kmask;
                e = (live && !bad) ? nxt : 0;
            }
        }
        pend0 += pending;
        pending = 0;
        arena_used = 0;
        fresh = true;
    };

    if (S == 1) {
        // a single stage: nothing to compute, C = P[L]
        const int key = rows[L];
        for (long long c = c0; c < c1; ++c) {
            int d = lane == 0 ? ord[c] : 0;
            const bool bad = a.validate && (d < 0 || d >= D);
            if (lane == pending) v_top = __builtin_amdgcn_readfirstlane(bad) ? -1 : key;
            if (++pending == DPT_PENDING) flush();
        }
        if (pending) flush();
        return;
    }

    // Lane n carries device o[n] of the candidate (v_o) and the link index o[n-1]*D + o[n]
    // that row n needs (v_link).
    int v_prev = 0;
    bool have_prev = false;
    int v_o = lane < S ? ord[c0 * S + lane] : 0;

    // Looks at candidate ordering v (previous valid one in v_prev): returns the first row to
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
        // rows below p are reused, so their split indices must still be in the arena
        p = (p > 1 && !fresh) ? p : 1;
        return p < S - 1 ? p : S - 1;  // the last row is always recomputed
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

    // prio_until[k]: the last candidate with more than prio_left[k] candidates still to do
    // (itself included)
    long long prio_until[3];
    for (int k = 0; k < 3; ++k) prio_until[k] = c1 - 1 - a.prio_left[k];

    // first candidate of the chunk (bad ones are recorded and skipped)
    long long c = c0;
    int first = inspect(v_o);
    while (first < 0) {
        if (lane == pending) v_top = -1;
        if (++pending == DPT_PENDING) flush();
        if (++c >= c1) break;
        v_o = lane < S ? ord[c * S + lane] : 0;
        first = inspect(v_o);
    }
    if (c >= c1) {
        if (pending) flush();
        return;
    }
    int v_link = links(v_o);
    int xk[NT];
    fetch_x(xk, __builtin_amdgcn_readlane(v_link, first));

    for (;;) {
        // c is a valid candidate whose rows first..S-1 are to be computed; xk holds (or is
        // about to receive) the channel keys of row `first`
        fresh = false;
        // Of the waves that share a SIMD the one with more of its chunk still to do issues
        // first, so that they finish together and none runs alone at the end (levels from
        // thresholds worked out once: a division here costs as much as a tenth of a row).
        if (c <= prio_until[2]) __builtin_amdgcn_s_setprio(3);
        else if (c <= prio_until[1]) __builtin_amdgcn_s_setprio(2);
        else if (c <= prio_until[0]) __builtin_amdgcn_s_setprio(1);
        else __builtin_amdgcn_s_setprio(0);
        const bool more = c + 1 < c1;
        int v_on = (more && lane < S) ? ord[(c + 1) * S + lane] : 0;
        int first_n = -2, v_link_n = 0;  // next candidate: -2 none, -1 bad ordering
        bool flush_after = false;

        // candidate finished with key `top` in cell (S-1, L): remember it and the arena rows of
        // its path
        auto finish_candidate = [&](int top) __attribute__((always_inline)) {
            if (lane == pending) v_top = top;
            if (lane < S) slots[pending * S + lane] = (unsigned char)v_cur;
            if (stages && lane < S) tops[pending * S + lane] = v_tops;
            ++pending;
        };

        // One DP row.  xc holds this row's channel keys; the keys of the row computed next are
        // fetched into xf while this one is computed.  After the candidate's last row that is
        // the first row of the next candidate (looked at here), or, if there is none, this
        // row's keys once more.
        auto row = [&](int n, int (&xc)[NT], int (&xf)[NT]) __attribute__((always_inline)) {
            int next_link = __builtin_amdgcn_readlane(v_link, n + 1 < S ? n + 1 : n);
            // the candidate ends with this row: the last row itself, or row S-2 with cell
            // (S-1, L) worked out at its end
            const bool fused = FUSE && n == S - 2;
            int xl[HC];
            if (fused) {
                const int *xp = a.xct + ((size_t)next_link * 16 + (la * 2 + (lb >> 2))) * HC;
#pragma unroll
                for (int r = 0; r < HC; ++r) xl[r] = xp[r];
            }
            if ((n == S - 1 || fused) && more) {
                v_prev = v_o;
                have_prev = true;
                first_n = inspect(v_on);
                if (first_n >= 0) {
                    // rows first_n..S-2 need arena rows (and so does this row, if it is row
                    // S-2); one more pending candidate needs a lane
                    if (arena_used + (fused ? 1 : 0) + (S - 1 - first_n) > DPT_ARENA_ROWS ||
                        pending + 2 > DPT_PENDING) {
                        flush_after = true;
                        first_n = 1;
                    }
                    v_link_n = links(v_on);
                    next_link = __builtin_amdgcn_readlane(v_link_n, first_n);
                }
            }
            fetch_x(xf, next_link);

            int *nrow = rows + n * RS;
            // the previous row is read through an index of its own, so that the NT reads are
            // one address and NT immediate offsets (seen as nrow minus a constant the offsets
            // would be negative, which the instruction cannot hold)
            int pidx = (n - 1) * RS + lb;
            asm volatile("" : "+v"(pidx));
            int g[NT];
#pragma unroll
            for (int j = 0; j < NT; ++j) g[j] = rows[pidx + 8 * j];
#pragma unroll
            for (int j = 0; j < NT; ++j) asm volatile("" : "+v"(g[j]));  // all reads in flight at once
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                // previous row's time with this split's index (the low bits of the channel
                // key) in the low bits, then the larger of that and the channel key
                int wk;
                asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(wk) : "s"(kmask), "v"(xc[j]), "v"(g[j]));
                g[j] = imax(wk, xc[j]);
            }
            if (n < S - 1) {
                int acc[NT];
#pragma unroll
                for (int i = 0; i < NT; ++i) {
                    int v = PP_INF32;
#pragma unroll
                    for (int j = 0; j <= i; ++j) v = imin(v, imax(g[j], dkey(i, j)));
                    acc[i] = v;
                }
                min_over_b_halves<NT>(acc);
                pairs += (unsigned long long)((L - n) * (L - n + 1) / 2);
                ++nrows;
                const int slot = arena_used++;
                const int top_n = NT == 1 ? __builtin_amdgcn_readlane(acc[0], top_lane)
                                          : __builtin_amdgcn_readlane(acc[NT - 1 - H], top_lane + 4);
                if (lane == n) { v_cur = slot; v_tops = top_n; }
                unsigned char *arow = arena + slot * RB;
                // lanes b = 0 hold tiles 0..H-1, lanes b = 4 tiles H..NT-1 (one fewer if NT is odd)
                if ((lb & 3) == 0) {
                    // keys first, then bytes: stores of one kind in a row can be paired
#pragma unroll
                    for (int i = 0; i < H; ++i)
                        if (i + H < NT || lb == 0) nrow[8 * i + wofs] = acc[i];
                    // low byte of the key: the split index in its low K <= 7 bits
#pragma unroll
                    for (int i = 0; i < H; ++i)
                        if (i + H < NT || lb == 0) arow[8 * i + wofs] = (unsigned char)acc[i];
                }
                if (fused) {
                    int m = PP_INF32;
#pragma unroll
                    for (int r = 0; r < HC; ++r) {
                        int wk;
                        asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(wk) : "s"(kmask), "v"(xl[r]), "v"(acc[r]));
                        m = imin(m, imax(imax(wk, xl[r]), DL[r]));
                    }
                    m = dpp_min<DPP_HALF_MIRROR>(m);  // the two halves of the row
                    m = dpp_min<DPP_ROW_ROR8>(m);     // a and a + 1
                    const int top = imin(imin(__builtin_amdgcn_readlane(m, 0), __builtin_amdgcn_readlane(m, 16)),
                                         imin(__builtin_amdgcn_readlane(m, 32), __builtin_amdgcn_readlane(m, 48)));
                    pairs += (unsigned long long)(L - (S - 1));
                    ++nrows;
                    finish_candidate(top);
                }
                lds_sync();
            } else {
                // only W[S-1][L] is needed of the last row; L lies in tile NT-1
                constexpr int i = NT - 1;
                int v = PP_INF32;
#pragma unroll
                for (int j = 0; j <= i; ++j) v = imin(v, imax(g[j], dkey(i, j)));
                v = min_over_b(v);
                pairs += (unsigned long long)(L - n);
                ++nrows;
                finish_candidate(__builtin_amdgcn_readlane(v, top_lane));
            }
        };
        // rows alternate between the two key buffers, so that no row has to copy them; only a
        // candidate with an odd number of rows moves the last fetch into xk once
        int xn[NT];
        // (with FUSE the last row is a row of its own only when no other row is computed)
        const int end = (FUSE && first <= S - 2) ? S - 1 : S;
        for (int n = first;;) {
            row(n, xk, xn);
            if (++n >= end) {
#pragma unroll
                for (int j = 0; j < NT; ++j) xk[j] = xn[j];
                break;
            }
            row(n, xn, xk);
            if (++n >= end) break;
        }

        if (flush_after) flush();
        // bad orderings after this candidate are recorded and skipped
        while (first_n == -1) {
            if (lane == pending) v_top = -1;
            if (++pending == DPT_PENDING) flush();
            ++c;
            first_n = -2;
            if (c + 1 < c1) {
                v_on = lane < S ? ord[(c + 1) * S + lane] : 0;
                first_n = inspect(v_on);  // compared with the last valid candidate
                if (first_n >= 0) {
                    if (arena_used + (S - 1 - first_n) > DPT_ARENA_ROWS || pending + 2 > DPT_PENDING) {
                        flush();
                        first_n = 1;
                    }
                    v_link_n = links(v_on);
                    fetch_x(xk, __builtin_amdgcn_readlane(v_link_n, first_n));
                }
            }
        }
        if (first_n < 0) break;  // no candidate left
        ++c;
        v_o = v_on;
        v_link = v_link_n;
        first = first_n;
    }
    if (pending) flush();
    if (lane == 0) pp_count_work(a.g.hdr, pairs, nrows, (unsigned)wave);
}

template <int NT>
static int launch_nt(const dp_tile_args &a, int grid, int wpb, size_t lds, hipStream_t st) {
    hipLaunchKernelGGL(k_dp_tile<NT>, dim3(grid), dim3(64 * wpb), lds, st, a);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_HIP;
}

int pp_launch_dp_tile(const dp_tile_args &a, int nt, int grid, int wpb, hipStream_t st) {
    size_t lds = (size_t)wpb * pp_dp_tile_lds_per_wave(a.S, nt);
    const size_t generic = (size_t)3 * (a.L + 1) * 8;  // the int64 fallback's rows
    if (lds < generic) lds = generic;
    const size_t flat = pp_flat_lds_wanted(a.L, a.D, a.S, wpb);  // the closed-form body's tables
    if (lds < flat) lds = flat;
    dp_tile_args b = a;
    b.g.lds_bytes = lds;
    switch (nt) {
#define CASE(n) case n: return launch_nt<n>(b, grid, wpb, lds, st);
        CASE(1) CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7) CASE(8)
        CASE(9) CASE(10) CASE(11) CASE(12) CASE(13) CASE(14) CASE(15) CASE(16)
#undef CASE
    }
    return PP_ERR_INVALID_ARG;
}
