// Shared declarations of the GPU library's translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "pp.h"

#define PP_INF64 INT64_MAX
#define PP_INF32 0x7fffffff
#define PP_CAP62 ((long long)1 << 62)

__host__ __device__ static inline size_t pp_align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Number of key bits that hold a split index 0..L-1.
static inline int pp_index_bits(int L) {
    int K = 1;
    while ((1 << K) < L) ++K;
    return K;
}

// Header at the start of the workspace, filled by the pack kernels.
// pmax[b] is the largest per-microbatch time pack block b saw (P[L], or an XF+XB entry of its
// slice); the largest value a DP cell can take is the maximum over all PP_PACK_BLOCKS entries.
#define PP_PACK_BLOCKS 64
struct pp_ws_header {
    unsigned long long pmax[PP_PACK_BLOCKS];  // byte 0
    // byte 512: flat[b] != 0 iff, in pack block b's slice of the tables, the channel time
    // XF + XB of every link is the same at every cut position (all 64 set: it is so everywhere)
    unsigned flat[PP_PACK_BLOCKS];
    // byte 768: candidates that share a partition DP (pp_share.hip).  share_active != 0: the
    // links fall into share_nc classes of equal channel-time rows and the share_tsize =
    // share_nc^(S-1) sequences of classes index a table; share_nreps candidates (one per
    // sequence that occurs, plus every candidate with a bad ordering) stand for all of them.
    unsigned share_active, share_nc, share_tsize, share_nreps;
    // the first share_nsorted entries of the list are the representatives in the order of their
    // keys (first link most significant); the share_nbad candidates with a bad ordering follow,
    // stored from the end of the array backwards (pp_share_at)
    unsigned share_nsorted, share_nbad;
    // share_sorted != 0 (only when share_active == 0): the list holds all N candidates ordered
    // by their first share_kdev devices, so that neighbours share the first share_kdev - 1 rows
    unsigned share_sorted, share_kdev;
    // share_active: the sorted representatives are cut into share_nchunks runs of about equal
    // work (rows to compute); run w is entries start[w] .. start[w + 1] - 1 of the list
    unsigned share_nchunks;
    unsigned pad0[55];
    // byte 1024: work the partition DP actually did in this call, in 64 records of 128 bytes
    // (atomics that hit one cache line are served one after another, so every record has a
    // line of its own): (cell, split) pairs evaluated (rows shared between candidates are
    // counted once) and DP rows computed (the single-cell last row counts too).  Zeroed by
    // the pack kernel; the totals are the sums over the 64 records.
    struct {
        unsigned long long pairs, rows, pad[14];
    } work[64];
};

static_assert(offsetof(pp_ws_header, share_active) == PP_WS_SHARE, "header layout");
static_assert(offsetof(pp_ws_header, work) == PP_WS_WORK, "header layout");

__device__ __forceinline__ void pp_count_work(pp_ws_header *hdr, unsigned long long pairs,
                                              unsigned long long rows, unsigned who) {
    atomicAdd(&hdr->work[who & 63].pairs, pairs);
    atomicAdd(&hdr->work[who & 63].rows, rows);
}

// Workspace carving, identical for pp_partition_dp and pp_best_plan.
struct pp_ws_layout {
    size_t hdr, p32, x32, xkt, xct, bfl, ord, arg, bounds, C, T, part, total;
    // candidates that share a DP (0 = not carved: see pp_share_possible)
    size_t sh_hash, sh_rep, sh_table, sh_keys, sh_reps, sh_cnt, sh_start, sh_rows;
    long long sh_row_slots;  // DP rows (of pp_share_row_stride(L) keys) the area sh_rows holds
    int slots;  // resident workgroups of the generic DP kernel (one backtrack table each)
    int nt;     // 8-cell tiles per row of the register-tiled DP kernel, 0 if L is too large for it
};

#define PP_TILE_MAX_L 128
#define PP_DP_SLOTS 4096
// Sharing of one partition DP between the candidates whose links have the same channel times
// (pp_share.hip): table entries, and the sizes it is built for.
#define PP_SHARE_TABLE (1 << 20)
#define PP_SHARE_MAX_D 64
static inline bool pp_share_possible(int L, int D, int64_t N) {
    return L > PP_TILE_MAX_L && D <= PP_SHARE_MAX_D && N < 0x7fffffff;
}
// Saved DP rows (see pp_dp_big.hip): waves that walk the list, bytes in all, keys per row.
#ifndef PP_SHARE_ROW_WAVES
#define PP_SHARE_ROW_WAVES 2048
#endif
#ifndef PP_SHARE_ROW_BYTES
#define PP_SHARE_ROW_BYTES ((size_t)64 << 20)
#endif
__host__ __device__ static inline int pp_share_row_stride(int L) { return 128 * ((L + 127) / 128) + 4; }
// Entry r of the list of representatives (hdr as the share kernels left it).
__device__ __forceinline__ long long pp_share_at(const pp_ws_header *hdr, const int *reps, long long N,
                                                 long long r) {
    const long long ns = hdr->share_nsorted;
    return r < ns ? reps[r] : reps[N - 1 - (r - ns)];
}

static inline pp_ws_layout pp_layout(int L, int D, int S, int64_t N) {
    pp_ws_layout w;
    size_t off = 0;
    w.hdr = off;    off += pp_align256(sizeof(pp_ws_header));
    w.nt = L <= PP_TILE_MAX_L ? (L + 7) / 8 : 0;
    w.p32 = off;    off += pp_align256((size_t)(L + 17) * 4);  // padded to a whole tile
    w.x32 = off;    off += pp_align256((size_t)D * D * L * 4);
    w.xkt = off;    off += pp_align256((size_t)D * D * 8 * w.nt * 4);
    w.xct = off;    off += pp_align256((size_t)D * D * 16 * ((w.nt + 1) / 2) * 4);
    // channel-free DP table: values [S][L+1] int64, then lowest minimising splits [S][L+1] int32
    w.bfl = off;    off += pp_align256((size_t)S * (L + 1) * 12);
    w.ord = off;    off += pp_align256((size_t)N * S * 4);
    w.slots = (int)(N < PP_DP_SLOTS ? N : PP_DP_SLOTS);
    w.arg = off;    off += pp_align256((size_t)w.slots * S * (L + 128) * 2);  // rows padded to 128 cells
    w.bounds = off; off += pp_align256((size_t)N * S * 4);
    w.C = off;      off += pp_align256((size_t)N * 8);
    w.T = off;      off += pp_align256((size_t)N * 8);
    w.part = off;   off += pp_align256((size_t)((N + 63) / 64) * 16 * PP_MAX_M_LIST);
    w.sh_hash = w.sh_rep = w.sh_table = w.sh_keys = w.sh_reps = w.sh_cnt = w.sh_start = w.sh_rows = 0;
    w.sh_row_slots = 0;
    if (pp_share_possible(L, D, N)) {
        w.sh_hash = off;  off += pp_align256((size_t)D * D * 8);
        w.sh_rep = off;   off += pp_align256((size_t)D * D * 4);
        w.sh_table = off; off += pp_align256((size_t)PP_SHARE_TABLE * 4);
        w.sh_keys = off;  off += pp_align256((size_t)N * 4);
        w.sh_reps = off;  off += pp_align256((size_t)N * 4);
        w.sh_cnt = off;   off += pp_align256((size_t)(PP_SHARE_TABLE / 256) * 4);
        w.sh_start = off; off += pp_align256((size_t)(PP_DP_SLOTS + 2) * 4);
        // DP rows the waves keep for the next candidate of their runs: S - 1 rows each for up
        // to PP_SHARE_ROW_WAVES waves, at most 64 MiB (fewer rows per wave: more waves)
        const size_t row = (size_t)pp_share_row_stride(L) * 4;
        size_t nr = (size_t)PP_SHARE_ROW_WAVES * (S > 1 ? S - 1 : 1);
        if (nr > PP_SHARE_ROW_BYTES / row) nr = PP_SHARE_ROW_BYTES / row;
        if (nr > (size_t)w.slots * (S > 1 ? S - 1 : 1)) nr = (size_t)w.slots * (S > 1 ? S - 1 : 1);
        w.sh_row_slots = (long long)nr;
        w.sh_rows = off;  off += pp_align256(nr * row);
    }
    w.total = off;
    return w;
}

// Extra workspace of the stage-count search, carved after the common part.
struct pp_stage_layout {
    size_t bounds, C, T, part, total;
};

static inline pp_stage_layout pp_layout_stages(const pp_ws_layout &base, int S, int64_t N, int nM) {
    pp_stage_layout w;
    size_t off = base.total;
    w.bounds = off; off += pp_align256((size_t)N * (S * (S + 1) / 2) * 4);
    w.C = off;      off += pp_align256((size_t)N * S * 8);
    w.T = off;      off += pp_align256((size_t)nM * N * S * 8);
    w.part = off;   off += pp_align256((size_t)1024 * 16 * PP_MAX_M_LIST);
    w.total = off;
    return w;
}

// Host-side checks shared by the entry points; returns PP_OK or PP_ERR_INVALID_ARG.
int pp_check_sizes(int L, int D, int S, int64_t N, const int32_t *orderings);

// Enqueue helpers implemented next to their kernels (all return PP_OK / PP_ERR_HIP).
// Fills the workspace tables (and, for orderings == NULL, the explicit list of all D!
// orderings); returns in *ord the ordering array the later kernels must read.
int pp_launch_pack(int L, int D, int S, int64_t N, const int64_t *PF, const int64_t *PB,
                   const int64_t *XF, const int64_t *XB, const int32_t *orderings, void *ws,
                   const pp_ws_layout &lay, const int32_t **ord, hipStream_t st);
// Exactly one of lex_ord (the library's own list of all D! orderings, known to be valid and
// lexicographic) and user_ord (the caller's list, to be validated) is non-NULL.
// stages == 0: C_out [N], bounds_out [N][S].  stages == 1: the plans for every stage count
// xi = 1..S on the first xi devices: C_out [N][S], bounds_out [N][S(S+1)/2], the xi bounds of
// stage count xi at offset xi(xi-1)/2.
// defer_mmax > 0: see pp_fuse_info (the plans are left to the makespan kernel that follows when
// the closed form applies and the times for defer_mmax microbatches fit 32 bits).
// keep_list != 0 (only where lay.sh_table != 0): where candidates share their DP, leave the
// results with the representatives - the caller schedules the list (rlist of
// pp_launch_makespan) and calls pp_launch_share_scatter itself - and set every partial of the
// arg-min in the workspace to "none".
int pp_launch_dp(int L, int D, int S, int64_t N, const int64_t *PF, const int64_t *PB,
                 const int64_t *XF, const int64_t *XB, const int32_t *lex_ord,
                 const int32_t *user_ord, int stages, int defer_mmax, int keep_list,
                 int64_t *C_out, int32_t *bounds_out, void *ws, const pp_ws_layout &lay,
                 int32_t *status, hipStream_t st);
// Candidates whose links have equal channel-time rows, position by position, have the same
// partition DP (pp_share.hip).  pp_launch_share_prepare finds, on the device, one
// representative per sequence of link classes (the lowest candidate index) and leaves the list
// in the workspace (header fields share_*); the DP kernel for L > 128 then walks that list
// only, and pp_launch_share_scatter copies every representative's results (nC entries of C_out
// and nB of bounds_out per candidate) to the candidates it stands for.  Both do nothing when
// the class sequences do not fit the table.  Only where lay.sh_table != 0.
// fill_part != 0: also set the arg-min partials of the workspace (lay.part) to "none".
// run_waves (1 .. PP_DP_SLOTS): the waves of the DP kernel that will walk the list of
// representatives; the list is cut into at most that many runs of about equal work.
int pp_launch_share_prepare(int L, int D, int S, int64_t N, const int64_t *XF, const int64_t *XB,
                            const int32_t *ord, int validate, int fill_part, int run_waves, void *ws,
                            const pp_ws_layout &lay, hipStream_t st);
// With nT > 0 also T_out [nT][N][tw] (the makespan kernel ran over the representatives as well).
int pp_launch_share_scatter(int64_t N, int nC, int nB, int nT, int tw, int64_t *C_out,
                            int32_t *bounds_out, int64_t *T_out, void *ws, const pp_ws_layout &lay,
                            hipStream_t st);

// Makespan of every candidate's plan for each of the nM microbatch counts in Ms (host array).
// With part/C/out non-NULL the launch also finds, per microbatch count, the candidate
// with the smallest T (lowest index on ties) and fills out[q] (one pair of int64 per wave of
// 64 candidates and microbatch count in part).  T_out ([nM][N]) may then be NULL; T_scratch
// ([N]) is needed for S > 16 in that case.  hdr: the workspace header the pack kernel has filled
// for these tables (its largest time decides between 32-bit and 64-bit kernels), or NULL.
// fuse != NULL (pp_best_plan only, needs hdr): the partition DP kernel was told (defer_mmax of
// pp_launch_dp) to leave the plans to the makespan kernel whenever no link's channel time
// depends on the cut position and all finish times for fuse->mmax microbatches fit 32 bits;
// the makespan kernel then builds them from the channel-free tables fuse->bfl and writes
// fuse->C [N] and fuse->bounds [N][S] (the arrays `C` and `bounds` point at as well).  Only
// where pp_makespan_can_fuse(L, D, S) holds.
struct pp_fuse_info {
    int mmax;            // largest microbatch count of the call
    int validate;        // the ordering list came from the caller
    const int64_t *bfl;  // the channel-free tables in the workspace
    int64_t *C;
    int32_t *bounds;
};
bool pp_makespan_can_fuse(int L, int D, int S);
// rlist != NULL (needs hdr and part, and pp_makespan_takes_list(S)): see mk_args.
bool pp_makespan_takes_list(int S);
int pp_launch_makespan(int L, int D, int S, int64_t N, int nM, const int *Ms, const int64_t *PF,
                       const int64_t *PB, const int64_t *XF, const int64_t *XB,
                       const int32_t *orderings, const int32_t *bounds, int64_t *T_out,
                       int64_t *T_scratch, int32_t *status, const int64_t *C, void *part,
                       pp_result *out, const pp_ws_header *hdr, const pp_fuse_info *fuse,
                       const int32_t *rlist, hipStream_t st);
// Stage-count search: makespan of the plan with xi stages of every candidate for xi = 1..S
// (bounds [N][S(S+1)/2] and C [N][S] as pp_launch_dp leaves them with stages == 1), written to
// T_st [nM][N][S], then per microbatch count the smallest T over all (candidate, xi), lowest
// candidate and then lowest xi on ties, into out[q].  part must hold 1024 * nM pairs of int64.
// lex: `orderings` is the library's own list of all D! orderings in lexicographic order.
// rlist != NULL (S <= 16, needs hdr): only the representatives are scheduled (see mk_args).
int pp_launch_makespan_stages(int L, int D, int S, int64_t N, int nM, const int *Ms,
                              const int64_t *PF, const int64_t *PB, const int64_t *XF,
                              const int64_t *XB, const int32_t *orderings, const int32_t *bounds,
                              const int64_t *C, int64_t *T_st, int32_t *status, void *part,
                              pp_result *out, const pp_ws_header *hdr, int lex,
                              const int32_t *rlist, hipStream_t st);
// Makespan (Eq. 2) of the plans with replicated stages of every (candidate, stage count) and
// the keep-the-minimum over them; arrays laid out as pp_plan_replicated documents; part holds
// 1024 pairs of int64.
int pp_launch_rep_makespan(int L, int D, int64_t N, int M, const int64_t *PF, const int64_t *PB,
                           const int64_t *PA, const int64_t *actf, const int64_t *actb,
                           const int64_t *bw, const int32_t *orderings, const int32_t *bounds,
                           const int32_t *reps, const int64_t *W, int64_t *T_out, int32_t *status,
                           void *part, pp_rep_result *out, hipStream_t st);
// Makespan of given plans under a comparison schedule (PP_SCHED_DUPLEX, PP_SCHED_GPIPE).
int pp_launch_makespan_variant(int variant, int L, int D, int S, int64_t N, int M, const int64_t *PF,
                               const int64_t *PB, const int64_t *XF, const int64_t *XB,
                               const int32_t *orderings, const int32_t *bounds, int64_t *T_out,
                               int32_t *status, hipStream_t st);
int pp_launch_argmin(int D, int S, int64_t N, const int64_t *T, const int64_t *C,
                     const int32_t *bounds, const int32_t *orderings, void *part,
                     pp_result *out, hipStream_t st);

// Largest time in the tables (all lanes of a full wave must call; result is uniform).
__device__ __forceinline__ unsigned long long pp_vmax(const pp_ws_header *hdr) {
    unsigned long long m = hdr->pmax[threadIdx.x & (PP_PACK_BLOCKS - 1)];
    for (int off = 32; off; off >>= 1) {
        unsigned long long o = __shfl_xor(m, off);
        m = o > m ? o : m;
    }
    return m;
}

// True iff every link's channel time is the same at every cut position (all lanes of a full
// wave must call; result is uniform).
__device__ __forceinline__ bool pp_is_flat(const pp_ws_header *hdr) {
    return __ballot(hdr->flat[threadIdx.x & (PP_PACK_BLOCKS - 1)] != 0) == ~0ull;
}

__device__ __forceinline__ void pp_raise(int32_t *status, int bit) {
    if (status) atomicOr(status, bit);
}

// Device o[n] of the candidate with lexicographic rank c among all D! orderings
// (factorial number system: digit n = floor(c / (D-1-n)!) mod (D-n) selects the
// digit-th smallest device not used by o[0..n-1]).  Walk n = 0, 1, ... in order with
// `rem` starting at c and `used` at 0.
__device__ __forceinline__ int pp_unrank_next(int D, int n, unsigned long long &rem,
                                              unsigned &used) {
    unsigned long long f = 1;
    for (int i = 2; i <= D - 1 - n; ++i) f *= (unsigned long long)i;
    int digit = (int)(rem / f);
    rem -= (unsigned long long)digit * f;
    int dev = 0;
    for (int d = 0; d < D; ++d) {
        if (!((used >> d) & 1u)) {
            if (digit == 0) { dev = d; break; }
            --digit;
        }
    }
    used |= 1u << dev;
    return dev;
}
