/*
 * pp.h - batched evaluation of synchronous-pipeline plans on one MI355X.
 *
 * C ABI of libpp (hand-written HIP kernels for gfx950).  The library is the
 * data-parallel hot path of the planner of arXiv 2204.10562: for a batch of
 * candidate device orderings it partitions the L layers of a model into
 * contiguous stages with a min-max dynamic program, computes every plan's
 * per-iteration time for M microbatches under the paper's pipeline execution
 * scheduler, and keeps the best plan.
 *
 * General rules
 *   - Every array pointer is a DEVICE pointer unless marked "host".  The
 *     caller owns all buffers; the library allocates nothing, keeps no state
 *     between calls and never synchronises.  All work is enqueued on
 *     `stream` (a hipStream_t passed as void*, NULL = the default stream)
 *     and the outputs are valid once that stream has reached the call's end.
 *   - Times are int64 microseconds, sizes int64 bytes, bandwidth int64 bytes
 *     per microsecond (1 GB/s = 1000).  Everything is exact integer work.
 *   - Layers 0..L-1.  PF[l] = sum_{i<l} fwd[i], PB likewise (length L+1).
 *     Boundary k (1 <= k <= L-1) is the cut between layers k-1 and k.
 *     XF[(u*D+v)*L + (k-1)] is the forward transfer time over the link u->v
 *     at boundary k, XB[(u*D+v)*L + (k-1)] the backward one (over v->u).
 *   - A candidate c is a row o_c[0..S-1] of distinct devices: stage n runs on
 *     device o_c[n].  A plan is its end-exclusive stage bounds
 *     e[0] < e[1] < ... < e[S-1] = L (stage n = layers [e[n-1], e[n])).
 *   - Return value: PP_OK, or a negative PP_ERR_* for a problem the host can
 *     see (then nothing was enqueued).  Problems in the data can only be seen
 *     on the device: they are OR-ed (atomically) as PP_FAULT_* bits into the
 *     caller's int32 `*status` (device memory, cleared by the caller).  When
 *     a call sets a fault bit its outputs are unspecified, but no kernel
 *     reads or writes out of bounds because of bad data.
 *   - Limits: 1 <= S <= min(L, D, PP_MAX_STAGES); L <= PP_MAX_LAYERS;
 *     D <= PP_MAX_DEVICES; M >= 1; N >= 1.
 */
#ifndef PP_H
#define PP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PP_OK 0
#define PP_ERR_INVALID_ARG (-1) /* NULL required pointer, size out of range  */
#define PP_ERR_WORKSPACE (-2)   /* workspace NULL, misaligned or too small   */
#define PP_ERR_HIP (-3)         /* a kernel launch failed                    */

#define PP_FAULT_BANDWIDTH 1 /* an off-diagonal bandwidth is <= 0            */
#define PP_FAULT_NEGATIVE 2  /* a negative time or size                      */
#define PP_FAULT_ORDERING 4  /* an ordering row is not distinct devices<D    */
#define PP_FAULT_BOUNDS 8    /* bounds not strictly increasing up to L       */
#define PP_FAULT_OVERFLOW 16 /* a value reached 2^62                         */

#define PP_MAX_STAGES 64
#define PP_MAX_LAYERS 2048
#define PP_MAX_DEVICES 1024
#define PP_MAX_M_LIST 16 /* microbatch counts per pp_best_plan_multi call */

/* Winner record written by pp_best_plan (device memory, 536 bytes). */
typedef struct {
    int64_t best_index; /* lowest candidate index with the minimum T       */
    int64_t T;          /* its per-iteration time (us)                     */
    int64_t C;          /* its per-microbatch bottleneck (us); W = M * C   */
    int32_t S;
    int32_t bounds[PP_MAX_STAGES]; /* entries 0..S-1                       */
    int32_t order[PP_MAX_STAGES];  /* entries 0..S-1                       */
} pp_result;

/*
 * Cost tables, once per problem.
 * Stage compute time is the sum of its layers' forward+backward times
 * (Lemma 1, definition of C), hence the prefix sums.  Transfer time between
 * consecutive stages is size / bandwidth of the link that joins their GPUs
 * (Sec. III-B, c^f over b_{v,v'} and c^b over b_{v',v}, one GPU per stage),
 * here ceil(bytes / bw) per direction.
 *   fwd_us, bwd_us        [L]   per-layer per-microbatch times
 *   act_fwd_bytes         [L]   bytes sent forward across the boundary after
 *                               layer l; entry L-1 is ignored
 *   act_bwd_bytes         [L]   bytes sent backward across it; NULL = same
 *                               as act_fwd_bytes
 *   bw_bytes_per_us       [D*D] bw[u*D+v] = bandwidth u -> v; diagonal ignored
 *   PF, PB                [L+1] out
 *   XF, XB                [D*D*L] out; entry L-1 of each row and the
 *                               diagonal rows are 0
 * Faults: BANDWIDTH, NEGATIVE, OVERFLOW.
 */
int pp_prefix_costs(int L, int D, const int64_t *fwd_us, const int64_t *bwd_us,
                    const int64_t *act_fwd_bytes, const int64_t *act_bwd_bytes,
                    const int64_t *bw_bytes_per_us, int64_t *PF, int64_t *PB,
                    int64_t *XF, int64_t *XB, int32_t *status, void *stream);

/*
 * Bytes of device workspace pp_partition_dp and pp_best_plan need for a
 * problem of this size (host function; 0 if the sizes are out of range).
 * The workspace must be 256-byte aligned; its contents need not be kept
 * between calls.
 *
 * Diagnostics: after pp_partition_dp or pp_best_plan the workspace holds, from
 * byte PP_WS_WORK on, 64 records PP_WS_WORK_STRIDE bytes apart; the uint64 at
 * the start of each record adds up (over the 64) to the number of (cell,
 * split) pairs the dynamic program actually evaluated in that call, the
 * uint64 after it to the number of DP rows it computed.  Rows that
 * consecutive candidates share (equal ordering prefixes) are computed and
 * counted once, and the kernel for L > 128 skips splits that cannot matter, so
 * these can be far below N * pairs-per-candidate.
 *
 * For L > 128 and D <= 64 the dynamic program is computed once for every
 * group of candidates whose links have the same transfer times at every cut
 * position (the rows of XF and XB of link (o[n-1], o[n]) equal, n = 1..S-1)
 * whenever (number of distinct link rows)^(S-1) <= 2^20; the four uint32 at
 * byte PP_WS_SHARE then hold: 1 (0 if every candidate was computed on its
 * own), the number of distinct link rows, that power, and the number of
 * candidates computed.  Where that power is too large the candidates are
 * instead taken in the order of their first k devices (D^k <= 2^20), so that
 * consecutive ones share the first k - 1 rows: the uint32 at byte
 * PP_WS_SHARE + 24 is then 1 and the one after it k.
 */
#define PP_WS_WORK 1024
#define PP_WS_WORK_STRIDE 128
#define PP_WS_SHARE 768
size_t pp_workspace_bytes(int L, int D, int S, int64_t N);

/*
 * Min-max partition along every candidate ordering.
 * Recursion for W(l, xi, r, i) of Sec. IV-B and the PRM listing (appendix)
 * with one replica per stage (r = r' = 1, AllReduce term 0) and the common
 * factor M divided out:
 *   W[0][l] = P[l],   P = PF + PB
 *   W[n][l] = min_{n <= k <= l-1} max( W[n-1][k],
 *                                      XF[o[n-1]][o[n]][k-1] + XB[..][k-1],
 *                                      P[l] - P[k] )
 * The lowest minimising k is kept (strict-improvement update with k
 * ascending), and the plan is read back from (S-1, L).
 *   orderings   [N*S] int32, or NULL = all D! orderings in lexicographic
 *               order, candidate index = lexicographic rank (needs S == D,
 *               N == D!)
 *   C_out       [N]   per-microbatch bottleneck W[S-1][L] of each candidate
 *   bounds_out  [N*S] its plan
 * Faults: ORDERING.
 */
int pp_partition_dp(int L, int D, int S, int64_t N, const int64_t *PF,
                    const int64_t *PB, const int64_t *XF, const int64_t *XB,
                    const int32_t *orderings, int64_t *C_out,
                    int32_t *bounds_out, void *workspace,
                    size_t workspace_bytes, int32_t *status, void *stream);

/*
 * Per-iteration time of given plans (any valid bounds, not only the DP's)
 * under the pipeline execution scheduler (Alg. 1, Sec. IV-A): 2S-1 serial
 * resources (stages and, between them, one channel for both directions);
 * 4S-3 blocks per microbatch (the last stage's forward and backward are one
 * block); block j serves microbatch t-j+1 in sweep t; every resource serves
 * its work in (sweep, block) order, each item starting once its microbatch
 * has left the preceding block and the resource is idle.  T is the finish of
 * the last backward block on stage 0 (first term of the makespan objective,
 * Eq. 2; nothing is replicated).
 *   bounds  [N*S]   T_out  [N]
 * Faults: ORDERING, BOUNDS, OVERFLOW ((M+4S-4) * largest block >= 2^62).
 */
int pp_schedule_makespan(int L, int D, int S, int64_t N, int M,
                         const int64_t *PF, const int64_t *PB,
                         const int64_t *XF, const int64_t *XB,
                         const int32_t *orderings, const int32_t *bounds,
                         int64_t *T_out, int32_t *status, void *stream);

/*
 * pp_schedule_makespan for several microbatch counts in one launch (Alg. 1 once
 * per count on the same plans): the plans' block durations are gathered once
 * and the counts are scheduled side by side.
 *   nM      number of microbatch counts, 1..PP_MAX_M_LIST
 *   M_list  [nM] HOST array, every entry >= 1
 *   T_out   [nM*N], T of candidate c for M_list[q] at q*N + c
 * Same faults as pp_schedule_makespan.
 */
int pp_schedule_makespan_multi(int L, int D, int S, int64_t N, int nM,
                               const int32_t *M_list, const int64_t *PF,
                               const int64_t *PB, const int64_t *XF,
                               const int64_t *XB, const int32_t *orderings,
                               const int32_t *bounds, int64_t *T_out,
                               int32_t *status, void *stream);

/*
 * pp_schedule_makespan under a comparison schedule.  The timing rule is that of
 * Alg. 1's scheduling phase in every case (an item starts when its microbatch
 * has left the preceding block and its resource is idle; resources follow their
 * service lists); what changes is the resources or the lists:
 *   PP_SCHED_PE      Alg. 1 itself (same as pp_schedule_makespan)
 *   PP_SCHED_DUPLEX  Alg. 1's blocks and ordering phase, but the forward and the
 *                    backward transfers of a stage pair use separate channels
 *   PP_SCHED_GPIPE   every stage and channel serves all forward items before
 *                    any backward item, microbatches in order (the schedule
 *                    Sec. II attributes to GPipe: all FP before any BP); the
 *                    last stage's forward and backward are separate items
 *   PP_SCHED_ADDITIVE  stages are the only resources: the transfers over a
 *                    stage's inbound link are part of that stage's passes
 *                    (forward block of stage n: XF + F, backward block:
 *                    B + XB; the last stage's merged block all four), so a
 *                    microbatch passes 2S-1 blocks; Alg. 1's ordering and
 *                    scheduling phases on that list ("stage cost = compute
 *                    plus transfer" instead of overlapping channels)
 *   PP_SCHED_FIFO    Alg. 1 read strictly: only computation blocks follow the
 *                    lists; a channel that is idle starts the waiting transfer
 *                    whose preceding block finished first (equal times: the
 *                    one earlier in the order of Alg. 1's first phase).
 *                    Evaluated as an event simulation that commits the item
 *                    with the earliest start next (equal starts: the lowest
 *                    resource, resources numbered along the pipeline)
 * Same arguments, limits and faults as pp_schedule_makespan; an unknown variant
 * returns PP_ERR_INVALID_ARG.
 */
#define PP_SCHED_PE 0
#define PP_SCHED_DUPLEX 1
#define PP_SCHED_GPIPE 2
#define PP_SCHED_ADDITIVE 3
#define PP_SCHED_FIFO 4
int pp_schedule_makespan_variant(int variant, int L, int D, int S, int64_t N, int M,
                                 const int64_t *PF, const int64_t *PB,
                                 const int64_t *XF, const int64_t *XB,
                                 const int32_t *orderings, const int32_t *bounds,
                                 int64_t *T_out, int32_t *status, void *stream);

/*
 * The whole path: partition DP per candidate, makespan of each plan, and the
 * keep-the-minimum of the SPP listing (Alg. 3: replace only on strictly
 * smaller T while scanning candidates in index order, so the lowest index
 * wins ties).
 *   out     one pp_result
 *   T_all   [N] or NULL     C_all  [N] or NULL
 * Faults: ORDERING, OVERFLOW.
 */
int pp_best_plan(int L, int D, int S, int64_t N, int M, const int64_t *PF,
                 const int64_t *PB, const int64_t *XF, const int64_t *XB,
                 const int32_t *orderings, pp_result *out, int64_t *T_all,
                 int64_t *C_all, void *workspace, size_t workspace_bytes,
                 int32_t *status, void *stream);

/*
 * pp_best_plan for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, outputs, faults and results as
 * pp_best_plan, minus the workspace: the scratch memory is a device array of
 * PP_STATIC_WORKSPACE_BYTES that is part of the library's code object (every
 * GPU the library runs on holds one copy until the process ends).  The call
 * allocates nothing and frees nothing; the first call on a device looks up
 * the array's address (no allocation either).
 *   - Problems whose pp_workspace_bytes(L, D, S, N) exceeds
 *     PP_STATIC_WORKSPACE_BYTES are rejected with PP_ERR_WORKSPACE and nothing
 *     is enqueued (the GPT-shaped configuration, L = 128, D = S = 8, all 40320
 *     orderings, needs 19.4 MiB).
 *   - All calls on one GPU share that GPU's array: two calls that overlap in
 *     time on one GPU (different streams, different host threads) race.  The
 *     array keeps the previous call's contents; nothing in it needs to start
 *     at zero except the work counters, which the call's first kernel clears.
 *   - Returns PP_ERR_HIP if the array's address cannot be obtained.
 */
#define PP_STATIC_WORKSPACE_BYTES (32u << 20)
int pp_best_plan_static(int L, int D, int S, int64_t N, int M, const int64_t *PF,
                        const int64_t *PB, const int64_t *XF, const int64_t *XB,
                        const int32_t *orderings, pp_result *out, int64_t *T_all,
                        int64_t *C_all, int32_t *status, void *stream);

/*
 * pp_best_plan for several microbatch counts at once.  The partition (a
 * plan's bounds and C) does not depend on M, because every term of the
 * recursion for W carries the same factor M when nothing is replicated
 * (Sec. IV-B); so the dynamic program runs once and only the schedule
 * (Alg. 1) and the keep-the-minimum (Alg. 3) are repeated per M.
 *   nM      number of microbatch counts, 1..PP_MAX_M_LIST
 *   M_list  [nM] HOST array, every entry >= 1
 *   out     [nM] pp_result, out[q] = winner for M_list[q]
 *   T_all   [nM*N] (T of candidate c for M_list[q] at q*N + c) or NULL
 *   C_all   [N] or NULL
 * Same workspace size and faults as pp_best_plan.
 */
int pp_best_plan_multi(int L, int D, int S, int64_t N, int nM,
                       const int32_t *M_list, const int64_t *PF,
                       const int64_t *PB, const int64_t *XF, const int64_t *XB,
                       const int32_t *orderings, pp_result *out, int64_t *T_all,
                       int64_t *C_all, void *workspace, size_t workspace_bytes,
                       int32_t *status, void *stream);

/*
 * Stage-count search: the outer loop of the SPP listing (Alg. 3), which varies
 * the number of stages xi and keeps the plan with the smallest per-iteration
 * time.  Every candidate row holds S devices; with xi stages (1 <= xi <= S)
 * the pipeline runs on the first xi of them (with one replica per stage the
 * recursion for W(l, xi, r, i) places stage n on the n-th device of the
 * ordering).  Row xi-1 of the table W of pp_partition_dp depends only on those
 * xi devices, so one dynamic program per candidate yields all S plans:
 * C(c, xi) = W[xi-1][L], bounds read back from (xi-1, L).
 *
 * pp_partition_dp_stages: the S plans of every candidate.
 *   C_out       [N*S]          C(c, xi) at c*S + xi-1
 *   bounds_out  [N*S(S+1)/2]   the xi bounds of (c, xi) at
 *                              c*S(S+1)/2 + xi(xi-1)/2
 *   workspace   as for pp_partition_dp (pp_workspace_bytes)
 *   Faults: ORDERING (checked on the whole row of S devices).
 *
 * pp_best_plan_stages: those plans, the makespan (Alg. 1) of each for every
 * microbatch count, and per microbatch count the keep-the-minimum of Alg. 3
 * with strict '<', candidates scanned in index order and, per candidate,
 * xi = 1, 2, ..., S: smallest T, then lowest candidate, then fewest stages.
 *   out     [nM] pp_result; out[q].S is the winning stage count and bounds /
 *           order hold that many entries (the rest are 0)
 *   T_all   [nM*N*S] (T of (c, xi) for M_list[q] at (q*N + c)*S + xi-1) or NULL
 *   C_all   [N*S] or NULL
 *   workspace   pp_workspace_bytes_stages(L, D, S, N, nM) bytes (host function;
 *               0 if a size is out of range)
 *   Faults: ORDERING, OVERFLOW.
 */
size_t pp_workspace_bytes_stages(int L, int D, int S, int64_t N, int nM);
int pp_partition_dp_stages(int L, int D, int S, int64_t N, const int64_t *PF,
                           const int64_t *PB, const int64_t *XF, const int64_t *XB,
                           const int32_t *orderings, int64_t *C_out,
                           int32_t *bounds_out, void *workspace,
                           size_t workspace_bytes, int32_t *status, void *stream);
int pp_best_plan_stages(int L, int D, int S, int64_t N, int nM,
                        const int32_t *M_list, const int64_t *PF,
                        const int64_t *PB, const int64_t *XF, const int64_t *XB,
                        const int32_t *orderings, pp_result *out, int64_t *T_all,
                        int64_t *C_all, void *workspace, size_t workspace_bytes,
                        int32_t *status, void *stream);

/*
 * The complete planner with replicated stages (Alg. 3 with Alg. 4 and Alg. 1)
 * for a batch of orderings of ALL D devices.  A stage may run on k GPUs of
 * consecutive ranks (Sec. III-B): a replica then takes ceil(sum p / k) per
 * microbatch and pass, a transfer between stages of k' and k replicas
 * ceil(d / (k' k min b)) per direction (minimum over the links from the
 * sending to the receiving GPU set), and a replicated stage ends with a ring
 * AllReduce of A = ceil(2 (k-1) sum alpha / (k min b)) (Eq. 1; minimum over the
 * ordered pairs of its GPUs; 0 for k = 1).
 *   PRM (Alg. 4; recursion for W(l, xi, r, i) of Sec. IV-B):
 *     W(l, 1, i, i)  = M (F + B) + A,   layers [0, l) on ranks 0..i-1
 *     W(l, xi, r, i) = min over l' = xi-1..l-1 and r' = 1..i-r of
 *                      max{ W(l', xi-1, r', i-r), M (c^f + c^b), M (F + B) + A }
 *     the first minimiser in (l', r') order is kept (strict-improvement update).
 *   SPP (Alg. 3), per candidate: for xi = 1..D the first r with the smallest
 *     W(L, xi, r, D), its plan, and the plan's T = max(end of the last backward
 *     block on stage 0 under Alg. 1, end of the last AllReduce) (Eq. 2, an
 *     AllReduce starts when its stage's last backward pass has finished); then
 *     keep-the-minimum with strict '<': smallest T, then lowest candidate, then
 *     fewest stages.
 *   fwd_us, bwd_us, act_fwd_bytes, act_bwd_bytes (NULL = forward's), alpha_bytes
 *   [L]; bw_bytes_per_us [D*D]; orderings [N*D] or NULL = all D! orderings in
 *   lexicographic order (N = D!).
 *   out      one pp_rep_result
 *   T_all, W_all  [N*D]: value of (c, xi) at c*D + xi-1, INT64_MAX where no plan
 *                 with xi stages exists (xi > L); either may be NULL
 *   bounds_all, reps_all  [N*D(D+1)/2]: the xi entries of (c, xi) at
 *                 c*D(D+1)/2 + xi(xi-1)/2; either may be NULL
 *   workspace     pp_workspace_bytes_replicated(L, D, N) bytes, 256-byte aligned
 * Limits: D <= 16 and (48 + 8 D)(L + 1) + 88 <= 65536 (the tables of one state
 * live in LDS): L <= 583 at D = 8, L <= 370 at D = 16; otherwise
 * PP_ERR_INVALID_ARG (pp_workspace_bytes_replicated returns 0);
 * sums of times * (M + 4D) and of parameter sizes * 2D below 2^62.
 * Faults: NEGATIVE, BANDWIDTH, ORDERING, OVERFLOW.
 */
typedef struct {
    int64_t best_index; /* lowest candidate index with the minimum T; -1 if none */
    int64_t T;          /* its per-iteration time (us)                           */
    int64_t W;          /* its W(|S|) (us)                                        */
    int32_t S;          /* its number of stages                                  */
    int32_t bounds[PP_MAX_STAGES]; /* entries 0..S-1                             */
    int32_t reps[PP_MAX_STAGES];   /* GPUs per stage, entries 0..S-1, sum = D    */
    int32_t order[PP_MAX_STAGES];  /* device of every rank, entries 0..D-1      */
} pp_rep_result;

size_t pp_workspace_bytes_replicated(int L, int D, int64_t N);
int pp_plan_replicated(int L, int D, int64_t N, int M, const int64_t *fwd_us,
                       const int64_t *bwd_us, const int64_t *act_fwd_bytes,
                       const int64_t *act_bwd_bytes, const int64_t *alpha_bytes,
                       const int64_t *bw_bytes_per_us, const int32_t *orderings,
                       pp_rep_result *out, int64_t *T_all, int64_t *W_all,
                       int32_t *bounds_all, int32_t *reps_all, void *workspace,
                       size_t workspace_bytes, int32_t *status, void *stream);

/*
 * Recursive device ordering (Alg. 2, Sec. IV-B): one heuristic ordering of the
 * D devices, meant as an extra candidate row (or the only one when D! is out
 * of reach).  HOST function, host pointers, no GPU work: the device graph is
 * split at a minimum cut, each side is ordered recursively, and the ranks of
 * the first side precede those of the second, so that weak links end up
 * between far-apart ranks.
 *   bw_bytes_per_us  [D*D] host, the matrix pp_prefix_costs takes; the graph is
 *                    undirected with weight bw[u][v] + bw[v][u] on edge {u,v};
 *                    diagonal ignored; entries must lie in [0, 2^62 / D^2]
 *   order_out        [D] host, order_out[rank] = device
 * The minimum cut is Stoer-Wagner's (the routine the paper cites), made
 * deterministic: a merged vertex counts as its lowest device; a phase starts
 * at the lowest remaining vertex and adds the most tightly connected one,
 * ties to the lowest; a later phase replaces the lightest cut so far only if
 * strictly lighter; the side that holds the lowest device is ordered first.
 * Returns PP_OK or PP_ERR_INVALID_ARG.
 */
int pp_rdo_order(int D, const int64_t *bw_bytes_per_us, int32_t *order_out);

/* Text for a PP_ERR_* code (host function, static storage). */
const char *pp_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif
