/*
 * ppo.h - CPU oracle for batched synchronous-pipeline plan evaluation.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, obviously-correct host
 * implementation written from the paper (arXiv 2204.10562).  It exists so
 * that the GPU library can be checked against it; it shares no code, header,
 * table or helper with the GPU path, and the product never calls it.
 *
 * Everything is integer (int64 microseconds, bytes, bytes per microsecond),
 * so the results are exact.  All pointers are HOST pointers.
 *
 * Conventions (0-based, half-open):
 *   layers 0..L-1;  PF[l] = sum_{i<l} fwd[i], PB likewise, P = PF + PB.
 *   boundary k (1 <= k <= L-1) = the cut between layer k-1 and layer k; it
 *     carries act_fwd[k-1] bytes forward and act_bwd[k-1] bytes backward.
 *   XF[(u*D+v)*L + (k-1)] = ceil(act_fwd[k-1] / bw[u*D+v])   (u -> v, forward)
 *   XB[(u*D+v)*L + (k-1)] = ceil(act_bwd[k-1] / bw[v*D+u])   (v -> u, backward)
 *     entry L-1 of every row and every diagonal row (u == v) is 0.
 *   candidate c = ordering o_c[0..S-1] of distinct devices; stage n runs on
 *     o_c[n].  A plan = end-exclusive bounds e[0] < e[1] < ... < e[S-1] = L.
 *
 * Pins (tests/, marker "not gpu"): brute force over all contiguous
 * partitions and all orderings on tiny inputs; the paper's cycle example
 * (Sec. IV-A, proof of Lemma 1: M = 6, two stages, 10 cycles); hand-worked
 * two-stage schedules; the bounds M*C <= T <= (M + 4S - 4)*C of Lemma 1;
 * closed forms for S = 1, S = L, M = 1; an independent event-driven
 * simulator.  Parity with the authors' own (unreleased) planner: unpinned.
 */
#ifndef PPO_H
#define PPO_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PPO_OK 0
#define PPO_ERR_INVALID_ARG (-1)
#define PPO_ERR_NOMEM (-2)

/* data faults: returned as a positive OR of these bits; outputs are then
 * unspecified. */
#define PPO_FAULT_BANDWIDTH 1 /* off-diagonal bandwidth <= 0               */
#define PPO_FAULT_NEGATIVE 2  /* negative time or size                     */
#define PPO_FAULT_ORDERING 4  /* ordering row not distinct devices in [0,D)*/
#define PPO_FAULT_BOUNDS 8    /* bounds not strictly increasing to L       */
#define PPO_FAULT_OVERFLOW 16 /* a value reached 2^62                      */

#define PPO_MAX_STAGES 64

typedef struct {
    int64_t best_index; /* lowest c attaining the minimum T; -1 if none */
    int64_t T;          /* per-iteration time of that plan              */
    int64_t C;          /* its per-microbatch bottleneck                */
    int32_t S;
    int32_t bounds[PPO_MAX_STAGES];
    int32_t order[PPO_MAX_STAGES];
} ppo_result;

/* Stage compute time is the sum of per-layer forward+backward times
 * (Lemma 1, definition of C); transfer time is size / bandwidth with one
 * GPU per stage (Sec. III-B, c^f and c^b), rounded up per direction. */
int ppo_prefix_costs(int L, int D, const int64_t *fwd_us, const int64_t *bwd_us,
                     const int64_t *act_fwd_bytes, const int64_t *act_bwd_bytes,
                     const int64_t *bw_bytes_per_us, int64_t *PF, int64_t *PB,
                     int64_t *XF, int64_t *XB);

/* Min-max partition of L layers into S contiguous stages along one device
 * ordering: recursion for W(l, xi, r, i) in Sec. IV-B / the PRM listing in
 * the appendix, with one replica per stage (r = r' = 1, AllReduce term 0),
 * and the factor M divided out.  orderings == NULL means all D! orderings
 * in lexicographic order (requires S == D, N == D!). */
int ppo_partition_dp(int L, int D, int S, int64_t N, const int64_t *PF,
                     const int64_t *PB, const int64_t *XF, const int64_t *XB,
                     const int32_t *orderings, int64_t *C_out,
                     int32_t *bounds_out);

/* Per-iteration time of given plans under the PE scheduler (Alg. 1). */
int ppo_schedule_makespan(int L, int D, int S, int64_t N, int M,
                          const int64_t *PF, const int64_t *PB,
                          const int64_t *XF, const int64_t *XB,
                          const int32_t *orderings, const int32_t *bounds,
                          int64_t *T_out);

/* DP plan per candidate, its makespan, and the keep-the-minimum of the SPP
 * listing (Alg. 3, strict '<' while scanning candidates in order). */
int ppo_best_plan(int L, int D, int S, int64_t N, int M, const int64_t *PF,
                  const int64_t *PB, const int64_t *XF, const int64_t *XB,
                  const int32_t *orderings, ppo_result *out, int64_t *T_all,
                  int64_t *C_all);

/* ppo_best_plan with the stage count searched as well (outer loop of the SPP
 * listing, Alg. 3): every candidate row holds S devices; with xi stages
 * (1 <= xi <= S) the pipeline runs on the first xi of them, partitioned by
 * the recursion for W with xi stages (one replica per stage) and timed by
 * Alg. 1.  Keep-the-minimum with strict '<', scanning candidates in index
 * order and, per candidate, xi = 1, 2, ..., S as the listing does: the winner
 * has the smallest T, then the lowest candidate index, then the fewest stages.
 *   T_all, C_all   [N*S]  value for (c, xi) at c*S + xi-1           (or NULL)
 *   bounds_all     [N*S(S+1)/2]  plan of (c, xi) at c*S(S+1)/2 + xi(xi-1)/2,
 *                  xi entries                                        (or NULL)
 *   out->S is the winning stage count; bounds/order hold that many entries. */
int ppo_best_plan_stages(int L, int D, int S, int64_t N, int M, const int64_t *PF,
                         const int64_t *PB, const int64_t *XF, const int64_t *XB,
                         const int32_t *orderings, ppo_result *out, int64_t *T_all,
                         int64_t *C_all, int32_t *bounds_all);

/* The complete planner with replicated stages, for every candidate ordering of
 * all D devices (Alg. 3 with Alg. 4 and Alg. 1; the ordering is given instead
 * of computed by Alg. 2).
 *   PRM (Alg. 4, recursion for W(l, xi, r, i) in Sec. IV-B): memoised recursion
 *   written as the listing: base case one stage replicated over all i GPUs,
 *   otherwise min over l' = 1..l-1 and r' = 1..i-r (in this order, replaced only
 *   on strict improvement) of the max of the sub-problem, the channel and the
 *   last stage.  Integer readings: a stage of r replicas takes
 *   ceil(sum p^f / r) forward and ceil(sum p^b / r) backward per microbatch;
 *   c^f = ceil(d^f / (r' r min b_{v',v})), c^b = ceil(d^b / (r' r min b_{v,v'}))
 *   (v' in the earlier stage); A = ceil(2 (r-1) sum alpha / (r min b)) over
 *   the ordered pairs of the replica set (Eq. 1), 0 for r = 1; the stage term
 *   is M (F + B) + A and the channel term M (c^f + c^b).
 *   SPP (Alg. 3): for xi = 1..D: r = first minimiser of W(L, xi, r, D); plan;
 *   T = max(T_PE, max over replicated stages of (end of its last backward pass
 *   + A)) (Eq. 2, Alg. 1 on the per-replica times); keep the smallest T,
 *   strict '<', candidates in index order and xi ascending.
 *   alpha_bytes [L]; orderings [N*D] or NULL = all D! in lexicographic order.
 *   T_all, W_all [N*D] at c*D + xi-1 (INT64_MAX = no plan with xi stages);
 *   bounds_all, reps_all [N*D(D+1)/2], the xi entries of (c, xi) at
 *   c*D(D+1)/2 + xi(xi-1)/2.  All optional. */
typedef struct {
    int64_t best_index, T, W;
    int32_t S;
    int32_t bounds[PPO_MAX_STAGES]; /* S entries */
    int32_t reps[PPO_MAX_STAGES];   /* S entries, sum = D */
    int32_t order[PPO_MAX_STAGES];  /* D entries: device of every rank */
} ppo_rep_result;

int ppo_spp_replicated(int L, int D, int64_t N, int M, const int64_t *fwd_us,
                       const int64_t *bwd_us, const int64_t *act_fwd_bytes,
                       const int64_t *act_bwd_bytes, const int64_t *alpha_bytes,
                       const int64_t *bw_bytes_per_us, const int32_t *orderings,
                       ppo_rep_result *out, int64_t *T_all, int64_t *W_all,
                       int32_t *bounds_all, int32_t *reps_all);

/* Execution-ordering phase of Alg. 1 alone, for a pipeline of S stages and
 * M microbatches.  rounds_out[t*(4S-3) + (j-1)] = microbatch (1-based) that
 * block j handles in sweep t, or 0.  Returns the number of sweeps, or a
 * negative error; max_rounds is the capacity of rounds_out in sweeps. */
int ppo_execution_order(int S, int M, int32_t *rounds_out, int max_rounds);

/* Makespan of one pipeline given directly by its durations (no tables):
 * F[n], B[n] for stages 0..S-1; cf[n], cb[n] for channel n (between stage
 * n-1 and n), entries 1..S-1 used.  start_out/finish_out, if not NULL, get
 * the start/finish time of block j (1-based) for microbatch m (1-based) at
 * [(j-1)*M + (m-1)]. */
int64_t ppo_pe_makespan(int S, int M, const int64_t *F, const int64_t *B,
                        const int64_t *cf, const int64_t *cb,
                        int64_t *start_out, int64_t *finish_out);

/* Schedule variants, for comparison with the PE scheduler.  Same timing rule as
 * the scheduling phase of Alg. 1 (an item starts when its microbatch has left
 * the preceding block and its resource is idle; resources follow their lists):
 *   PPO_SCHED_PE      Alg. 1 itself (equals ppo_pe_makespan)
 *   PPO_SCHED_DUPLEX  Alg. 1 with separate channels for the forward and the
 *                     backward transfers of a stage pair
 *   PPO_SCHED_GPIPE   all forward passes before any backward pass on every
 *                     stage and channel (the GPipe schedule as Sec. II describes
 *                     it), microbatches in order; last stage's F and B separate
 *   PPO_SCHED_ADDITIVE  no channels as resources: a stage's inbound transfers are
 *                     part of its passes (forward block of stage n takes
 *                     cf[n] + F[n], backward block B[n] + cb[n]; the last stage's
 *                     merged block all four), so a microbatch passes 2S-1 blocks
 *                     on S resources; ordering and scheduling phases of Alg. 1
 *                     on that shorter list ("stage cost = compute plus transfer")
 *   PPO_SCHED_FIFO    Alg. 1 read strictly: only computation blocks follow the
 *                     lists U_s; a channel, whenever idle, starts the waiting
 *                     transfer whose preceding block finished first (equal
 *                     times: the one earlier in the order of Alg. 1's first
 *                     phase).  Evaluated as an event simulation that always
 *                     commits the item with the earliest start next (equal
 *                     starts: the lowest resource).
 * F, B per stage; cf, cb per channel with entry 0 unused. */
#define PPO_SCHED_PE 0
#define PPO_SCHED_DUPLEX 1
#define PPO_SCHED_GPIPE 2
#define PPO_SCHED_ADDITIVE 3
#define PPO_SCHED_FIFO 4
int64_t ppo_variant_makespan(int variant, int S, int M, const int64_t *F,
                             const int64_t *B, const int64_t *cf, const int64_t *cb);
int ppo_schedule_makespan_variant(int variant, int L, int D, int S, int64_t N, int M,
                                  const int64_t *PF, const int64_t *PB,
                                  const int64_t *XF, const int64_t *XB,
                                  const int32_t *orderings, const int32_t *bounds,
                                  int64_t *T_out);

/* Recursive device ordering (Alg. 2, Sec. IV-B): find a minimum cut of the
 * GPU graph, order the two sides recursively, first side first.  The graph
 * is undirected with weight bw[u][v] + bw[v][u] on edge {u, v} (twice the
 * bandwidth for a symmetric matrix).  The minimum cut is found with the
 * Stoer-Wagner algorithm (the routine the paper cites): vertices of the
 * current subgraph in ascending index order; every phase starts from the
 * remaining vertex of lowest index (a merged vertex counts as its lowest
 * member), adds the most tightly connected vertex, ties to the lowest index;
 * a later phase replaces the best cut only if strictly lighter.  The side
 * that holds the lowest-index vertex comes first.  order_out[rank] = device.
 * Returns PPO_OK or PPO_ERR_*. */
int ppo_rdo_order(int D, const int64_t *bw_bytes_per_us, int32_t *order_out);

/* threads the candidate loops use (OpenMP), and a setter */
int ppo_get_num_threads(void);
void ppo_set_num_threads(int n);

#ifdef __cplusplus
}
#endif
#endif
