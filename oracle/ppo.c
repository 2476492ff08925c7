/*
 * ppo.c - CPU oracle for batched synchronous-pipeline plan evaluation.
 *
 * TEST INFRASTRUCTURE ONLY (see ppo.h).  Plain nested loops in int64, one
 * function per step of the method, each following the passage it cites.
 * No blocking, fusion or reordering; the only parallelism is an OpenMP loop
 * over independent candidates.
 */
#include "ppo.h"

#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define INF INT64_MAX
#define CAP ((int64_t)1 << 62)

static int g_threads = 0; /* 0 = OpenMP default */

int ppo_get_num_threads(void) {
#ifdef _OPENMP
    return g_threads > 0 ? g_threads : omp_get_max_threads();
#else
    return 1;
#endif
}

void ppo_set_num_threads(int n) { g_threads = n > 0 ? n : 0; }

static int64_t max2(int64_t a, int64_t b) { return a > b ? a : b; }

/* ceil(a / b) for a >= 0, b >= 1 */
static int64_t ceil_div(int64_t a, int64_t b) { return a / b + (a % b != 0); }

/* ------------------------------------------------------------------ */
/* Step 1: prefix sums and transfer-time tables                         */
/* ------------------------------------------------------------------ */

int ppo_prefix_costs(int L, int D, const int64_t *fwd_us, const int64_t *bwd_us,
                     const int64_t *act_fwd_bytes, const int64_t *act_bwd_bytes,
                     const int64_t *bw, int64_t *PF, int64_t *PB, int64_t *XF,
                     int64_t *XB) {
    if (L < 1 || D < 1 || !fwd_us || !bwd_us || !act_fwd_bytes || !bw || !PF ||
        !PB || !XF || !XB)
        return PPO_ERR_INVALID_ARG;
    if (!act_bwd_bytes) act_bwd_bytes = act_fwd_bytes;
    int fault = 0;

    /* stage compute time = sum over its layers of p^f_l + p^b_l */
    PF[0] = 0;
    PB[0] = 0;
    for (int l = 0; l < L; ++l) {
        if (fwd_us[l] < 0 || bwd_us[l] < 0) fault |= PPO_FAULT_NEGATIVE;
        if (fwd_us[l] >= CAP || bwd_us[l] >= CAP) fault |= PPO_FAULT_OVERFLOW;
        /* unsigned add: wrap-around is defined; a wrapped value is a fault */
        PF[l + 1] = (int64_t)((uint64_t)PF[l] + (uint64_t)fwd_us[l]);
        PB[l + 1] = (int64_t)((uint64_t)PB[l] + (uint64_t)bwd_us[l]);
        if (PF[l + 1] >= CAP || PF[l + 1] < 0 || PB[l + 1] >= CAP ||
            PB[l + 1] < 0)
            fault |= PPO_FAULT_OVERFLOW;
    }
    for (int l = 0; l + 1 < L; ++l)
        if (act_fwd_bytes[l] < 0 || act_bwd_bytes[l] < 0)
            fault |= PPO_FAULT_NEGATIVE;

    /* c^f = d^f / b_{v,v'},  c^b = d^b / b_{v',v}  (one GPU per stage) */
    for (int u = 0; u < D; ++u)
        for (int v = 0; v < D; ++v) {
            int64_t *xf = XF + ((size_t)u * D + v) * L;
            int64_t *xb = XB + ((size_t)u * D + v) * L;
            for (int k = 0; k < L; ++k) xf[k] = xb[k] = 0;
            if (u == v) continue;
            int64_t buv = bw[(size_t)u * D + v], bvu = bw[(size_t)v * D + u];
            if (buv <= 0 || bvu <= 0) {
                fault |= PPO_FAULT_BANDWIDTH;
                continue;
            }
            for (int k = 0; k + 1 < L; ++k) {
                if (act_fwd_bytes[k] >= 0) xf[k] = ceil_div(act_fwd_bytes[k], buv);
                if (act_bwd_bytes[k] >= 0) xb[k] = ceil_div(act_bwd_bytes[k], bvu);
                if (xf[k] >= CAP || xb[k] >= CAP) fault |= PPO_FAULT_OVERFLOW;
            }
        }
    return fault;
}

/* ------------------------------------------------------------------ */
/* candidate orderings                                                  */
/* ------------------------------------------------------------------ */

static int64_t factorial_or_neg(int D) {
    int64_t f = 1;
    for (int i = 2; i <= D; ++i) {
        if (f > INT64_MAX / i) return -1;
        f *= i;
    }
    return f;
}

/* next permutation in lexicographic order (textbook: find the longest
 * non-increasing suffix, swap its predecessor with the next larger element
 * of the suffix, reverse the suffix) */
static void next_perm(int32_t *a, int n) {
    int i = n - 2;
    while (i >= 0 && a[i] >= a[i + 1]) --i;
    if (i < 0) return;
    int j = n - 1;
    while (a[j] <= a[i]) --j;
    int32_t t = a[i];
    a[i] = a[j];
    a[j] = t;
    for (int p = i + 1, q = n - 1; p < q; ++p, --q) {
        t = a[p];
        a[p] = a[q];
        a[q] = t;
    }
}

/* all D! orderings, row c = the c-th in lexicographic order */
static int32_t *all_orderings(int D, int64_t N) {
    int32_t *o = (int32_t *)malloc((size_t)N * D * sizeof(int32_t));
    if (!o) return NULL;
    for (int i = 0; i < D; ++i) o[i] = i;
    for (int64_t c = 1; c < N; ++c) {
        memcpy(o + c * D, o + (c - 1) * D, (size_t)D * sizeof(int32_t));
        next_perm(o + c * D, D);
    }
    return o;
}

static int check_common(int L, int D, int S, int64_t N, const int32_t *orderings) {
    if (L < 1 || D < 1 || S < 1 || S > L || S > D || S > PPO_MAX_STAGES || N < 1)
        return PPO_ERR_INVALID_ARG;
    if (!orderings) {
        if (S != D) return PPO_ERR_INVALID_ARG;
        int64_t f = factorial_or_neg(D);
        if (f < 0 || f != N) return PPO_ERR_INVALID_ARG;
    }
    return PPO_OK;
}

static int ordering_ok(const int32_t *o, int S, int D) {
    for (int n = 0; n < S; ++n) {
        if (o[n] < 0 || o[n] >= D) return 0;
        for (int q = 0; q < n; ++q)
            if (o[q] == o[n]) return 0;
    }
    return 1;
}

static int bounds_ok(const int32_t *e, int S, int L) {
    int prev = 0;
    for (int n = 0; n < S; ++n) {
        if (e[n] <= prev) return 0;
        prev = e[n];
    }
    return prev == L;
}

/* ------------------------------------------------------------------ */
/* Step 2+3: partition DP and backtrack, one candidate                  */
/* ------------------------------------------------------------------ */

/*
 * W[n][l] (n = xi-1 stages before the last one, first l layers) is the
 * paper's W(l, xi, 1, xi) divided by M:
 *   W(l, 1)  = sum_{i<=l} (p^f_i + p^b_i)
 *   W(l, xi) = min_{1 <= l' <= l-1} max{ W(l', xi-1),
 *                                        c^f + c^b at the cut after l',
 *                                        sum_{l' < i <= l} (p^f_i + p^b_i) }
 * with W = INF when l < xi (no feasible split).  The update is strict
 * (replace only if the stored value is larger), l' ascending, so the lowest
 * minimising l' is kept.  Wbuf: S*(L+1) int64, argbuf: S*(L+1) int32.
 */
static void dp_one(int L, int D, int S, const int64_t *PF, const int64_t *PB,
                   const int64_t *XF, const int64_t *XB, const int32_t *o,
                   int64_t *Wbuf, int32_t *argbuf, int64_t *C, int32_t *bounds) {
    const int W1 = L + 1;
    for (int n = 0; n < S; ++n)
        for (int l = 0; l <= L; ++l) {
            Wbuf[n * W1 + l] = INF;
            argbuf[n * W1 + l] = 0;
        }
    for (int l = 1; l <= L; ++l) Wbuf[l] = PF[l] + PB[l];

    for (int xi = 2; xi <= S; ++xi) {
        const int n = xi - 1;
        const size_t link = ((size_t)o[n - 1] * D + o[n]) * L;
        for (int l = xi; l <= L; ++l) {
            int64_t min_max_time = INF;
            int32_t best_lp = 0;
            for (int lp = 1; lp <= l - 1; ++lp) {
                int64_t sub = Wbuf[(n - 1) * W1 + lp];
                int64_t comm = XF[link + lp - 1] + XB[link + lp - 1];
                int64_t last = (PF[l] + PB[l]) - (PF[lp] + PB[lp]);
                int64_t max_time = max2(sub, max2(comm, last));
                if (min_max_time > max_time) {
                    min_max_time = max_time;
                    best_lp = lp;
                }
            }
            Wbuf[n * W1 + l] = min_max_time;
            argbuf[n * W1 + l] = best_lp;
        }
    }
    *C = Wbuf[(S - 1) * W1 + L];
    int e = L;
    for (int n = S - 1; n >= 0; --n) {
        bounds[n] = e;
        e = argbuf[n * W1 + e];
    }
}

int ppo_partition_dp(int L, int D, int S, int64_t N, const int64_t *PF,
                     const int64_t *PB, const int64_t *XF, const int64_t *XB,
                     const int32_t *orderings, int64_t *C_out,
                     int32_t *bounds_out) {
    int rc = check_common(L, D, S, N, orderings);
    if (rc) return rc;
    if (!PF || !PB || !XF || !XB || !C_out || !bounds_out)
        return PPO_ERR_INVALID_ARG;
    int32_t *own = NULL;
    if (!orderings) {
        own = all_orderings(D, N);
        if (!own) return PPO_ERR_NOMEM;
        orderings = own;
    }
    int fault = 0, nomem = 0;
    int nt = ppo_get_num_threads();
    (void)nt;
#pragma omp parallel num_threads(nt) reduction(| : fault, nomem)
    {
        int64_t *Wbuf = (int64_t *)malloc((size_t)S * (L + 1) * sizeof(int64_t));
        int32_t *argbuf = (int32_t *)malloc((size_t)S * (L + 1) * sizeof(int32_t));
        if (!Wbuf || !argbuf) nomem = 1;
#pragma omp for schedule(static)
        for (int64_t c = 0; c < N; ++c) {
            if (nomem) continue;
            const int32_t *o = orderings + c * S;
            if (!ordering_ok(o, S, D)) {
                fault |= PPO_FAULT_ORDERING;
                C_out[c] = INF;
                for (int n = 0; n < S; ++n) bounds_out[c * S + n] = 0;
                continue;
            }
            dp_one(L, D, S, PF, PB, XF, XB, o, Wbuf, argbuf, &C_out[c],
                   bounds_out + c * S);
        }
        free(Wbuf);
        free(argbuf);
    }
    free(own);
    if (nomem) return PPO_ERR_NOMEM;
    return fault;
}

/* ------------------------------------------------------------------ */
/* Step 4: PE scheduler (Alg. 1)                                        */
/* ------------------------------------------------------------------ */

/*
 * Resources in pipeline order, r = 1..R, R = 2S-1: odd r = stage (r-1)/2,
 * even r = the channel between stages r/2-1 and r/2 (one serial resource
 * for both directions: C and W charge a channel c^f + c^b).
 * Blocks j = 1..J, J = 4S-3 = 2R-1, in dependency order: j < R forward on
 * resource j; j == R the merged forward+backward of the last stage; j > R
 * backward on resource 2R-j.
 */
static int block_resource(int j, int R) { return j <= R ? j : 2 * R - j; }

/*
 * Execution ordering (first loop of Alg. 1).  One sweep over the block list
 * moves at most one microbatch per block; which queues are non-empty is
 * looked up at the start of the sweep, so a microbatch advances one block
 * per sweep (the paper's cycle example: in the second cycle only F of
 * microbatch 2 and the forward transfer of microbatch 1 run).  U[r] receives
 * the (microbatch, block) pairs of resource r in the order they are drawn;
 * channels follow the same list order as stages.
 * Returns the number of sweeps.  handled, if not NULL, gets per sweep the
 * microbatch handled by each block (0 = none), capacity max_rounds sweeps.
 */
typedef struct {
    int32_t m, j;
} pe_item;

static int pe_order(int S, int M, pe_item **U, int *Ulen, int32_t *handled,
                    int max_rounds) {
    const int R = 2 * S - 1, J = 2 * R - 1;
    /* Q[j] holds microbatch ids; each queue sees every microbatch once */
    int32_t *Q = (int32_t *)malloc((size_t)(J + 2) * M * sizeof(int32_t));
    int *head = (int *)calloc((size_t)J + 2, sizeof(int));
    int *tail = (int *)calloc((size_t)J + 2, sizeof(int));
    char *nonempty = (char *)malloc((size_t)J + 2);
    if (!Q || !head || !tail || !nonempty) {
        free(Q); free(head); free(tail); free(nonempty);
        return PPO_ERR_NOMEM;
    }
    for (int m = 1; m <= M; ++m) Q[1 * M + tail[1]++] = m;
    for (int r = 1; r <= R; ++r) Ulen[r] = 0;

    int rounds = 0;
    for (;;) {
        int any = 0;
        for (int j = 1; j <= J; ++j) {
            nonempty[j] = head[j] < tail[j];
            any |= nonempty[j];
        }
        if (!any) break;
        for (int j = 1; j <= J; ++j) {
            int32_t got = 0;
            if (nonempty[j]) {
                int32_t m = Q[j * M + head[j]++];
                if (j < J) Q[(j + 1) * M + tail[j + 1]++] = m;
                int r = block_resource(j, R);
                U[r][Ulen[r]].m = m;
                U[r][Ulen[r]].j = j;
                Ulen[r]++;
                got = m;
            }
            if (handled && rounds < max_rounds) handled[(size_t)rounds * J + j - 1] = got;
        }
        ++rounds;
    }
    free(Q); free(head); free(tail); free(nonempty);
    return rounds;
}

int ppo_execution_order(int S, int M, int32_t *rounds_out, int max_rounds) {
    if (S < 1 || S > PPO_MAX_STAGES || M < 1 || !rounds_out || max_rounds < 1)
        return PPO_ERR_INVALID_ARG;
    const int R = 2 * S - 1;
    pe_item **U = (pe_item **)calloc((size_t)R + 1, sizeof(pe_item *));
    int *Ulen = (int *)calloc((size_t)R + 1, sizeof(int));
    if (!U || !Ulen) { free(U); free(Ulen); return PPO_ERR_NOMEM; }
    int ok = 1;
    for (int r = 1; r <= R; ++r) {
        U[r] = (pe_item *)malloc((size_t)2 * M * sizeof(pe_item));
        if (!U[r]) ok = 0;
    }
    int rounds = ok ? pe_order(S, M, U, Ulen, rounds_out, max_rounds) : PPO_ERR_NOMEM;
    for (int r = 1; r <= R; ++r) free(U[r]);
    free(U);
    free(Ulen);
    return rounds;
}

/*
 * Scheduling (second loop of Alg. 1): every resource works through its list
 * U[r] in order and starts the head item as soon as its microbatch has left
 * the preceding block and the resource is idle; e^f of microbatch 1 on stage
 * 1 is 0.  Returns max_m (e^b_{m,s_1} + backward time of stage 1), the first
 * term of the makespan objective (nothing is replicated, so there is no
 * AllReduce term).
 */
int64_t ppo_pe_makespan(int S, int M, const int64_t *F, const int64_t *B,
                        const int64_t *cf, const int64_t *cb,
                        int64_t *start_out, int64_t *finish_out) {
    if (S < 1 || S > PPO_MAX_STAGES || M < 1 || !F || !B) return -1;
    if (S > 1 && (!cf || !cb)) return -1;
    const int R = 2 * S - 1, J = 2 * R - 1;
    int64_t *dur = (int64_t *)malloc((size_t)(J + 1) * sizeof(int64_t));
    int64_t *done = (int64_t *)malloc((size_t)(J + 1) * (M + 1) * sizeof(int64_t));
    int64_t *idle_at = (int64_t *)calloc((size_t)R + 1, sizeof(int64_t));
    int *next = (int *)calloc((size_t)R + 1, sizeof(int));
    int *Ulen = (int *)calloc((size_t)R + 1, sizeof(int));
    pe_item **U = (pe_item **)calloc((size_t)R + 1, sizeof(pe_item *));
    int64_t T = -1;
    if (!dur || !done || !idle_at || !next || !Ulen || !U) goto out;
    for (int r = 1; r <= R; ++r) {
        U[r] = (pe_item *)malloc((size_t)2 * M * sizeof(pe_item));
        if (!U[r]) goto out;
    }
    /* block durations */
    for (int j = 1; j <= J; ++j) {
        int r = block_resource(j, R);
        int is_stage = r & 1;
        int n = is_stage ? (r - 1) / 2 : r / 2; /* stage index or channel index */
        if (j == R)
            dur[j] = F[S - 1] + B[S - 1];
        else if (j < R)
            dur[j] = is_stage ? F[n] : cf[n];
        else
            dur[j] = is_stage ? B[n] : cb[n];
    }
    if (pe_order(S, M, U, Ulen, NULL, 0) < 0) goto out;

    for (size_t i = 0; i < (size_t)(J + 1) * (M + 1); ++i) done[i] = -1;
    for (;;) {
        int progress = 0, remaining = 0;
        for (int r = 1; r <= R; ++r) {
            while (next[r] < Ulen[r]) {
                pe_item it = U[r][next[r]];
                int64_t ready = 0;
                if (it.j > 1) {
                    ready = done[(size_t)(it.j - 1) * (M + 1) + it.m];
                    if (ready < 0) break; /* predecessor block not finished */
                }
                int64_t start = max2(idle_at[r], ready);
                int64_t fin = start + dur[it.j];
                done[(size_t)it.j * (M + 1) + it.m] = fin;
                idle_at[r] = fin;
                if (start_out) start_out[(size_t)(it.j - 1) * M + it.m - 1] = start;
                if (finish_out) finish_out[(size_t)(it.j - 1) * M + it.m - 1] = fin;
                next[r]++;
                progress = 1;
            }
            remaining |= next[r] < Ulen[r];
        }
        if (!remaining) break;
        if (!progress) goto out; /* cannot happen: the lists are consistent */
    }
    T = 0;
    for (int m = 1; m <= M; ++m) T = max2(T, done[(size_t)J * (M + 1) + m]);
out:
    if (U)
        for (int r = 1; r <= R; ++r) free(U[r]);
    free(U); free(Ulen); free(next); free(idle_at); free(done); free(dur);
    return T;
}

/* durations of one plan from the tables; returns fault bits */
static int plan_durations(int L, int D, int S, int M, const int64_t *PF,
                          const int64_t *PB, const int64_t *XF, const int64_t *XB,
                          const int32_t *o, const int32_t *e, int64_t *F,
                          int64_t *B, int64_t *cf, int64_t *cb) {
    int64_t worst = 0;
    for (int n = 0; n < S; ++n) {
        int lo = n ? e[n - 1] : 0, hi = e[n];
        F[n] = PF[hi] - PF[lo];
        B[n] = PB[hi] - PB[lo];
        worst = max2(worst, F[n] + B[n]);
        cf[n] = cb[n] = 0;
        if (n) {
            size_t at = ((size_t)o[n - 1] * D + o[n]) * L + (size_t)(lo - 1);
            cf[n] = XF[at];
            cb[n] = XB[at];
            worst = max2(worst, cf[n] + cb[n]);
        }
    }
    /* the schedule is no longer than (M + 4S - 4) * C (Lemma 1) */
    if (worst > (CAP - 1) / ((int64_t)M + 4 * S - 4)) return PPO_FAULT_OVERFLOW;
    return 0;
}

int ppo_schedule_makespan(int L, int D, int S, int64_t N, int M,
                          const int64_t *PF, const int64_t *PB,
                          const int64_t *XF, const int64_t *XB,
                          const int32_t *orderings, const int32_t *bounds,
                          int64_t *T_out) {
    int rc = check_common(L, D, S, N, orderings);
    if (rc) return rc;
    if (M < 1 || !PF || !PB || !XF || !XB || !bounds || !T_out)
        return PPO_ERR_INVALID_ARG;
    int32_t *own = NULL;
    if (!orderings) {
        own = all_orderings(D, N);
        if (!own) return PPO_ERR_NOMEM;
        orderings = own;
    }
    int fault = 0, nomem = 0;
    int nt = ppo_get_num_threads();
    (void)nt;
#pragma omp parallel for schedule(static) num_threads(nt) reduction(| : fault, nomem)
    for (int64_t c = 0; c < N; ++c) {
        const int32_t *o = orderings + c * S, *e = bounds + c * S;
        int64_t F[PPO_MAX_STAGES], B[PPO_MAX_STAGES], cf[PPO_MAX_STAGES],
            cb[PPO_MAX_STAGES];
        T_out[c] = INF;
        if (!ordering_ok(o, S, D)) { fault |= PPO_FAULT_ORDERING; continue; }
        if (!bounds_ok(e, S, L)) { fault |= PPO_FAULT_BOUNDS; continue; }
        int f = plan_durations(L, D, S, M, PF, PB, XF, XB, o, e, F, B, cf, cb);
        if (f) { fault |= f; continue; }
        int64_t T = ppo_pe_makespan(S, M, F, B, cf, cb, NULL, NULL);
        if (T < 0) { nomem = 1; continue; }
        T_out[c] = T;
    }
    free(own);
    if (nomem) return PPO_ERR_NOMEM;
    return fault;
}

/* ------------------------------------------------------------------ */
/* Step 5: keep the candidate with the smallest makespan                */
/* ------------------------------------------------------------------ */

int ppo_best_plan(int L, int D, int S, int64_t N, int M, const int64_t *PF,
                  const int64_t *PB, const int64_t *XF, const int64_t *XB,
                  const int32_t *orderings, ppo_result *out, int64_t *T_all,
                  int64_t *C_all) {
    int rc = check_common(L, D, S, N, orderings);
    if (rc) return rc;
    if (M < 1 || !PF || !PB || !XF || !XB || !out) return PPO_ERR_INVALID_ARG;
    int32_t *own = NULL;
    if (!orderings) {
        own = all_orderings(D, N);
        if (!own) return PPO_ERR_NOMEM;
        orderings = own;
    }
    int64_t *T = (int64_t *)malloc((size_t)N * sizeof(int64_t));
    int64_t *C = (int64_t *)malloc((size_t)N * sizeof(int64_t));
    int32_t *bounds = (int32_t *)malloc((size_t)N * S * sizeof(int32_t));
    int fault = PPO_ERR_NOMEM;
    if (T && C && bounds) {
        fault = ppo_partition_dp(L, D, S, N, PF, PB, XF, XB, orderings, C, bounds);
        if (fault == 0)
            fault = ppo_schedule_makespan(L, D, S, N, M, PF, PB, XF, XB,
                                          orderings, bounds, T);
    }
    if (fault == 0) {
        /* T_SPP <- T_PE only if T_PE < T_SPP, candidates in index order */
        int64_t T_best = INF, best = -1;
        for (int64_t c = 0; c < N; ++c)
            if (T[c] < T_best) {
                T_best = T[c];
                best = c;
            }
        memset(out, 0, sizeof(*out));
        out->best_index = best;
        out->S = S;
        out->T = T_best;
        out->C = best >= 0 ? C[best] : INF;
        for (int n = 0; n < S && best >= 0; ++n) {
            out->bounds[n] = bounds[best * S + n];
            out->order[n] = orderings[best * S + n];
        }
        if (T_all) memcpy(T_all, T, (size_t)N * sizeof(int64_t));
        if (C_all) memcpy(C_all, C, (size_t)N * sizeof(int64_t));
    }
    free(T); free(C); free(bounds); free(own);
    return fault;
}

/* ------------------------------------------------------------------ */
/* Stage-count search (outer loop of Alg. 3)                            */
/* ------------------------------------------------------------------ */

int ppo_best_plan_stages(int L, int D, int S, int64_t N, int M, const int64_t *PF,
                         const int64_t *PB, const int64_t *XF, const int64_t *XB,
                         const int32_t *orderings, ppo_result *out, int64_t *T_all,
                         int64_t *C_all, int32_t *bounds_all) {
    int rc = check_common(L, D, S, N, orderings);
    if (rc) return rc;
    if (M < 1 || !PF || !PB || !XF || !XB || !out) return PPO_ERR_INVALID_ARG;
    int32_t *own = NULL;
    if (!orderings) {
        own = all_orderings(D, N);
        if (!own) return PPO_ERR_NOMEM;
        orderings = own;
    }
    const int tri = S * (S + 1) / 2;
    int64_t *T = (int64_t *)malloc((size_t)N * S * sizeof(int64_t));
    int64_t *C = (int64_t *)malloc((size_t)N * S * sizeof(int64_t));
    int32_t *bounds = (int32_t *)malloc((size_t)N * tri * sizeof(int32_t));
    int32_t *pre = (int32_t *)malloc((size_t)N * S * sizeof(int32_t));
    int32_t *bxi = (int32_t *)malloc((size_t)N * S * sizeof(int32_t));
    int64_t *Txi = (int64_t *)malloc((size_t)N * sizeof(int64_t));
    int64_t *Cxi = (int64_t *)malloc((size_t)N * sizeof(int64_t));
    int fault = (T && C && bounds && pre && bxi && Txi && Cxi) ? 0 : PPO_ERR_NOMEM;
    /* for every stage count xi: the plan (PRM) and its schedule (PE) on the first xi
     * devices of every candidate's ordering */
    for (int xi = 1; xi <= S && fault == 0; ++xi) {
        for (int64_t c = 0; c < N; ++c)
            for (int n = 0; n < xi; ++n) pre[c * xi + n] = orderings[c * S + n];
        fault = ppo_partition_dp(L, D, xi, N, PF, PB, XF, XB, pre, Cxi, bxi);
        if (fault == 0)
            fault = ppo_schedule_makespan(L, D, xi, N, M, PF, PB, XF, XB, pre, bxi, Txi);
        if (fault) break;
        for (int64_t c = 0; c < N; ++c) {
            T[c * S + xi - 1] = Txi[c];
            C[c * S + xi - 1] = Cxi[c];
            for (int n = 0; n < xi; ++n)
                bounds[c * tri + xi * (xi - 1) / 2 + n] = bxi[c * xi + n];
        }
    }
    if (fault == 0) {
        /* T_SPP <- T_PE only if T_PE < T_SPP: candidates in index order, and for each
         * candidate the stage counts in the listing's order 1, 2, ... */
        int64_t T_best = INF, best = -1;
        int xi_best = 0;
        for (int64_t c = 0; c < N; ++c)
            for (int xi = 1; xi <= S; ++xi)
                if (T[c * S + xi - 1] < T_best) {
                    T_best = T[c * S + xi - 1];
                    best = c;
                    xi_best = xi;
                }
        memset(out, 0, sizeof(*out));
        out->best_index = best;
        out->S = xi_best;
        out->T = T_best;
        out->C = best >= 0 ? C[best * S + xi_best - 1] : INF;
        for (int n = 0; n < xi_best && best >= 0; ++n) {
            out->bounds[n] = bounds[best * tri + xi_best * (xi_best - 1) / 2 + n];
            out->order[n] = orderings[best * S + n];
        }
        if (T_all) memcpy(T_all, T, (size_t)N * S * sizeof(int64_t));
        if (C_all) memcpy(C_all, C, (size_t)N * S * sizeof(int64_t));
        if (bounds_all) memcpy(bounds_all, bounds, (size_t)N * tri * sizeof(int32_t));
    }
    free(T); free(C); free(bounds); free(pre); free(bxi); free(Txi); free(Cxi); free(own);
    return fault;
}

/* ------------------------------------------------------------------ */
/* Recursive device ordering (Alg. 2)                                   */
/* ------------------------------------------------------------------ */

/* Stoer-Wagner minimum cut of the subgraph induced by verts[0..nv-1] (ascending device
 * indices).  side[i] = 1 marks the vertices of one side of the lightest cut found. */
static int min_cut(int D, const int64_t *bw, const int *verts, int nv, char *side) {
    int64_t *W = (int64_t *)malloc((size_t)nv * nv * sizeof(int64_t));
    int64_t *wsum = (int64_t *)malloc((size_t)nv * sizeof(int64_t));
    int *low = (int *)malloc((size_t)nv * sizeof(int));      /* lowest device index in the group */
    int *next = (int *)malloc((size_t)nv * sizeof(int));     /* member list of a merged vertex */
    int *tail = (int *)malloc((size_t)nv * sizeof(int));
    char *active = (char *)malloc((size_t)nv), *inA = (char *)malloc((size_t)nv);
    if (!W || !wsum || !low || !next || !tail || !active || !inA) {
        free(W); free(wsum); free(low); free(next); free(tail); free(active); free(inA);
        return PPO_ERR_NOMEM;
    }
    for (int i = 0; i < nv; ++i) {
        for (int j = 0; j < nv; ++j)
            W[(size_t)i * nv + j] = i == j ? 0 : bw[(size_t)verts[i] * D + verts[j]] + bw[(size_t)verts[j] * D + verts[i]];
        low[i] = verts[i]; next[i] = -1; tail[i] = i; active[i] = 1;
    }
    int64_t best = INF;
    for (int remaining = nv; remaining > 1; --remaining) {
        /* one phase: grow A from the lowest-index vertex by maximum adjacency */
        int start = -1;
        for (int i = 0; i < nv; ++i)
            if (active[i] && (start < 0 || low[i] < low[start])) start = i;
        for (int i = 0; i < nv; ++i) { inA[i] = 0; wsum[i] = W[(size_t)start * nv + i]; }
        inA[start] = 1;
        int s = start, t = start;
        for (int added = 1; added < remaining; ++added) {
            int pick = -1;
            for (int i = 0; i < nv; ++i) {
                if (!active[i] || inA[i]) continue;
                if (pick < 0 || wsum[i] > wsum[pick] || (wsum[i] == wsum[pick] && low[i] < low[pick])) pick = i;
            }
            inA[pick] = 1;
            s = t; t = pick;
            if (added + 1 < remaining)
                for (int i = 0; i < nv; ++i) wsum[i] += W[(size_t)pick * nv + i];
        }
        /* cut of the phase: the last vertex against the rest */
        if (wsum[t] < best) {
            best = wsum[t];
            for (int i = 0; i < nv; ++i) side[i] = 0;
            for (int i = t; i >= 0; i = next[i]) side[i] = 1;
        }
        /* merge t into s */
        for (int i = 0; i < nv; ++i) {
            W[(size_t)s * nv + i] += W[(size_t)t * nv + i];
            W[(size_t)i * nv + s] = W[(size_t)s * nv + i];
        }
        W[(size_t)s * nv + s] = 0;
        if (low[t] < low[s]) low[s] = low[t];
        next[tail[s]] = t; tail[s] = tail[t];
        active[t] = 0;
    }
    free(W); free(wsum); free(low); free(next); free(tail); free(active); free(inA);
    return PPO_OK;
}

static int rdo(int D, const int64_t *bw, const int *verts, int nv, int32_t *order, int rank_lo) {
    if (nv == 1) { order[rank_lo] = verts[0]; return PPO_OK; }
    char *side = (char *)malloc((size_t)nv);
    int *g1 = (int *)malloc((size_t)nv * sizeof(int)), *g2 = (int *)malloc((size_t)nv * sizeof(int));
    int rc = (side && g1 && g2) ? min_cut(D, bw, verts, nv, side) : PPO_ERR_NOMEM;
    if (rc == PPO_OK) {
        /* G1 = the side with the lowest device index (verts is ascending, so verts[0]) */
        int n1 = 0, n2 = 0;
        for (int i = 0; i < nv; ++i) {
            if (side[i] == side[0]) g1[n1++] = verts[i];
            else g2[n2++] = verts[i];
        }
        rc = rdo(D, bw, g1, n1, order, rank_lo);
        if (rc == PPO_OK) rc = rdo(D, bw, g2, n2, order, rank_lo + n1);
    }
    free(side); free(g1); free(g2);
    return rc;
}

int ppo_rdo_order(int D, const int64_t *bw, int32_t *order_out) {
    if (D < 1 || !bw || !order_out) return PPO_ERR_INVALID_ARG;
    for (int u = 0; u < D; ++u)
        for (int v = 0; v < D; ++v)
            if (u != v && bw[(size_t)u * D + v] < 0) return PPO_ERR_INVALID_ARG;
    int *verts = (int *)malloc((size_t)D * sizeof(int));
    if (!verts) return PPO_ERR_NOMEM;
    for (int i = 0; i < D; ++i) verts[i] = i;
    int rc = rdo(D, bw, verts, D, order_out, 0);
    free(verts);
    return rc;
}

/* ------------------------------------------------------------------ */
/* Partition, replication and mapping (PRM, Alg. 4) and the complete    */
/* planner (SPP, Alg. 3) with replicated stages                         */
/* ------------------------------------------------------------------ */

typedef struct {
    int L, D, M;
    const int64_t *PF, *PB, *PA;     /* prefix sums of p^f, p^b, alpha (length L+1) */
    const int64_t *actf, *actb, *bw; /* d^f, d^b per boundary; bandwidth matrix      */
    const int32_t *o;                /* device of rank 0..D-1                        */
    int64_t *memo;                   /* W(l, xi, r, n) or -1                         */
    int32_t *arg_l, *arg_r;          /* minimising (l', r')                          */
} prm_ctx;

static size_t prm_at(const prm_ctx *x, int l, int n, int xi, int r) {
    const size_t d1 = (size_t)x->D + 1;
    return (((size_t)l * d1 + n) * d1 + xi) * d1 + r;
}

/* min of b_{u,v} over u in ranks [a0,a1), v in ranks [b0,b1), u != v */
static int64_t min_bw(const prm_ctx *x, int a0, int a1, int b0, int b1) {
    int64_t m = INF;
    for (int u = a0; u < a1; ++u)
        for (int v = b0; v < b1; ++v)
            if (u != v) {
                int64_t b = x->bw[(size_t)x->o[u] * x->D + x->o[v]];
                if (b < m) m = b;
            }
    return m;
}

/* Eq. 1: ring AllReduce of layers [l0, l1) replicated over ranks [n-r, n) */
static int64_t allreduce_time(const prm_ctx *x, int l0, int l1, int r, int n) {
    if (r == 1) return 0;
    int64_t b = min_bw(x, n - r, n, n - r, n);
    return ceil_div(2 * (int64_t)(r - 1) * (x->PA[l1] - x->PA[l0]), (int64_t)r * b);
}

/* per-microbatch forward / backward time of layers [l0, l1) on r replicas: p / k */
static int64_t rep_fwd(const prm_ctx *x, int l0, int l1, int r) { return ceil_div(x->PF[l1] - x->PF[l0], r); }
static int64_t rep_bwd(const prm_ctx *x, int l0, int l1, int r) { return ceil_div(x->PB[l1] - x->PB[l0], r); }

/* c^f, c^b (Sec. III-B) across the boundary after layer lp-1: stage on ranks
 * [n-r-rp, n-r) with rp replicas feeds the stage on ranks [n-r, n) with r replicas */
static int64_t rep_cf(const prm_ctx *x, int lp, int rp, int r, int n) {
    int64_t b = min_bw(x, n - r - rp, n - r, n - r, n);
    return ceil_div(x->actf[lp - 1], (int64_t)rp * r * b);
}
static int64_t rep_cb(const prm_ctx *x, int lp, int rp, int r, int n) {
    int64_t b = min_bw(x, n - r, n, n - r - rp, n - r);
    return ceil_div(x->actb[lp - 1], (int64_t)rp * r * b);
}

/* W(l, xi, r, n): first l layers in xi stages on ranks 0..n-1, last stage on r replicas */
static int64_t prm(prm_ctx *x, int l, int n, int xi, int r) {
    if (l < xi || n < xi) return INF;
    size_t at = prm_at(x, l, n, xi, r);
    if (x->memo[at] >= 0) return x->memo[at];
    int64_t best = INF;
    int bl = 0, br = 0;
    if (xi == 1 && r == n) {
        best = x->M * (rep_fwd(x, 0, l, n) + rep_bwd(x, 0, l, n)) + allreduce_time(x, 0, l, n, n);
    } else if (xi == 1 || r == n) {
        best = INF;
    } else {
        for (int lp = 1; lp <= l - 1; ++lp)
            for (int rp = 1; rp <= n - r; ++rp) {
                int64_t w = prm(x, lp, n - r, xi - 1, rp);
                if (w == INF) continue; /* max{INF, ...} never improves */
                int64_t comm = x->M * (rep_cf(x, lp, rp, r, n) + rep_cb(x, lp, rp, r, n));
                int64_t last = x->M * (rep_fwd(x, lp, l, r) + rep_bwd(x, lp, l, r)) +
                               allreduce_time(x, lp, l, r, n);
                int64_t t = max2(w, max2(comm, last));
                if (best > t) {
                    best = t;
                    bl = lp;
                    br = rp;
                }
            }
    }
    x->memo[at] = best;
    x->arg_l[at] = bl;
    x->arg_r[at] = br;
    return best;
}

/* T of a plan with replicated stages: Alg. 1 on the stages' per-replica times, then Eq. 2:
 * an AllReduce starts when the stage's last backward pass has finished. */
static int64_t rep_makespan(const prm_ctx *x, int S, const int32_t *bounds, const int32_t *reps) {
    int64_t F[PPO_MAX_STAGES], B[PPO_MAX_STAGES], cf[PPO_MAX_STAGES], cb[PPO_MAX_STAGES];
    int64_t A[PPO_MAX_STAGES];
    int M = x->M, n = 0, l0 = 0;
    for (int s = 0; s < S; ++s) {
        int r = reps[s], l1 = bounds[s];
        n += r;
        F[s] = rep_fwd(x, l0, l1, r);
        B[s] = rep_bwd(x, l0, l1, r);
        A[s] = allreduce_time(x, l0, l1, r, n);
        cf[s] = cb[s] = 0;
        if (s) {
            cf[s] = rep_cf(x, l0, reps[s - 1], r, n);
            cb[s] = rep_cb(x, l0, reps[s - 1], r, n);
        }
        l0 = l1;
    }
    const int R = 2 * S - 1, J = 2 * R - 1;
    int64_t *fin = (int64_t *)malloc((size_t)J * M * sizeof(int64_t));
    if (!fin) return -1;
    int64_t T = ppo_pe_makespan(S, M, F, B, cf, cb, NULL, fin);
    for (int s = 0; s < S && T >= 0; ++s) {
        if (reps[s] == 1) continue;
        /* last backward block of stage s: block 2R - (2s+1), or the merged block R */
        int j = s == S - 1 ? R : 2 * R - (2 * s + 1);
        int64_t done = 0;
        for (int m = 0; m < M; ++m) done = max2(done, fin[(size_t)(j - 1) * M + m]);
        T = max2(T, done + A[s]);
    }
    free(fin);
    return T;
}

int ppo_spp_replicated(int L, int D, int64_t N, int M, const int64_t *fwd_us,
                       const int64_t *bwd_us, const int64_t *act_fwd_bytes,
                       const int64_t *act_bwd_bytes, const int64_t *alpha_bytes,
                       const int64_t *bw, const int32_t *orderings, ppo_rep_result *out,
                       int64_t *T_all, int64_t *W_all, int32_t *bounds_all, int32_t *reps_all) {
    if (L < 1 || D < 1 || D > PPO_MAX_STAGES || N < 1 || M < 1 || !fwd_us || !bwd_us ||
        !act_fwd_bytes || !alpha_bytes || !bw || !out)
        return PPO_ERR_INVALID_ARG;
    if (!act_bwd_bytes) act_bwd_bytes = act_fwd_bytes;
    if (!orderings && factorial_or_neg(D) != N) return PPO_ERR_INVALID_ARG;
    int fault = 0;
    for (int l = 0; l < L; ++l) {
        if (fwd_us[l] < 0 || bwd_us[l] < 0 || alpha_bytes[l] < 0) fault |= PPO_FAULT_NEGATIVE;
        if (l + 1 < L && (act_fwd_bytes[l] < 0 || act_bwd_bytes[l] < 0)) fault |= PPO_FAULT_NEGATIVE;
    }
    for (int u = 0; u < D; ++u)
        for (int v = 0; v < D; ++v)
            if (u != v && bw[(size_t)u * D + v] <= 0) fault |= PPO_FAULT_BANDWIDTH;
    int32_t *own = NULL;
    if (!orderings) {
        own = all_orderings(D, N);
        if (!own) return PPO_ERR_NOMEM;
        orderings = own;
    }
    for (int64_t c = 0; c < N && !fault; ++c)
        if (!ordering_ok(orderings + c * D, D, D)) fault |= PPO_FAULT_ORDERING;
    int64_t *PF = (int64_t *)calloc((size_t)L + 1, sizeof(int64_t));
    int64_t *PB = (int64_t *)calloc((size_t)L + 1, sizeof(int64_t));
    int64_t *PA = (int64_t *)calloc((size_t)L + 1, sizeof(int64_t));
    const int tri = D * (D + 1) / 2;
    int64_t *T = (int64_t *)malloc((size_t)N * D * sizeof(int64_t));
    int64_t *W = (int64_t *)malloc((size_t)N * D * sizeof(int64_t));
    int32_t *bd = (int32_t *)calloc((size_t)N * tri, sizeof(int32_t));
    int32_t *rp = (int32_t *)calloc((size_t)N * tri, sizeof(int32_t));
    if (!PF || !PB || !PA || !T || !W || !bd || !rp) fault = PPO_ERR_NOMEM;
    if (fault == 0) {
        for (int l = 0; l < L; ++l) {
            PF[l + 1] = PF[l] + fwd_us[l];
            PB[l + 1] = PB[l] + bwd_us[l];
            PA[l + 1] = PA[l] + alpha_bytes[l];
            /* M * (time) and 2 (r-1) * (parameter bytes) must stay far from 2^63 */
            if (PF[l + 1] + PB[l + 1] >= CAP / ((int64_t)M + 4 * D) || PA[l + 1] >= CAP / (2 * D))
                fault |= PPO_FAULT_OVERFLOW;
        }
    }
    int nomem = 0;
    if (fault == 0) {
        const size_t states = ((size_t)L + 1) * (D + 1) * (D + 1) * (D + 1);
#pragma omp parallel for schedule(dynamic, 1) num_threads(ppo_get_num_threads())
        for (int64_t c = 0; c < N; ++c) {
            prm_ctx x = {L, D, M, PF, PB, PA, act_fwd_bytes, act_bwd_bytes, bw, orderings + c * D,
                         NULL, NULL, NULL};
            x.memo = (int64_t *)malloc(states * sizeof(int64_t));
            x.arg_l = (int32_t *)malloc(states * sizeof(int32_t));
            x.arg_r = (int32_t *)malloc(states * sizeof(int32_t));
            if (!x.memo || !x.arg_l || !x.arg_r) {
                nomem = 1;
            } else {
                for (size_t i = 0; i < states; ++i) x.memo[i] = -1;
                /* Alg. 3: for every stage count, the replication of the last stage with the
                 * smallest W (first such r), its plan, and the plan's schedule */
                for (int xi = 1; xi <= D; ++xi) {
                    int64_t wbest = INF;
                    int rbest = 0;
                    for (int r = 1; r <= D; ++r) {
                        int64_t w = prm(&x, L, D, xi, r);
                        if (w < wbest) {
                            wbest = w;
                            rbest = r;
                        }
                    }
                    W[c * D + xi - 1] = wbest;
                    T[c * D + xi - 1] = INF;
                    if (wbest == INF) continue;
                    int32_t *b = bd + c * tri + xi * (xi - 1) / 2;
                    int32_t *k = rp + c * tri + xi * (xi - 1) / 2;
                    int l = L, n = D, r = rbest;
                    for (int s = xi - 1; s >= 0; --s) {
                        b[s] = l;
                        k[s] = r;
                        size_t at = prm_at(&x, l, n, s + 1, r);
                        int lp = x.arg_l[at], rq = x.arg_r[at];
                        n -= r;
                        l = lp;
                        r = rq;
                    }
                    int64_t t = rep_makespan(&x, xi, b, k);
                    if (t < 0) nomem = 1;
                    else T[c * D + xi - 1] = t;
                }
            }
            free(x.memo); free(x.arg_l); free(x.arg_r);
        }
        if (nomem) fault = PPO_ERR_NOMEM;
    }
    if (fault == 0) {
        /* keep-the-minimum with strict '<': candidates in index order, stage counts 1, 2, ... */
        int64_t T_best = INF, best = -1;
        int xi_best = 0;
        for (int64_t c = 0; c < N; ++c)
            for (int xi = 1; xi <= D; ++xi)
                if (T[c * D + xi - 1] < T_best) {
                    T_best = T[c * D + xi - 1];
                    best = c;
                    xi_best = xi;
                }
        memset(out, 0, sizeof(*out));
        out->best_index = best;
        out->T = T_best;
        out->S = xi_best;
        out->W = best >= 0 ? W[best * D + xi_best - 1] : INF;
        for (int n = 0; n < D && best >= 0; ++n) out->order[n] = orderings[best * D + n];
        for (int s = 0; s < xi_best && best >= 0; ++s) {
            out->bounds[s] = bd[best * tri + xi_best * (xi_best - 1) / 2 + s];
            out->reps[s] = rp[best * tri + xi_best * (xi_best - 1) / 2 + s];
        }
        if (T_all) memcpy(T_all, T, (size_t)N * D * sizeof(int64_t));
        if (W_all) memcpy(W_all, W, (size_t)N * D * sizeof(int64_t));
        if (bounds_all) memcpy(bounds_all, bd, (size_t)N * tri * sizeof(int32_t));
        if (reps_all) memcpy(reps_all, rp, (size_t)N * tri * sizeof(int32_t));
    }
    free(PF); free(PB); free(PA); free(T); free(W); free(bd); free(rp); free(own);
    return fault;
}

/* ------------------------------------------------------------------ */
/* Schedule variants (for comparison with the PE scheduler)             */
/* ------------------------------------------------------------------ */

/*
 * Alg. 1 with channels that serve by readiness (Sec. IV-A, scheduling phase: "the successor
 * communication block is immediately run upon the channel becoming idle"; only computation
 * blocks are entered into the lists U_s).  Blocks j = 1..J = 4S-3 on resources
 * r(j) = min(j, 2R - j), R = 2S-1, odd resources are stages.  Every block handles the
 * microbatches in index order (stages by their lists, a channel's two directions each first
 * come first served), so nxt[j] is the next microbatch of block j.
 *   stage r:   next item = the earlier of (nxt[r], r) and (nxt[2R-r], 2R-r) in the order of
 *              the first phase (sweep m + j - 1, then block); it can start once its microbatch
 *              has left the preceding block;
 *   channel r: of the (at most two) head items whose microbatch has left the preceding
 *              block, the one that left it first; equal times: earlier in the first phase's
 *              order.
 * The item with the earliest start max(ready, resource idle) over all resources is committed
 * next (equal starts: lowest resource), until all J M items are done.
 */
static int64_t fifo_makespan(int S, int M, const int64_t *F, const int64_t *B,
                             const int64_t *cf, const int64_t *cb) {
    const int R = 2 * S - 1, J = 2 * R - 1;
    int64_t *dur = (int64_t *)malloc((size_t)(J + 1) * sizeof(int64_t));
    int64_t *done = (int64_t *)malloc((size_t)(J + 1) * (M + 1) * sizeof(int64_t));
    int64_t *idle = (int64_t *)calloc((size_t)R + 1, sizeof(int64_t));
    int *nxt = (int *)malloc((size_t)(J + 1) * sizeof(int));
    int64_t T = -1;
    if (!dur || !done || !idle || !nxt) goto out;
    for (int n = 0; n < S; ++n) {
        const int r = 2 * n + 1;
        if (n == S - 1) dur[R] = F[n] + B[n];
        else { dur[r] = F[n]; dur[2 * R - r] = B[n]; }
        if (n) { dur[r - 1] = cf[n]; dur[2 * R - (r - 1)] = cb[n]; }
    }
    for (int j = 1; j <= J; ++j) nxt[j] = 1;
    for (size_t i = 0; i < (size_t)(J + 1) * (M + 1); ++i) done[i] = -1;
#define DONE(j, m) done[(size_t)(j) * (M + 1) + (m)]
    for (long long left = (long long)J * M; left > 0; --left) {
        int best_r = 0, best_j = 0;
        int64_t best_start = 0;
        for (int r = 1; r <= R; ++r) {
            const int ja = r, jb = 2 * R - r;
            int j = 0;
            int64_t ready = 0;
            if (r & 1) {
                /* the stage's list */
                int pick = 0;
                const int has_a = nxt[ja] <= M, has_b = jb != ja && nxt[jb] <= M;
                if (has_a && (!has_b || nxt[ja] + ja <= nxt[jb] + jb)) pick = ja;
                else if (has_b) pick = jb;
                if (!pick) continue;
                if (pick > 1 && DONE(pick - 1, nxt[pick]) < 0) continue;
                j = pick;
                ready = pick > 1 ? DONE(pick - 1, nxt[pick]) : 0;
            } else {
                /* the channel's waiting heads */
                for (int k = 0; k < 2; ++k) {
                    const int jj = k ? jb : ja;
                    if (nxt[jj] > M) continue;
                    const int64_t rd = DONE(jj - 1, nxt[jj]);
                    if (rd < 0) continue;
                    if (!j || rd < ready ||
                        (rd == ready && (nxt[jj] + jj < nxt[j] + j ||
                                         (nxt[jj] + jj == nxt[j] + j && jj < j)))) {
                        j = jj;
                        ready = rd;
                    }
                }
                if (!j) continue;
            }
            const int64_t start = max2(ready, idle[r]);
            if (!best_r || start < best_start) { best_r = r; best_j = j; best_start = start; }
        }
        if (!best_r) goto out; /* cannot happen: block 1 or a successor is always available */
        const int64_t fin = best_start + dur[best_j];
        DONE(best_j, nxt[best_j]) = fin;
        idle[best_r] = fin;
        nxt[best_j]++;
    }
    T = 0;
    for (int m = 1; m <= M; ++m) T = max2(T, DONE(J, m));
#undef DONE
out:
    free(dur); free(done); free(idle); free(nxt);
    return T;
}

/*
 * A schedule variant is a block list per microbatch, a resource per block and a service
 * order per resource; the timing rule is the scheduling phase of Alg. 1 in every case (an
 * item starts when its microbatch has left the preceding block and the resource is idle).
 *   PPO_SCHED_PE      the PE scheduler itself (same result as ppo_pe_makespan)
 *   PPO_SCHED_DUPLEX  PE's blocks and ordering phase, but the forward and the backward
 *                     transfers of a stage pair run on separate channels
 *   PPO_SCHED_GPIPE   every stage and channel serves all its forward items (microbatch
 *                     order) before any backward item: "all FP before any BP" (Sec. II).
 *                     The last stage's forward and backward are separate blocks here.
 *   PPO_SCHED_ADDITIVE  stages are the only resources; the transfers into a stage (forward
 *                     activations in, backward gradients out over the same link) are added
 *                     to that stage's forward and backward blocks.  2S-1 blocks per
 *                     microbatch, PE's ordering phase on that list.
 *   PPO_SCHED_FIFO    channels serve by readiness instead of by list: fifo_makespan above.
 */
int64_t ppo_variant_makespan(int variant, int S, int M, const int64_t *F, const int64_t *B,
                             const int64_t *cf, const int64_t *cb) {
    if (S < 1 || S > PPO_MAX_STAGES || M < 1 || !F || !B || (S > 1 && (!cf || !cb))) return -1;
    if (variant == PPO_SCHED_FIFO) return fifo_makespan(S, M, F, B, cf, cb);
    if (variant != PPO_SCHED_PE && variant != PPO_SCHED_DUPLEX && variant != PPO_SCHED_GPIPE &&
        variant != PPO_SCHED_ADDITIVE) return -1;
    const int merged = variant != PPO_SCHED_GPIPE;       /* last stage: one block or two */
    const int folded = variant == PPO_SCHED_ADDITIVE;    /* transfers inside the stage blocks */
    const int J = folded ? 2 * S - 1 : merged ? 4 * S - 3 : 4 * S - 2;  /* blocks per microbatch */
    const int nres = 3 * S;                                 /* stages, fwd channels, bwd channels */
    int *res = (int *)malloc((size_t)(J + 1) * sizeof(int));
    int *is_fwd = (int *)malloc((size_t)(J + 1) * sizeof(int));
    int64_t *dur = (int64_t *)malloc((size_t)(J + 1) * sizeof(int64_t));
    int64_t *done = (int64_t *)malloc((size_t)(J + 1) * (M + 1) * sizeof(int64_t));
    int64_t *idle_at = (int64_t *)calloc((size_t)nres, sizeof(int64_t));
    int *next = (int *)calloc((size_t)nres, sizeof(int));
    int *Ulen = (int *)calloc((size_t)nres, sizeof(int));
    pe_item *Uall = (pe_item *)malloc((size_t)nres * 2 * M * sizeof(pe_item));
    int32_t *Q = (int32_t *)malloc((size_t)(J + 2) * M * sizeof(int32_t));
    int *head = (int *)calloc((size_t)J + 2, sizeof(int));
    int *tail = (int *)calloc((size_t)J + 2, sizeof(int));
    char *nonempty = (char *)malloc((size_t)J + 2);
    int64_t T = -1;
    if (!res || !is_fwd || !dur || !done || !idle_at || !next || !Ulen || !Uall || !Q || !head || !tail || !nonempty)
        goto out;

    /* the blocks a microbatch passes, in order: forward through the stages and channels,
     * then backward; resources: stage n = n, forward channel n = S + n, backward channel
     * n = 2S + n (or S + n as well when both directions share the channel) */
    if (folded) {
        int j = 0;
        for (int n = 0; n < S; ++n) {
            ++j; res[j] = n; is_fwd[j] = 1;
            dur[j] = F[n] + (n ? cf[n] : 0);
            if (n == S - 1) dur[j] += B[n] + (n ? cb[n] : 0);
        }
        for (int n = S - 2; n >= 0; --n) {
            ++j; res[j] = n; is_fwd[j] = 0;
            dur[j] = B[n] + (n ? cb[n] : 0);
        }
        if (j != J) goto out;
    } else {
        int j = 0;
        for (int n = 0; n < S; ++n) {
            if (n) { ++j; res[j] = S + n; dur[j] = cf[n]; is_fwd[j] = 1; }
            ++j; res[j] = n; is_fwd[j] = 1;
            dur[j] = (n == S - 1 && merged) ? F[n] + B[n] : F[n];
        }
        for (int n = S - 1; n >= 0; --n) {
            if (!(n == S - 1 && merged)) { ++j; res[j] = n; dur[j] = B[n]; is_fwd[j] = 0; }
            if (n) {
                ++j; dur[j] = cb[n]; is_fwd[j] = 0;
                res[j] = variant == PPO_SCHED_DUPLEX ? 2 * S + n : S + n;
            }
        }
        if (j != J) goto out;
    }
#define ULIST(r) (Uall + (size_t)(r) * 2 * M)
    if (variant == PPO_SCHED_GPIPE) {
        /* all forward items of a resource in microbatch order, then all backward items */
        for (int pass = 1; pass >= 0; --pass)
            for (int j = 1; j <= J; ++j)
                if (is_fwd[j] == pass)
                    for (int m = 1; m <= M; ++m) {
                        pe_item it = {m, j};
                        ULIST(res[j])[Ulen[res[j]]++] = it;
                    }
    } else {
        /* ordering phase of Alg. 1: sweeps over the block list, one microbatch per non-empty
         * queue (looked up at the start of the sweep) moves on by one block */
        for (int m = 1; m <= M; ++m) Q[1 * M + tail[1]++] = m;
        for (;;) {
            int any = 0;
            for (int j = 1; j <= J; ++j) { nonempty[j] = head[j] < tail[j]; any |= nonempty[j]; }
            if (!any) break;
            for (int j = 1; j <= J; ++j)
                if (nonempty[j]) {
                    int32_t m = Q[j * M + head[j]++];
                    if (j < J) Q[(j + 1) * M + tail[j + 1]++] = m;
                    pe_item it = {m, j};
                    ULIST(res[j])[Ulen[res[j]]++] = it;
                }
        }
    }
    /* scheduling phase */
    for (size_t i = 0; i < (size_t)(J + 1) * (M + 1); ++i) done[i] = -1;
    for (;;) {
        int progress = 0, remaining = 0;
        for (int r = 0; r < nres; ++r) {
            while (next[r] < Ulen[r]) {
                pe_item it = ULIST(r)[next[r]];
                int64_t ready = 0;
                if (it.j > 1) {
                    ready = done[(size_t)(it.j - 1) * (M + 1) + it.m];
                    if (ready < 0) break;
                }
                int64_t fin = max2(idle_at[r], ready) + dur[it.j];
                done[(size_t)it.j * (M + 1) + it.m] = fin;
                idle_at[r] = fin;
                next[r]++;
                progress = 1;
            }
            remaining |= next[r] < Ulen[r];
        }
        if (!remaining) break;
        if (!progress) goto out;
    }
#undef ULIST
    T = 0;
    for (int m = 1; m <= M; ++m) T = max2(T, done[(size_t)J * (M + 1) + m]);
out:
    free(res); free(is_fwd); free(dur); free(done); free(idle_at); free(next); free(Ulen); free(Uall);
    free(Q); free(head); free(tail); free(nonempty);
    return T;
}

int ppo_schedule_makespan_variant(int variant, int L, int D, int S, int64_t N, int M,
                                  const int64_t *PF, const int64_t *PB, const int64_t *XF,
                                  const int64_t *XB, const int32_t *orderings,
                                  const int32_t *bounds, int64_t *T_out) {
    int rc = check_common(L, D, S, N, orderings);
    if (rc) return rc;
    if (M < 1 || !PF || !PB || !XF || !XB || !bounds || !T_out) return PPO_ERR_INVALID_ARG;
    if (variant != PPO_SCHED_PE && variant != PPO_SCHED_DUPLEX && variant != PPO_SCHED_GPIPE &&
        variant != PPO_SCHED_ADDITIVE && variant != PPO_SCHED_FIFO)
        return PPO_ERR_INVALID_ARG;
    int32_t *own = NULL;
    if (!orderings) {
        own = all_orderings(D, N);
        if (!own) return PPO_ERR_NOMEM;
        orderings = own;
    }
    int fault = 0, nomem = 0;
    int nt = ppo_get_num_threads();
    (void)nt;
#pragma omp parallel for schedule(static) num_threads(nt) reduction(| : fault, nomem)
    for (int64_t c = 0; c < N; ++c) {
        const int32_t *o = orderings + c * S, *e = bounds + c * S;
        int64_t F[PPO_MAX_STAGES], B[PPO_MAX_STAGES], cf[PPO_MAX_STAGES], cb[PPO_MAX_STAGES];
        T_out[c] = INF;
        if (!ordering_ok(o, S, D)) { fault |= PPO_FAULT_ORDERING; continue; }
        if (!bounds_ok(e, S, L)) { fault |= PPO_FAULT_BOUNDS; continue; }
        int f = plan_durations(L, D, S, M, PF, PB, XF, XB, o, e, F, B, cf, cb);
        if (f) { fault |= f; continue; }
        int64_t T = ppo_variant_makespan(variant, S, M, F, B, cf, cb);
        if (T < 0) { nomem = 1; continue; }
        T_out[c] = T;
    }
    free(own);
    if (nomem) return PPO_ERR_NOMEM;
    return fault;
}
