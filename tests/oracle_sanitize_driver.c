/* Drives every entry point of the oracle on small pseudo-random problems and prints a checksum.
 * tests/test_oracle_sanitized.py builds it twice, with and without -fsanitize=address,undefined,
 * and expects both builds to run clean and print the same line.  Test code: never shipped. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "ppo.h"

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd(void) {
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return state;
}
static int64_t below(int64_t n) { return (int64_t)(rnd() % (uint64_t)n); }

int main(void) {
    uint64_t sum = 0;
    for (int rep = 0; rep < 40; ++rep) {
        const int L = 1 + (int)below(24), D = 1 + (int)below(6);
        const int S = 1 + (int)below(L < D ? L : D), M = 1 + (int)below(9);
        const int64_t N = 1 + below(12);
        int64_t *fwd = malloc(sizeof(int64_t) * L), *bwd = malloc(sizeof(int64_t) * L);
        int64_t *af = malloc(sizeof(int64_t) * L), *ab = malloc(sizeof(int64_t) * L), *al = malloc(sizeof(int64_t) * L);
        int64_t *bw = malloc(sizeof(int64_t) * D * D);
        for (int l = 0; l < L; ++l) {
            fwd[l] = below(9); bwd[l] = below(17); al[l] = below(5000);
            af[l] = (rep & 1) ? 700 : below(4000); ab[l] = (rep & 1) ? 900 : below(4000);
        }
        for (int i = 0; i < D * D; ++i) bw[i] = 1 + below(200);
        int64_t *PF = malloc(sizeof(int64_t) * (L + 1)), *PB = malloc(sizeof(int64_t) * (L + 1));
        int64_t *XF = malloc(sizeof(int64_t) * D * D * L), *XB = malloc(sizeof(int64_t) * D * D * L);
        if (ppo_prefix_costs(L, D, fwd, bwd, af, (rep % 3) ? ab : NULL, bw, PF, PB, XF, XB) != 0) return 2;
        /* candidate rows: random distinct devices */
        int32_t *ord = malloc(sizeof(int32_t) * N * D);
        for (int64_t c = 0; c < N; ++c) {
            int32_t *row = ord + c * D;
            for (int d = 0; d < D; ++d) row[d] = d;
            for (int d = D - 1; d > 0; --d) { int j = (int)below(d + 1); int32_t t = row[d]; row[d] = row[j]; row[j] = t; }
        }
        int32_t *ordS = malloc(sizeof(int32_t) * N * S);
        for (int64_t c = 0; c < N; ++c) for (int n = 0; n < S; ++n) ordS[c * S + n] = ord[c * D + n];
        int64_t *C = malloc(sizeof(int64_t) * N), *T = malloc(sizeof(int64_t) * N);
        int32_t *bounds = malloc(sizeof(int32_t) * N * S);
        if (ppo_partition_dp(L, D, S, N, PF, PB, XF, XB, ordS, C, bounds) != 0) return 3;
        if (ppo_schedule_makespan(L, D, S, N, M, PF, PB, XF, XB, ordS, bounds, T) != 0) return 4;
        for (int64_t c = 0; c < N; ++c) sum = sum * 1000003u + (uint64_t)C[c] * 31u + (uint64_t)T[c] + (uint64_t)bounds[c * S];
        ppo_result res;
        if (ppo_best_plan(L, D, S, N, M, PF, PB, XF, XB, ordS, &res, T, C) != 0) return 5;
        sum = sum * 1000003u + (uint64_t)res.best_index + (uint64_t)res.T;
        const int tri = S * (S + 1) / 2;
        int64_t *Ts = malloc(sizeof(int64_t) * N * S), *Cs = malloc(sizeof(int64_t) * N * S);
        int32_t *bs = malloc(sizeof(int32_t) * N * tri);
        if (ppo_best_plan_stages(L, D, S, N, M, PF, PB, XF, XB, ordS, &res, Ts, Cs, bs) != 0) return 6;
        sum = sum * 1000003u + (uint64_t)res.S + (uint64_t)res.T;
        for (int v = 0; v <= PPO_SCHED_FIFO; ++v) {
            if (ppo_schedule_makespan_variant(v, L, D, S, N, M, PF, PB, XF, XB, ordS, bounds, T) != 0) return 7;
            for (int64_t c = 0; c < N; ++c) sum = sum * 1000003u + (uint64_t)T[c];
        }
        if (L <= 12) {
            const int triD = D * (D + 1) / 2;
            ppo_rep_result rr;
            int64_t *Tr = malloc(sizeof(int64_t) * N * D), *Wr = malloc(sizeof(int64_t) * N * D);
            int32_t *br = malloc(sizeof(int32_t) * N * triD), *rr2 = malloc(sizeof(int32_t) * N * triD);
            if (ppo_spp_replicated(L, D, N, M, fwd, bwd, af, ab, al, bw, ord, &rr, Tr, Wr, br, rr2) != 0) return 8;
            sum = sum * 1000003u + (uint64_t)rr.T + (uint64_t)rr.S;
            free(Tr); free(Wr); free(br); free(rr2);
        }
        int32_t *rdo = malloc(sizeof(int32_t) * D);
        if (ppo_rdo_order(D, bw, rdo) != 0) return 9;
        for (int d = 0; d < D; ++d) sum = sum * 31u + (uint64_t)rdo[d];
        int32_t *rounds = malloc(sizeof(int32_t) * (M + 4 * S + 8) * (4 * S - 3));
        const int sweeps = ppo_execution_order(S, M, rounds, M + 4 * S + 8);
        if (sweeps < 0) return 10;
        sum = sum * 31u + (uint64_t)sweeps;
        free(rounds); free(rdo); free(Ts); free(Cs); free(bs); free(C); free(T); free(bounds); free(ord); free(ordS);
        free(PF); free(PB); free(XF); free(XB); free(fwd); free(bwd); free(af); free(ab); free(al); free(bw);
    }
    printf("checksum %llu\n", (unsigned long long)sum);
    return 0;
}
