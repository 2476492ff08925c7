"""Pins for the oracle's planner with replicated stages (PRM, Alg. 4, inside SPP, Alg. 3).

Independent of oracle/: the optimum is found by enumerating every contiguous partition and
every replication vector and evaluating the paper's definition of W(|S|) directly; the
schedule by the event simulation of helpers.py plus the AllReduce term of Eq. 2."""
import itertools

import numpy as np
import pytest

from helpers import event_sim
from paper_2204_10562_amd import workloads


def cdiv(a, b):
    return -(-int(a) // int(b))


class Model:
    """The cost model of Sec. III-B for one ordering, written out from the definitions."""

    def __init__(self, w, alpha, order, M):
        self.L, self.D, self.M = w.L, w.D, M
        self.PF = np.concatenate([[0], np.cumsum(w.fwd)]).tolist()
        self.PB = np.concatenate([[0], np.cumsum(w.bwd)]).tolist()
        self.PA = np.concatenate([[0], np.cumsum(alpha)]).tolist()
        self.actf, self.actb, self.bw, self.o = w.actf, w.actb, w.bw, [int(d) for d in order]

    def minbw(self, A, B):
        return min(int(self.bw[self.o[u], self.o[v]]) for u in A for v in B if u != v)

    def stage(self, l0, l1, ranks):
        k = len(ranks)
        F = cdiv(self.PF[l1] - self.PF[l0], k)
        B = cdiv(self.PB[l1] - self.PB[l0], k)
        A = 0 if k == 1 else cdiv(2 * (k - 1) * (self.PA[l1] - self.PA[l0]), k * self.minbw(ranks, ranks))
        return F, B, A

    def channel(self, cut, left, right):
        cf = cdiv(self.actf[cut - 1], len(left) * len(right) * self.minbw(left, right))
        cb = cdiv(self.actb[cut - 1], len(left) * len(right) * self.minbw(right, left))
        return cf, cb

    def describe(self, bounds, reps):
        """Per-stage (F, B, A) and per-channel (cf, cb) of a plan."""
        ranks, n, l0 = [], 0, 0
        st, ch = [], [(0, 0)]
        for e, k in zip(bounds, reps):
            ranks.append(list(range(n, n + k)))
            st.append(self.stage(l0, e, ranks[-1]))
            if len(ranks) > 1:
                ch.append(self.channel(l0, ranks[-2], ranks[-1]))
            n += k
            l0 = e
        return st, ch

    def W(self, bounds, reps):
        """W(|S|) of Sec. IV-B for a plan."""
        st, ch = self.describe(bounds, reps)
        terms = [self.M * (F + B) + A for F, B, A in st] + [self.M * (cf + cb) for cf, cb in ch[1:]]
        return max(terms)

    def T(self, bounds, reps):
        """Eq. 2 with the event simulation as the schedule."""
        st, ch = self.describe(bounds, reps)
        S = len(st)
        F = [s[0] for s in st]; B = [s[1] for s in st]
        cf = [c[0] for c in ch]; cb = [c[1] for c in ch]
        T, start = event_sim(F, B, cf, cb, self.M)
        R = 2 * S - 1
        for s in range(S):
            if reps[s] == 1:
                continue
            j = R if s == S - 1 else 2 * R - (2 * s + 1)
            dur = F[s] + B[s] if s == S - 1 else B[s]
            done = max(start[(j, m)] + dur for m in range(1, self.M + 1))
            T = max(T, done + st[s][2])
        return T


def plans(L, D, xi):
    """All (bounds, reps): xi non-empty contiguous stages, replicas >= 1 summing to D."""
    for cuts in itertools.combinations(range(1, L), xi - 1):
        for bars in itertools.combinations(range(1, D), xi - 1):
            reps = [b - a for a, b in zip((0,) + bars, bars + (D,))]
            yield list(cuts) + [L], reps


def alpha_for(w, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(1, 5000, size=w.L).astype(np.int64)


@pytest.mark.parametrize("seed,L,D,M", [(51, 5, 3, 2), (52, 6, 4, 3), (53, 4, 4, 1), (54, 7, 3, 5), (55, 5, 5, 2)])
def test_optimum_and_schedule_by_brute_force(ppo, seed, L, D, M):
    w = workloads.random_small(seed, L, D, D, 1, hi_time=40, hi_act=3000)
    alpha = alpha_for(w, seed)
    orders = np.array(list(itertools.permutations(range(D))), np.int32)[::max(1, D - 1)][:8]
    N = len(orders)
    rc, res, T_all, W_all, b_all, r_all = ppo.spp_replicated(L, D, N, M, w.fwd, w.bwd, w.actf, w.actb,
                                                             alpha, w.bw, orders)
    assert rc == 0
    best = None
    for c, o in enumerate(orders):
        m = Model(w, alpha, o, M)
        for xi in range(1, D + 1):
            at = xi * (xi - 1) // 2
            if xi > L:
                assert W_all[c, xi - 1] == np.iinfo(np.int64).max
                continue
            opt = min(m.W(b, r) for b, r in plans(L, D, xi))
            assert W_all[c, xi - 1] == opt
            b, r = b_all[c, at:at + xi].tolist(), r_all[c, at:at + xi].tolist()
            assert sum(r) == D and b[-1] == L and all(x < y for x, y in zip(b, b[1:]))
            assert m.W(b, r) == opt                      # the reported plan attains it
            T = m.T(b, r)
            assert T_all[c, xi - 1] == T
            if best is None or T < best[0]:
                best = (T, c, xi, opt, b, r, [int(d) for d in o])
    assert (res["T"], res["best_index"], res["S"], res["W"], res["bounds"], res["reps"], res["order"]) == best


def tie_broken_plan(m, L, D, xi):
    """The plan Alg. 3 + Alg. 4 select: last stage's replication r ascending, then the cut l'
    ascending, then the previous stage's replication r' ascending - the first combination
    whose value reaches the optimum of its sub-problem (found by enumeration)."""
    def opt(l, n, k, r):      # best W for first l layers, k stages on ranks 0..n-1, last stage r replicas
        best = None
        for cuts in itertools.combinations(range(1, l), k - 1):
            for bars in itertools.combinations(range(1, n), k - 1):
                reps = [b - a for a, b in zip((0,) + bars, bars + (n,))]
                if reps[-1] != r:
                    continue
                v = sub.W(list(cuts) + [l], reps)
                best = v if best is None or v < best else best
        return best
    sub = m
    target = min(x for x in (opt(L, D, xi, r) for r in range(1, D + 1)) if x is not None)
    r = next(r for r in range(1, D + 1) if opt(L, D, xi, r) == target)
    bounds, reps = [L], [r]
    l, n, k = L, D, xi
    while k > 1:
        want = opt(l, n, k, r)
        found = None
        for lp in range(1, l):
            for rp in range(1, n - r + 1):
                head = opt(lp, n - r, k - 1, rp)
                if head is None:
                    continue
                left = list(range(n - r - rp, n - r)); right = list(range(n - r, n))
                cf, cb = m.channel(lp, left, right)
                F, B, A = m.stage(lp, l, right)
                if max(head, m.M * (cf + cb), m.M * (F + B) + A) == want:
                    found = (lp, rp)
                    break
            if found:
                break
        lp, rp = found
        bounds.append(lp); reps.append(rp)
        l, n, k, r = lp, n - r, k - 1, rp
    return bounds[::-1], reps[::-1]


@pytest.mark.parametrize("seed,L,D,M", [(61, 5, 3, 2), (62, 5, 4, 3), (63, 6, 4, 1)])
def test_plan_tie_break(ppo, seed, L, D, M):
    # narrow value ranges: many plans share the optimum
    w = workloads.random_small(seed, L, D, D, 1, hi_time=4, hi_act=30)
    alpha = np.full(L, 3, np.int64)
    order = np.arange(D, dtype=np.int32)[None, :]
    rc, res, T_all, W_all, b_all, r_all = ppo.spp_replicated(L, D, 1, M, w.fwd, w.bwd, w.actf, w.actb,
                                                             alpha, w.bw, order)
    assert rc == 0
    m = Model(w, alpha, order[0], M)
    for xi in range(1, min(L, D) + 1):
        at = xi * (xi - 1) // 2
        b, r = tie_broken_plan(m, L, D, xi)
        assert b_all[0, at:at + xi].tolist() == b
        assert r_all[0, at:at + xi].tolist() == r


def test_one_replica_per_stage_is_the_plain_partition(ppo):
    # D stages on D devices leave one device per stage: W = M * C of the plain recursion
    w = workloads.tiny()
    alpha = np.full(w.L, 1 << 20, np.int64)
    rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)
    for M in (1, 8):
        rc, res, T_all, W_all, b_all, r_all = ppo.spp_replicated(w.L, 4, 24, M, w.fwd, w.bwd, w.actf, w.actb,
                                                                 alpha, w.bw, None)
        rc2, C, bounds = ppo.partition_dp(w.L, 4, 4, 24, PF, PB, XF, XB, None)
        rc3, T = ppo.schedule_makespan(w.L, 4, 4, 24, M, PF, PB, XF, XB, None, bounds)
        assert rc == 0 and rc2 == 0 and rc3 == 0
        np.testing.assert_array_equal(W_all[:, 3], M * C)
        np.testing.assert_array_equal(b_all[:, 6:], bounds)
        assert (r_all[:, 6:] == 1).all()
        np.testing.assert_array_equal(T_all[:, 3], T)


def test_single_stage_closed_form(ppo):
    w = workloads.tiny()
    alpha = np.arange(1, w.L + 1, dtype=np.int64) * 100000
    M = 4
    rc, res, T_all, W_all, b_all, r_all = ppo.spp_replicated(w.L, 4, 24, M, w.fwd, w.bwd, w.actf, w.actb,
                                                             alpha, w.bw, None)
    assert rc == 0
    off = w.bw[~np.eye(4, dtype=bool)]
    want = M * (cdiv(w.fwd.sum(), 4) + cdiv(w.bwd.sum(), 4)) + cdiv(2 * 3 * int(alpha.sum()), 4 * int(off.min()))
    assert (W_all[:, 0] == want).all() and (T_all[:, 0] == want).all()
    assert (r_all[:, 0] == 4).all() and (b_all[:, 0] == w.L).all()


def test_bounds_of_lemma_1_with_allreduce(ppo):
    for seed in (71, 72, 73):
        L, D, M = 9, 4, 6
        w = workloads.random_small(seed, L, D, D, 1, hi_time=60, hi_act=4000)
        alpha = alpha_for(w, seed)
        rc, res, T_all, W_all, b_all, r_all = ppo.spp_replicated(L, D, 24, M, w.fwd, w.bwd, w.actf, w.actb,
                                                                 alpha, w.bw, None)
        assert rc == 0
        orders = workloads.all_orderings(D)
        for c in range(0, 24, 5):
            m = Model(w, alpha, orders[c], M)
            for xi in range(1, D + 1):
                at = xi * (xi - 1) // 2
                st, ch = m.describe(b_all[c, at:at + xi].tolist(), r_all[c, at:at + xi].tolist())
                C = max([F + B for F, B, A in st] + [cf + cb for cf, cb in ch])
                Amax = max(A for F, B, A in st)
                assert M * C <= T_all[c, xi - 1] <= (M + 4 * xi - 4) * C + Amax


def test_handworked_replicated_plan(ppo):
    from conftest import read_golden
    g = read_golden("replicated_handworked.txt")
    fwd = np.array(g["fwd"][0], np.int64); bwd = np.array(g["bwd"][0], np.int64)
    act = np.array(g["act"][0], np.int64); alpha = np.array(g["alpha"][0], np.int64)
    b = g["bw"][0][0]
    bw = np.array([[0, b], [b, 0]], np.int64)
    rc, res, T_all, W_all, b_all, r_all = ppo.spp_replicated(2, 2, 1, g["M"][0][0], fwd, bwd, act, act, alpha, bw,
                                                             np.array([[0, 1]], np.int32))
    assert rc == 0
    assert W_all[0, 0] == g["W_one_stage"][0][0] and T_all[0, 0] == g["T_one_stage"][0][0]
    assert W_all[0, 1] == g["W_two_stages"][0][0] and T_all[0, 1] == g["T_two_stages"][0][0]
    assert res["S"] == g["best_stages"][0][0] and res["reps"] == g["best_reps"][0]
    assert res["T"] == g["T_one_stage"][0][0]
