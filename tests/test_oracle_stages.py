"""Pins for the oracle's stage-count search (outer loop of Alg. 3): every (candidate, stage
count) entry against brute force over all contiguous partitions and an independent event
simulation, the winner against a scan written out here, and closed forms."""
import itertools

import numpy as np
import pytest

from helpers import brute_optimum, brute_plan, channel_table, event_sim
from paper_2204_10562_amd import workloads


def tables(ppo, w, bw=None):
    rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw if bw is None else bw)
    assert rc == 0
    return PF, PB, XF, XB


def plan_by_brute_force(PF, PB, XF, XB, L, D, order, M):
    """(C, bounds, T) of the tie-broken min-max plan along `order` (all of its devices)."""
    S = len(order)
    P = [int(a + b) for a, b in zip(PF, PB)]
    X = channel_table(XF, XB, D, L, order)
    C = brute_optimum(P, X, S, L)
    e = [0] + brute_plan(P, X, S, L)
    F = [int(PF[e[i + 1]] - PF[e[i]]) for i in range(S)]
    B = [int(PB[e[i + 1]] - PB[e[i]]) for i in range(S)]
    cf = [0] + [int(XF[(order[n - 1] * D + order[n]) * L + e[n] - 1]) for n in range(1, S)]
    cb = [0] + [int(XB[(order[n - 1] * D + order[n]) * L + e[n] - 1]) for n in range(1, S)]
    return C, e[1:], event_sim(F, B, cf, cb, M)[0]


@pytest.mark.parametrize("seed,L,D,S,M", [(41, 7, 4, 3, 1), (42, 8, 4, 4, 3), (43, 6, 3, 3, 6),
                                          (44, 9, 5, 3, 2), (45, 5, 5, 5, 4)])
def test_every_entry_by_brute_force(ppo, seed, L, D, S, M):
    w = workloads.random_small(seed, L, D, S, 1, hi_time=9, hi_act=500)
    PF, PB, XF, XB = tables(ppo, w)
    orders = np.array(list(itertools.permutations(range(D), S)), np.int32)[:: max(1, S - 1)]
    N = len(orders)
    rc, res, T_all, C_all, b_all = ppo.best_plan_stages(L, D, S, N, M, PF, PB, XF, XB, orders)
    assert rc == 0
    best = None
    for c, o in enumerate(orders):
        for xi in range(1, S + 1):
            C, e, T = plan_by_brute_force(PF, PB, XF, XB, L, D, [int(d) for d in o[:xi]], M)
            assert C_all[c, xi - 1] == C
            assert T_all[c, xi - 1] == T
            at = xi * (xi - 1) // 2
            assert b_all[c, at:at + xi].tolist() == e
            if best is None or T < best[0]:
                best = (T, c, xi, C, e, [int(d) for d in o[:xi]])
    assert (res["T"], res["best_index"], res["S"], res["C"], res["bounds"], res["order"]) == best


def test_one_stage_is_the_whole_model(ppo):
    w = workloads.tiny()
    PF, PB, XF, XB = tables(ppo, w)
    for M in (1, 8):
        rc, res, T_all, C_all, b_all = ppo.best_plan_stages(w.L, 4, 4, 24, M, PF, PB, XF, XB, None)
        assert rc == 0
        total = int(PF[w.L] + PB[w.L])
        assert (C_all[:, 0] == total).all() and (T_all[:, 0] == M * total).all()
        assert (b_all[:, 0] == w.L).all()


def test_last_column_is_the_fixed_stage_count_result(ppo):
    w = workloads.tiny()
    PF, PB, XF, XB = tables(ppo, w)
    rc, res, T_all, C_all, b_all = ppo.best_plan_stages(w.L, 4, 4, 24, 8, PF, PB, XF, XB, None)
    rc2, fixed, T_fix, C_fix = ppo.best_plan(w.L, 4, 4, 24, 8, PF, PB, XF, XB, None)
    assert rc == 0 and rc2 == 0
    np.testing.assert_array_equal(T_all[:, 3], T_fix)
    np.testing.assert_array_equal(C_all[:, 3], C_fix)
    assert res["T"] <= fixed["T"]


def test_free_transfers_make_more_stages_no_worse_per_microbatch(ppo):
    # without transfer cost a finer partition never has a larger bottleneck
    w = workloads.random_small(46, 12, 4, 4, 1, hi_time=50, hi_act=1)
    bw = np.full((4, 4), 10**9, np.int64)
    PF, PB, XF, XB = tables(ppo, w, bw)
    assert (np.asarray(XF) <= 1).all()
    rc, res, T_all, C_all, b_all = ppo.best_plan_stages(12, 4, 4, 24, 4, PF, PB, XF, XB, None)
    assert rc == 0
    assert (np.diff(C_all, axis=1) <= 1).all()   # transfers round up to at most 1 us


def test_slow_links_favour_a_single_stage(ppo):
    # a link so slow that any cut costs more than running everything on one GPU
    w = workloads.random_small(47, 10, 4, 4, 1, hi_time=20, hi_act=10**6)
    w.actf[:] = 10**6
    w.actb[:] = 10**6
    bw = np.ones((4, 4), np.int64)
    PF, PB, XF, XB = tables(ppo, w, bw)
    rc, res, T_all, C_all, b_all = ppo.best_plan_stages(10, 4, 4, 24, 16, PF, PB, XF, XB, None)
    assert rc == 0
    assert res["S"] == 1 and res["best_index"] == 0 and res["bounds"] == [10] and res["order"] == [0]
    assert res["T"] == 16 * int(PF[10] + PB[10])


def test_interior_stage_count_can_win(ppo):
    # fast link 0<->1, everything else slow: two stages beat one (overlap) and beat three or
    # four (a slow link in the chain)
    L = 8
    fwd = np.full(L, 10, np.int64)
    bwd = np.full(L, 20, np.int64)
    act = np.full(L, 1000, np.int64)
    bw = np.ones((4, 4), np.int64)          # 1000 us per transfer
    bw[0, 1] = bw[1, 0] = 1000              # 1 us per transfer
    rc, PF, PB, XF, XB = ppo.prefix_costs(fwd, bwd, act, act, bw)
    order = np.array([[0, 1, 2, 3]], np.int32)
    rc, res, T_all, C_all, b_all = ppo.best_plan_stages(L, 4, 4, 1, 32, PF, PB, XF, XB, order)
    assert rc == 0
    assert res["S"] == 2 and res["bounds"] == [4, 8]
    assert T_all[0, 1] < T_all[0, 0] and T_all[0, 1] < T_all[0, 2] and T_all[0, 1] < T_all[0, 3]


def test_ties_go_to_lowest_candidate_then_fewest_stages(ppo):
    # zero-cost layers at the end: splitting them off changes nothing, so xi = 1 ties with
    # larger xi in C, and T of one stage is the smallest possible sum
    L = 4
    fwd = np.array([5, 0, 0, 0], np.int64)
    bwd = np.array([5, 0, 0, 0], np.int64)
    act = np.zeros(L, np.int64)
    bw = np.full((3, 3), 10, np.int64)
    rc, PF, PB, XF, XB = ppo.prefix_costs(fwd, bwd, act, act, bw)
    rc, res, T_all, C_all, b_all = ppo.best_plan_stages(L, 3, 3, 6, 5, PF, PB, XF, XB, None)
    assert rc == 0
    assert (C_all == 10).all()
    assert (T_all == 50).all()
    assert res["best_index"] == 0 and res["S"] == 1
