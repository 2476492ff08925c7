"""Pins for the oracle's keep-the-minimum over candidates."""
import itertools

import numpy as np
import pytest

from helpers import brute_plan, channel_table, event_sim
from paper_2204_10562_amd import workloads


def test_best_plan_by_brute_force(ppo):
    for seed in (31, 32, 33):
        w = workloads.random_small(seed, 8, 4, 3, 1, hi_time=9, hi_act=500)
        rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)
        P = [int(a + b) for a, b in zip(PF, PB)]
        orders = np.array(list(itertools.permutations(range(4), 3)), np.int32)
        for M in (1, 4):
            best = None
            for c, o in enumerate(orders):
                X = channel_table(XF, XB, 4, 8, o)
                e = [0] + brute_plan(P, X, 3, 8)
                F = [int(PF[e[i + 1]] - PF[e[i]]) for i in range(3)]
                B = [int(PB[e[i + 1]] - PB[e[i]]) for i in range(3)]
                cf = [0] + [int(XF[(o[n - 1] * 4 + o[n]) * 8 + e[n] - 1]) for n in range(1, 3)]
                cb = [0] + [int(XB[(o[n - 1] * 4 + o[n]) * 8 + e[n] - 1]) for n in range(1, 3)]
                T = event_sim(F, B, cf, cb, M)[0]
                if best is None or T < best[0]:
                    best = (T, c, e[1:], o.tolist())
            rc, res, T_all, C_all = ppo.best_plan(8, 4, 3, len(orders), M, PF, PB, XF, XB, orders)
            assert rc == 0
            assert (res["T"], res["best_index"], res["bounds"], res["order"]) == best
            assert T_all[res["best_index"]] == res["T"] == T_all.min()
            assert C_all[res["best_index"]] == res["C"]


def test_ties_go_to_the_lowest_index(ppo):
    # identical links everywhere: every ordering gives the same T, index 0 must win
    w = workloads.tiny()
    bw = np.full((4, 4), 16000, np.int64)
    rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, bw)
    rc, res, T_all, C_all = ppo.best_plan(w.L, 4, 4, 24, 8, PF, PB, XF, XB, None)
    assert rc == 0
    assert (T_all == T_all[0]).all()
    assert res["best_index"] == 0 and res["order"] == [0, 1, 2, 3]
    # and with explicit, shuffled candidates the first row of the minimum wins
    o = workloads.all_orderings(4)[::-1].copy()
    rc, res, T_all, _ = ppo.best_plan(w.L, 4, 4, 24, 8, PF, PB, XF, XB, o)
    assert res["best_index"] == 0 and res["order"] == [3, 2, 1, 0]


def test_default_candidates_are_lexicographic(ppo):
    w = workloads.tiny()
    rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)
    a = ppo.best_plan(w.L, 4, 4, 24, 4, PF, PB, XF, XB, None)
    b = ppo.best_plan(w.L, 4, 4, 24, 4, PF, PB, XF, XB, workloads.all_orderings(4))
    assert a[0] == 0 and a[1] == b[1]
    np.testing.assert_array_equal(a[2], b[2])
    assert a[1]["order"] == workloads.all_orderings(4)[a[1]["best_index"]].tolist()
