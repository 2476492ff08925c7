"""Pins for the oracle's partition DP: exhaustive enumeration, closed forms, worked cases."""
import itertools
import math

import numpy as np
import pytest

from conftest import read_golden
from helpers import brute_optimum, brute_plan, channel_table
from paper_2204_10562_amd import workloads


def _tables_from_p_x(p, x):
    """Two devices, link 0->1 with per-cut channel cost x (forward carries all of it)."""
    L = len(p)
    PF = np.concatenate([[0], np.cumsum(p)]).astype(np.int64)
    PB = np.zeros(L + 1, np.int64)
    XF = np.zeros(2 * 2 * L, np.int64)
    XB = np.zeros(2 * 2 * L, np.int64)
    XF[(0 * 2 + 1) * L:(0 * 2 + 1) * L + len(x)] = x
    return L, PF, PB, XF, XB


def test_handworked_cases(ppo):
    g = read_golden("dp_handworked.txt")
    for case in ("caseA", "caseB"):
        p, x = g[case + "_p"][0], g[case + "_x"][0]
        L, PF, PB, XF, XB = _tables_from_p_x(p, x)
        rc, C, bounds = ppo.partition_dp(L, 2, 2, 1, PF, PB, XF, XB, np.array([[0, 1]], np.int32))
        assert rc == 0
        assert C[0] == g[case + "_C"][0][0]
        assert bounds[0].tolist() == g[case + "_bounds"][0]


@pytest.mark.parametrize("seed,L,D,S", [(1, 6, 3, 3), (2, 7, 4, 4), (3, 9, 4, 3), (4, 8, 4, 2),
                                         (5, 5, 4, 4), (6, 10, 3, 3), (7, 4, 4, 4), (8, 9, 2, 2)])
def test_exhaustive_partitions_and_orderings(ppo, seed, L, D, S):
    # narrow value ranges force many ties, zero durations and asymmetric links are in
    w = workloads.random_small(seed, L, D, S, 1, zero_frac=0.2, hi_time=6, hi_act=300)
    rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)
    assert rc == 0
    P = [int(a + b) for a, b in zip(PF, PB)]
    orders = np.array(list(itertools.permutations(range(D), S)), np.int32)
    rc, C, bounds = ppo.partition_dp(L, D, S, len(orders), PF, PB, XF, XB, orders)
    assert rc == 0
    for c, o in enumerate(orders):
        X = channel_table(XF, XB, D, L, o)
        assert C[c] == brute_optimum(P, X, S, L), (c, o)
        assert bounds[c].tolist() == brute_plan(P, X, S, L), (c, o)


def test_single_stage_is_total_time(ppo):
    w = workloads.tiny()
    rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)
    orders = np.arange(w.D, dtype=np.int32).reshape(-1, 1)
    rc, C, bounds = ppo.partition_dp(w.L, w.D, 1, w.D, PF, PB, XF, XB, orders)
    assert rc == 0
    assert (C == int(w.fwd.sum() + w.bwd.sum())).all()
    assert (bounds[:, 0] == w.L).all()


def test_one_layer_per_stage(ppo):
    # S = L leaves exactly one partition: C = max(layer times, channel cost at every cut)
    w = workloads.random_small(11, 4, 4, 4, 24)
    rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)
    orders = workloads.all_orderings(4)
    rc, C, bounds = ppo.partition_dp(4, 4, 4, 24, PF, PB, XF, XB, orders)
    assert rc == 0
    for c, o in enumerate(orders):
        chan = [int(XF[(o[n - 1] * 4 + o[n]) * 4 + n - 1]) + int(XB[(o[n - 1] * 4 + o[n]) * 4 + n - 1])
                for n in range(1, 4)]
        assert C[c] == max(list(w.fwd + w.bwd) + chan)
        assert bounds[c].tolist() == [1, 2, 3, 4]


@pytest.mark.parametrize("L,S,p", [(12, 4, 7), (13, 4, 7), (17, 5, 3), (9, 9, 2), (10, 3, 1)])
def test_identical_layers_no_transfer(ppo, L, S, p):
    PF = np.arange(L + 1, dtype=np.int64) * p
    PB = np.zeros(L + 1, np.int64)
    X = np.zeros(S * S * L, np.int64)
    o = np.arange(S, dtype=np.int32).reshape(1, S)
    rc, C, bounds = ppo.partition_dp(L, S, S, 1, PF, PB, X, X, o)
    assert rc == 0
    assert C[0] == p * math.ceil(L / S)


def test_lower_bounds_and_bounds_shape(ppo):
    w = workloads.transformer()
    rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)
    orders = workloads.all_orderings(8)[::97]
    rc, C, bounds = ppo.partition_dp(w.L, w.D, w.S, len(orders), PF, PB, XF, XB, orders)
    assert rc == 0
    total = int(PF[-1] + PB[-1])
    assert (C >= -(-total // w.S)).all()
    assert (C >= int((w.fwd + w.bwd).max())).all()
    assert (bounds[:, -1] == w.L).all()
    assert (np.diff(np.concatenate([np.zeros((len(orders), 1), np.int32), bounds], axis=1), axis=1) >= 1).all()
    # C is the largest per-resource time of the returned plan
    P = PF + PB
    for c, o in enumerate(orders):
        e = [0] + bounds[c].tolist()
        comp = [int(P[e[i + 1]] - P[e[i]]) for i in range(w.S)]
        chan = [int(XF[(o[n - 1] * w.D + o[n]) * w.L + e[n] - 1] + XB[(o[n - 1] * w.D + o[n]) * w.L + e[n] - 1])
                for n in range(1, w.S)]
        assert C[c] == max(comp + chan)


def test_lexicographic_default_equals_explicit(ppo):
    w = workloads.tiny()
    rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)
    a = ppo.partition_dp(w.L, w.D, w.S, w.N, PF, PB, XF, XB, None)
    b = ppo.partition_dp(w.L, w.D, w.S, w.N, PF, PB, XF, XB, workloads.all_orderings(w.D))
    assert a[0] == 0 and b[0] == 0
    np.testing.assert_array_equal(a[1], b[1])
    np.testing.assert_array_equal(a[2], b[2])


def test_argument_and_ordering_faults(ppo):
    w = workloads.tiny()
    rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)
    o = workloads.all_orderings(4)
    assert ppo.partition_dp(w.L, 4, 5, 24, PF, PB, XF, XB, o)[0] == ppo.ERR_INVALID_ARG  # S > D
    assert ppo.partition_dp(w.L, 4, 4, 23, PF, PB, XF, XB, None)[0] == ppo.ERR_INVALID_ARG  # N != D!
    assert ppo.partition_dp(w.L, 4, 3, 24, PF, PB, XF, XB, None)[0] == ppo.ERR_INVALID_ARG  # S != D
    bad = o.copy(); bad[3, 1] = bad[3, 0]
    assert ppo.partition_dp(w.L, 4, 4, 24, PF, PB, XF, XB, bad)[0] == ppo.FAULT_ORDERING
    bad = o.copy(); bad[5, 2] = 4
    assert ppo.partition_dp(w.L, 4, 4, 24, PF, PB, XF, XB, bad)[0] == ppo.FAULT_ORDERING


def test_bottleneck_is_not_monotone_in_the_number_of_layers(ppo):
    # With transfer times that depend on the cut position, more layers can mean a smaller
    # bottleneck: three layers cut after the second (cheap link time there) beat two layers,
    # whose only cut is the dear one after the first.  Any pruning of the recursion of Sec. IV-B
    # that assumes W(l, xi) grows with l is therefore wrong in general (it does grow when no
    # link's time depends on the position).
    o = np.array([[0, 1]], np.int32)
    L, PF, PB, XF, XB = _tables_from_p_x([1, 1], [100])
    rc, C2, b2 = ppo.partition_dp(L, 2, 2, 1, PF, PB, XF, XB, o)
    assert rc == 0 and C2[0] == 100 and b2[0].tolist() == [1, 2]
    L, PF, PB, XF, XB = _tables_from_p_x([1, 1, 1], [100, 0])
    rc, C3, b3 = ppo.partition_dp(L, 2, 2, 1, PF, PB, XF, XB, o)
    assert rc == 0 and C3[0] == 2 and b3[0].tolist() == [2, 3]
    assert C3[0] < C2[0]
