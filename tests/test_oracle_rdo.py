"""Pins for the oracle's recursive device ordering (Alg. 2): every split of the ordering is a
minimum cut of the subgraph it splits (checked by enumerating all bipartitions)."""
import itertools

import numpy as np
import pytest

from paper_2204_10562_amd import workloads


def cut_weight(w, a, b):
    return sum(int(w[u][v]) for u in a for v in b)


def brute_min_cut(w, verts):
    verts = list(verts)
    best = None
    first, rest = verts[0], verts[1:]
    for r in range(0, len(rest)):
        for extra in itertools.combinations(rest, r):
            a = [first] + list(extra)
            b = [v for v in rest if v not in extra]
            c = cut_weight(w, a, b)
            if best is None or c < best:
                best = c
    return best


def is_recursive_min_cut_order(w, order):
    """Some prefix/suffix split of `order` is a minimum cut of its vertex set, recursively."""
    if len(order) <= 1:
        return True
    target = brute_min_cut(w, order)
    for p in range(1, len(order)):
        a, b = order[:p], order[p:]
        if cut_weight(w, a, b) == target and is_recursive_min_cut_order(w, a) and is_recursive_min_cut_order(w, b):
            return True
    return False


def sym_weights(bw):
    bw = np.asarray(bw, dtype=np.int64)
    return bw + bw.T


@pytest.mark.parametrize("seed,D", [(1, 2), (2, 3), (3, 4), (4, 5), (5, 6), (6, 7), (7, 8), (8, 8), (9, 9)])
def test_every_split_is_a_minimum_cut(ppo, seed, D):
    rng = np.random.Generator(np.random.PCG64(seed))
    bw = rng.integers(1, 1000, size=(D, D)).astype(np.int64)   # asymmetric, distinct-ish
    np.fill_diagonal(bw, 0)
    order = ppo.rdo_order(bw)
    assert sorted(order) == list(range(D))
    assert is_recursive_min_cut_order(sym_weights(bw), order)


@pytest.mark.parametrize("seed,D", [(11, 4), (12, 6), (13, 8)])
def test_with_many_ties(ppo, seed, D):
    rng = np.random.Generator(np.random.PCG64(seed))
    bw = rng.integers(1, 3, size=(D, D)).astype(np.int64)
    bw = np.minimum(bw, bw.T)
    np.fill_diagonal(bw, 0)
    order = ppo.rdo_order(bw)
    assert sorted(order) == list(range(D))
    assert is_recursive_min_cut_order(sym_weights(bw), order)


def test_islands_stay_together(ppo):
    # two fast islands joined by slow links: the first cut separates the islands, so each
    # island occupies a contiguous half of the ordering; the side with device 0 comes first
    w = workloads.transformer()
    order = ppo.rdo_order(w.bw)
    assert sorted(order[:4]) == [0, 1, 2, 3] and sorted(order[4:]) == [4, 5, 6, 7]
    w = workloads.hetero(N=1)
    order = ppo.rdo_order(w.bw)
    groups = [sorted(order[i:i + 4]) for i in range(0, 16, 4)]
    assert sorted(groups) == [[0, 1, 2, 3], [4, 5, 6, 7], [8, 9, 10, 11], [12, 13, 14, 15]]
    assert 0 in order[:4]


def test_path_graph_by_hand(ppo):
    # path 0 -5- 1 -1- 2 -7- 3: the lightest cut is the middle edge, then each pair splits
    bw = np.zeros((4, 4), np.int64)
    for u, v, b in ((0, 1, 5), (1, 2, 1), (2, 3, 7)):
        bw[u, v] = bw[v, u] = b
    assert ppo.rdo_order(bw) == [0, 1, 2, 3]
    # relabelled so that index order and path order differ: path 2 -5- 0 -1- 3 -7- 1
    bw = np.zeros((4, 4), np.int64)
    for u, v, b in ((2, 0, 5), (0, 3, 1), (3, 1, 7)):
        bw[u, v] = bw[v, u] = b
    order = ppo.rdo_order(bw)
    assert sorted(order[:2]) == [0, 2] and sorted(order[2:]) == [1, 3]
    assert order[0] == 0  # the side (and the vertex) with the lowest index first


def test_single_device_and_large(ppo):
    assert ppo.rdo_order(np.zeros((1, 1), np.int64)) == [0]
    w = workloads.stress(N=1)
    order = ppo.rdo_order(w.bw)
    assert sorted(order) == list(range(32))
