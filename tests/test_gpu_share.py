"""Candidates whose links have the same transfer times share one partition DP (L > 128):
bit-exact parity with the CPU oracle for every candidate, and the bookkeeping the library
leaves in the workspace against the same grouping worked out here from the tables."""
import copy
import sys

import numpy as np
import pytest

from paper_2204_10562_amd import workloads
from test_gpu_parity import oracle_tables

pytestmark = pytest.mark.gpu


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def G():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2204_10562_amd.problem import GpuProblem
    return GpuProblem


def islands(w, size, fast, slow, jitter=None):
    """Bandwidth of a cluster of islands of `size` devices: `fast` inside, `slow` across
    (jitter: an int array [D, D] added on top, to make more classes)."""
    D = w.D
    bw = np.empty((D, D), np.int64)
    for u in range(D):
        for v in range(D):
            bw[u, v] = fast if u // size == v // size else slow
    if jitter is not None:
        bw += jitter
    np.fill_diagonal(bw, 0)
    v = copy.copy(w)
    v.bw = bw
    return v


def grouping(w, XF, XB, orderings):
    """(number of link classes, key of every candidate) from the tables: two links are one class
    iff their rows of XF and of XB agree at every cut position 1..L-1."""
    L, D, S = w.L, w.D, w.S
    xf = np.asarray(XF).reshape(D * D, L)[:, :L - 1]
    xb = np.asarray(XB).reshape(D * D, L)[:, :L - 1]
    cls, seen = {}, {}
    for u in range(D):
        for v in range(D):
            if u != v:
                row = xf[u * D + v].tobytes() + xb[u * D + v].tobytes()
                cls[(u, v)] = seen.setdefault(row, len(seen))
    keys = [tuple(cls[(int(o[n - 1]), int(o[n]))] for n in range(1, S)) for o in orderings]
    return len(seen), keys


def check_shared(ppo, g, w, tables, expect_active=True):
    from paper_2204_10562_amd import binding as pp
    st, C, bounds = g.dp()
    rc, C0, b0 = ppo.partition_dp(w.L, w.D, w.S, w.N, *tables, w.orderings)
    assert rc == 0 and st == 0
    np.testing.assert_array_equal(C, C0)
    np.testing.assert_array_equal(bounds, b0)
    stats = pp.read_workspace_stats(g.ws)
    nc, keys = grouping(w, tables[2], tables[3], w.orderings)
    if expect_active:
        assert stats["share_active"] == 1
        assert stats["share_classes"] == nc and stats["share_keys"] == nc ** (w.S - 1)
        assert stats["share_computed"] == len(set(keys))
        # neighbours in the sorted list of keys share their first rows: at best every distinct
        # prefix of a key is computed once, at worst every row of every key
        prefixes = len({k[:n] for k in keys for n in range(1, w.S)})
        assert prefixes <= stats["rows_executed"] <= len(set(keys)) * (w.S - 1)
        if len(set(keys)) == 1:
            assert stats["rows_executed"] == prefixes
    else:
        # every candidate is computed, in the order of its first k devices; those with the same
        # first n + 1 devices can share rows 1..n (n < k)
        assert stats["share_active"] == 0 and stats["share_sorted"] == 1
        k = stats["share_sort_devices"]
        assert k >= 2 and w.D ** k <= 2 ** 20 and (k == w.S or w.D ** (k + 1) > 2 ** 20)
        o = [tuple(int(x) for x in row) for row in w.orderings]
        least = sum(len({r[:n + 1] for r in o}) for n in range(1, min(k, w.S - 1))) + w.N * (w.S - 1 - (min(k, w.S - 1) - 1))
        assert least <= stats["rows_executed"] <= w.N * (w.S - 1)
    return stats


@pytest.mark.parametrize("seed,L,D,S,N,size", [(4101, 150, 6, 5, 400, 2), (4102, 131, 8, 8, 900, 4),
                                               (4103, 300, 16, 16, 3000, 4), (4104, 257, 5, 2, 100, 2),
                                               (4105, 129, 12, 3, 500, 3)])
def test_shared_dp_two_bandwidths(ppo, G, seed, L, D, S, N, size):
    w = islands(workloads.random_small(seed, L, D, S, N, hi_time=60, hi_act=50000), size, 190, 23)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("shared dp, two bandwidths", seed, L, D, S, N)
    stats = check_shared(ppo, g, w, tables)
    assert stats["share_classes"] == 2 and stats["share_computed"] <= 2 ** (S - 1)


def test_shared_dp_directional_and_many_classes(ppo, G):
    # forward and backward sizes differ and the bandwidth is not symmetric: a class needs both
    # rows equal; the jitter makes a dozen classes
    rng = np.random.Generator(np.random.PCG64(4201))
    base = workloads.random_small(4201, 140, 6, 4, 700, hi_time=60, hi_act=90000)
    w = islands(base, 3, 150, 20, jitter=rng.integers(0, 3, size=(6, 6)))
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("shared dp, several classes")
    stats = check_shared(ppo, g, w, tables)
    assert 2 < stats["share_classes"] <= 30


def test_shared_dp_equal_rows_from_different_bandwidths(ppo, G):
    # activations so small that every bandwidth moves them in one microsecond (or none, where
    # the size is 0): all links are one class although no two bandwidths are equal, and the
    # times still depend on the cut position
    w = workloads.random_small(4301, 160, 5, 5, 300, hi_time=60, hi_act=40, zero_frac=0.3)
    w.actf = w.actf.copy(); w.actb = w.actb.copy()
    w.actf[::3] = 0
    w.actb[:] = w.actf
    w.bw = (np.arange(25, dtype=np.int64).reshape(5, 5) * 7 + 50)
    np.fill_diagonal(w.bw, 0)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("shared dp, one class")
    stats = check_shared(ppo, g, w, tables)
    assert stats["share_classes"] == 1 and stats["share_computed"] == 1


@pytest.mark.parametrize("seed,L,D,S,N", [(4401, 133, 8, 8, 300), (4402, 150, 6, 6, 5000), (4403, 200, 40, 5, 900),
                                          (4404, 140, 7, 7, 6000)])
def test_shared_dp_keys_beyond_the_table(ppo, G, seed, L, D, S, N):
    # random bandwidths: every link a class of its own and too many sequences for the table:
    # every candidate is computed, sorted by its first devices so that neighbours share rows
    w = workloads.random_small(seed, L, D, S, N, hi_time=60, hi_act=90000)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("shared dp, keys beyond the table", seed, L, D, S, N)
    stats = check_shared(ppo, g, w, tables, expect_active=False)
    if N > 4096:  # (more candidates than waves: runs of at least two)
        assert stats["rows_executed"] < w.N * (w.S - 1)
    # a list with bad rows and repeated rows, and the search over the stage counts
    v = copy.copy(w)
    v.orderings = w.orderings.copy()
    v.orderings[N // 3] = v.orderings[N // 3 + 1]
    v.orderings[7, 1] = v.orderings[7, 0]
    v.orderings[N - 1, S - 1] = -1
    g = G(v)
    g.set_tables(*tables)
    st, C, b = g.dp()
    rc, C0, b0 = ppo.partition_dp(v.L, v.D, v.S, v.N, *tables, v.orderings)
    assert st == rc == ppo.FAULT_ORDERING
    np.testing.assert_array_equal(C, C0)
    np.testing.assert_array_equal(b, b0)
    g = G(w)
    g.set_tables(*tables)
    st, C, b = g.dp_stages()
    rc, res0, T0, C0, b0 = ppo.best_plan_stages(w.L, w.D, w.S, w.N, 5, *tables, w.orderings)
    assert st == 0 and rc == 0
    np.testing.assert_array_equal(C, C0)
    np.testing.assert_array_equal(b, b0)


def test_shared_dp_bad_orderings(ppo, G):
    # bad rows are reported as always and do not disturb the groups they would have joined
    w = islands(workloads.random_small(4501, 170, 6, 6, 600, hi_time=60, hi_act=50000), 3, 200, 31)
    tables = oracle_tables(ppo, w)
    good = ppo.partition_dp(w.L, w.D, w.S, w.N, *tables, w.orderings)
    v = copy.copy(w)
    v.orderings = w.orderings.copy()
    bad = (0, 77, 78, 599)
    v.orderings[0, 3] = v.orderings[0, 1]
    v.orderings[77, 5] = 6
    v.orderings[78, 0] = -2
    v.orderings[599, 2] = 1 << 20
    g = G(v)
    g.set_tables(*tables)
    say("shared dp, bad orderings")
    st, C, b = g.dp()
    rc0, C0, b0 = ppo.partition_dp(v.L, v.D, v.S, v.N, *tables, v.orderings)
    assert st == ppo.FAULT_ORDERING == rc0
    np.testing.assert_array_equal(C, C0)
    np.testing.assert_array_equal(b, b0)
    keep = np.array([c for c in range(w.N) if c not in bad])
    np.testing.assert_array_equal(C[keep], good[1][keep])
    np.testing.assert_array_equal(b[keep], good[2][keep])
    from paper_2204_10562_amd import binding as pp
    stats = pp.read_workspace_stats(g.ws)
    _, keys = grouping(v, tables[2], tables[3], v.orderings[keep])
    assert stats["share_computed"] == len(set(keys)) + len(bad)


@pytest.mark.parametrize("seed,L,D,S,N,size", [(4601, 145, 6, 6, 800, 2), (4602, 170, 12, 12, 1500, 4),
                                               (4603, 133, 10, 8, 600, 5)])
def test_shared_dp_stage_counts_and_best_plan(ppo, G, seed, L, D, S, N, size):
    # the plans for every stage count, and the whole search with its arg-min, on shared DPs
    # (the schedules too run over the representatives only)
    w = islands(workloads.random_small(seed, L, D, S, N, hi_time=60, hi_act=50000), size, 210, 17)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("shared dp, stage counts", seed, L, D, S, N)
    st, C, bounds = g.dp_stages()
    assert st == 0
    Ms = (7, 2 * S + 1)
    want = [ppo.best_plan_stages(w.L, w.D, w.S, w.N, M, *tables, w.orderings) for M in Ms]
    assert all(x[0] == 0 for x in want)
    np.testing.assert_array_equal(C, want[0][3])
    np.testing.assert_array_equal(bounds, want[0][4])
    for want_all in (True, False):
        st, res, T, C2 = g.best_stages(Ms, want_all=want_all)
        assert st == 0
        for q in range(len(Ms)):
            assert res[q] == want[q][1]
            if want_all:
                np.testing.assert_array_equal(T[q], want[q][2])
                np.testing.assert_array_equal(C2, want[q][3])
    say("shared dp, best plan")
    for want_all in (True, False):
        st, res, T, C1 = g.best_multi((3, 24), want_all=want_all)
        assert st == 0
        for q, M in enumerate((3, 24)):
            rc, r0, T0, C0 = ppo.best_plan(w.L, w.D, w.S, w.N, M, *tables, w.orderings)[:4]
            assert rc == 0 and res[q] == r0
            if want_all:
                np.testing.assert_array_equal(T[q], T0)
                np.testing.assert_array_equal(C1, C0)


@pytest.mark.parametrize("seed,L,D,S,N,size", [(4701, 200, 12, 12, 2500, 4), (4702, 129, 9, 9, 700, 3),
                                               (4703, 260, 16, 16, 1500, 4), (4704, 150, 16, 10, 1000, 8)])
def test_shared_schedule(ppo, G, seed, L, D, S, N, size):
    # 9..16 stages: the schedule too is evaluated once per group of candidates; T and C of every
    # candidate (when asked for), the winner with its lowest-index tie-break, and bad rows
    clean = islands(workloads.random_small(seed, L, D, S, N, hi_time=60, hi_act=50000), size, 170, 29)
    tables = oracle_tables(ppo, clean)
    Ms = (1, S, 4 * S + 3)
    big = np.iinfo(np.int64).max
    bad = [5, N // 2, N - 1]
    rc, C0, b0 = ppo.partition_dp(L, D, S, N, *tables, clean.orderings)
    assert rc == 0
    C0[bad] = big
    want = []
    for M in Ms:
        rc, T0 = ppo.schedule_makespan(L, D, S, N, M, *tables, clean.orderings, b0)
        assert rc == 0
        T0[bad] = big
        best = int(np.argmin(T0))  # the first of the smallest
        want.append((T0, dict(best_index=best, T=int(T0[best]), C=int(C0[best]), S=S,
                              bounds=[int(x) for x in b0[best]],
                              order=[int(x) for x in clean.orderings[best]])))
    w = copy.copy(clean)
    w.orderings = clean.orderings.copy()
    w.orderings[5, 1] = w.orderings[5, 0]
    w.orderings[N // 2, S - 1] = D
    w.orderings[N - 1, 0] = -7
    g = G(w)
    g.set_tables(*tables)
    say("shared schedule", seed, L, D, S, N)
    for want_all in (True, False):
        st, res, T, C = g.best_multi(Ms, want_all=want_all)
        assert st == ppo.FAULT_ORDERING
        for q, M in enumerate(Ms):
            assert res[q] == want[q][1]
            if want_all:
                np.testing.assert_array_equal(T[q], want[q][0])
                np.testing.assert_array_equal(C, C0)
    from paper_2204_10562_amd import binding as pp
    stats = pp.read_workspace_stats(g.ws)
    keep = np.array([c for c in range(N) if c not in bad])
    _, keys = grouping(w, tables[2], tables[3], w.orderings[keep])
    assert stats["share_active"] == 1 and stats["share_computed"] == len(set(keys)) + len(bad)
    # a single count through pp_best_plan
    st, r1, T1, C1 = g.best(Ms[1])
    assert st == ppo.FAULT_ORDERING and r1 == want[1][1]
    np.testing.assert_array_equal(T1, want[1][0])
    np.testing.assert_array_equal(C1, C0)
    # and without bad rows the whole search against the oracle's
    g = G(clean)
    g.set_tables(*tables)
    st, res, T, C = g.best_multi(Ms[1:])
    assert st == 0
    for q, M in enumerate(Ms[1:]):
        rc, r0, T0, C1 = ppo.best_plan(L, D, S, N, M, *tables, clean.orderings)
        assert rc == 0 and res[q] == r0
        np.testing.assert_array_equal(T[q], T0)
        np.testing.assert_array_equal(C, C1)


def test_shared_corner_shapes(ppo, G):
    # a single stage (one key for everybody), and a list in which every row is bad
    w = islands(workloads.random_small(4801, 140, 4, 1, 50, hi_time=60, hi_act=50000), 2, 100, 10)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("shared dp, one stage")
    check_shared(ppo, g, w, tables)
    w = islands(workloads.random_small(4802, 150, 5, 4, 40, hi_time=60, hi_act=50000), 2, 100, 10)
    w.orderings = w.orderings.copy()
    w.orderings[:, 2] = w.orderings[:, 0]
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("shared dp, every row bad")
    st, C, b = g.dp()
    assert st == ppo.FAULT_ORDERING
    assert (C == np.iinfo(np.int64).max).all() and (b == 0).all()
    st, res, T, C = g.best(3)
    assert st == ppo.FAULT_ORDERING and res["best_index"] == -1
    assert (T == np.iinfo(np.int64).max).all()


@pytest.mark.parametrize("kind", ["equal_activations", "wide_times"])
def test_shared_schedule_other_dp_paths(ppo, G, kind):
    # 9..16 stages on more than 128 layers where the DP itself takes another path: the closed
    # form (transfer times that do not depend on the cut position) and the 64-bit fallback
    # (times beyond the 32-bit keys); the schedule still runs over the representatives
    w = workloads.random_small(4901, 180, 12, 10, 1200, hi_time=40, hi_act=30000, same_act=kind == "equal_activations")
    w = islands(w, 4, 160, 21)
    if kind == "wide_times":
        w.fwd = w.fwd << 34
        w.bwd = w.bwd << 34
        w.actf = w.actf << 30
        w.actb = w.actb << 30
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("shared schedule,", kind)
    Ms = (2, 37)
    st, res, T, C = g.best_multi(Ms)
    assert st == 0
    for q, M in enumerate(Ms):
        rc, r0, T0, C0 = ppo.best_plan(w.L, w.D, w.S, w.N, M, *tables, w.orderings)
        assert rc == 0 and res[q] == r0
        np.testing.assert_array_equal(T[q], T0)
        np.testing.assert_array_equal(C, C0)
    st, res2, _, _ = g.best_multi(Ms, want_all=False)
    assert st == 0 and res2 == res
    from paper_2204_10562_amd import binding as pp
    stats = pp.read_workspace_stats(g.ws)
    assert stats["share_active"] == 1 and stats["share_computed"] < w.N
    if kind == "equal_activations":
        assert stats["rows_executed"] == 0


def test_more_devices_than_the_class_table_holds(ppo, G):
    # more than 64 devices: no grouping and no sorting, every candidate on its own as ever
    w = workloads.random_small(5001, 140, 66, 3, 60, hi_time=60, hi_act=90000)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("dp, 66 devices")
    st, C, b = g.dp()
    rc, C0, b0 = ppo.partition_dp(w.L, w.D, w.S, w.N, *tables, w.orderings)
    assert st == 0 and rc == 0
    np.testing.assert_array_equal(C, C0)
    np.testing.assert_array_equal(b, b0)
    st, res, T, C = g.best(4)
    rc, r0, T0, C0 = ppo.best_plan(w.L, w.D, w.S, w.N, 4, *tables, w.orderings)
    assert st == 0 and rc == 0 and res == r0
    np.testing.assert_array_equal(T, T0)


@pytest.mark.parametrize("two_bandwidths", [True, False])
def test_library_list_of_all_orderings_with_many_layers(ppo, G, two_bandwidths):
    # orderings = NULL (all D! in lexicographic order, generated on the device) with more than
    # 128 layers: grouped by link classes (two bandwidths) or sorted by devices (random ones)
    import math
    w = workloads.random_small(5101, 150, 6, 6, 1, hi_time=60, hi_act=50000)
    if two_bandwidths:
        w = islands(w, 3, 180, 25)
    w.orderings = None
    w.N = math.factorial(6)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("all 6! orderings, 150 layers, two bandwidths:", two_bandwidths)
    explicit = workloads.all_orderings(6)
    st, C, b = g.dp()
    rc, C0, b0 = ppo.partition_dp(w.L, w.D, w.S, w.N, *tables, explicit)
    assert st == 0 and rc == 0
    np.testing.assert_array_equal(C, C0)
    np.testing.assert_array_equal(b, b0)
    from paper_2204_10562_amd import binding as pp
    stats = pp.read_workspace_stats(g.ws)
    assert stats["share_active"] == int(two_bandwidths) and stats["share_sorted"] == int(not two_bandwidths)
    for want_all in (True, False):
        st, res, T, C1 = g.best_multi((2, 30), want_all=want_all)
        assert st == 0
        for q, M in enumerate((2, 30)):
            rc, r0, T0, C0 = ppo.best_plan(w.L, w.D, w.S, w.N, M, *tables, explicit)
            assert rc == 0 and res[q] == r0
            if want_all:
                np.testing.assert_array_equal(T[q], T0)
        st, res, T, C2 = g.best_stages((9,), want_all=want_all)
        rc, r0, T0, C0, _ = ppo.best_plan_stages(w.L, w.D, w.S, w.N, 9, *tables, explicit)
        assert st == 0 and rc == 0 and res[0] == r0
        if want_all:
            np.testing.assert_array_equal(T[0], T0)
            np.testing.assert_array_equal(C2, C0)


@pytest.mark.parametrize("seed", range(5200, 5240))
def test_shared_random_shapes(ppo, G, seed):
    # shapes drawn at random above 128 layers: islands of random size and two to four bandwidth
    # levels (grouped), or random bandwidths (sorted); any S up to D; plans, schedules for two
    # microbatch counts, winners, and every stage count
    rng = np.random.Generator(np.random.PCG64(seed))
    L = int(rng.integers(129, 400))
    D = int(rng.integers(2, 13))
    S = int(rng.integers(1, D + 1))
    N = int(rng.integers(1, 6000)) if seed % 4 == 0 else int(rng.integers(1, 400))
    w = workloads.random_small(seed, L, D, S, N, zero_frac=0.1 if seed % 2 else 0.0,
                               hi_time=int(rng.integers(2, 200)), hi_act=int(rng.integers(1, 60000)))
    if seed % 3:
        levels = rng.integers(5, 300, size=int(rng.integers(2, 5)))
        size = int(rng.integers(1, D + 1))
        bw = np.empty((D, D), np.int64)
        for u in range(D):
            for v in range(D):
                bw[u, v] = levels[0] if u // size == v // size else levels[1 + (u + v) % (len(levels) - 1)]
        np.fill_diagonal(bw, 0)
        w.bw = bw
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("shared random", seed, L, D, S, N)
    Ms = (int(rng.integers(1, 9)), int(rng.integers(9, 200)))
    st, res, T, C = g.best_multi(Ms)
    assert st == 0
    for q, M in enumerate(Ms):
        rc, r0, T0, C0 = ppo.best_plan(L, D, S, N, M, *tables, w.orderings)
        assert rc == 0 and res[q] == r0
        np.testing.assert_array_equal(T[q], T0)
        np.testing.assert_array_equal(C, C0)
    st, C, b = g.dp()
    rc, C0, b0 = ppo.partition_dp(L, D, S, N, *tables, w.orderings)
    assert st == 0 and rc == 0
    np.testing.assert_array_equal(C, C0)
    np.testing.assert_array_equal(b, b0)
    st, res, T, C = g.best_stages(Ms[:1])
    rc, r0, T0, C0, b0 = ppo.best_plan_stages(L, D, S, N, Ms[0], *tables, w.orderings)
    assert st == 0 and rc == 0 and res[0] == r0
    np.testing.assert_array_equal(T[0], T0)
    np.testing.assert_array_equal(C, C0)
