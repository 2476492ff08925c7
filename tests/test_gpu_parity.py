"""Bit-exact parity of the HIP path (through the C ABI) with the CPU oracle."""
import itertools
import sys

import numpy as np
import pytest

from paper_2204_10562_amd import workloads

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


def oracle_tables(ppo, w):
    rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)
    assert rc == 0
    return PF, PB, XF, XB


def sub_workload(w, idx):
    """The same problem restricted to the candidates in idx (explicit orderings)."""
    import copy
    v = copy.copy(w)
    v.orderings = np.ascontiguousarray(w.explicit_orderings()[idx])
    v.N = len(idx)
    return v


# ------------------------------------------------------------------ prefix / tables

@pytest.mark.parametrize("name", ["tiny", "transformer", "gpt", "hetero", "stress"])
def test_prefix_costs_configs(ppo, G, name):
    w = workloads.CONFIGS[name](N=64) if name in ("hetero", "stress") else workloads.CONFIGS[name]()
    say("prefix_costs", name, "L", w.L, "D", w.D)
    g = G(w)
    assert g.prefix() == 0
    PF, PB, XF, XB = oracle_tables(ppo, w)
    np.testing.assert_array_equal(g.PF.cpu().numpy(), PF)
    np.testing.assert_array_equal(g.PB.cpu().numpy(), PB)
    np.testing.assert_array_equal(g.XF.cpu().numpy(), XF)
    np.testing.assert_array_equal(g.XB.cpu().numpy(), XB)


@pytest.mark.parametrize("seed,L,D", [(1, 1, 1), (2, 2, 2), (3, 257, 3), (4, 700, 5), (5, 2048, 2), (6, 63, 9)])
def test_prefix_costs_ragged(ppo, G, seed, L, D):
    w = workloads.random_small(seed, L, D, 1, 1, zero_frac=0.1, hi_time=10 ** 6, hi_act=10 ** 9)
    say("prefix_costs ragged", seed, L, D)
    g = G(w)
    assert g.prefix() == 0
    rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)
    assert rc == 0
    for a, b in ((g.PF, PF), (g.PB, PB), (g.XF, XF), (g.XB, XB)):
        np.testing.assert_array_equal(a.cpu().numpy(), b)
    # act_bwd = NULL means "same as forward"
    assert g.prefix(actb_none=True) == 0
    rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, None, w.bw)
    np.testing.assert_array_equal(g.XB.cpu().numpy(), XB)


def test_prefix_costs_faults(ppo, G):
    base = workloads.random_small(9, 300, 3, 1, 1)
    cases = []
    a = base.bw.copy(); a[0, 2] = 0; cases.append(("bw0", dict(bw=a)))
    a = base.bw.copy(); a[2, 1] = -5; cases.append(("bwneg", dict(bw=a)))
    a = base.fwd.copy(); a[299] = -1; cases.append(("fwdneg", dict(fwd=a)))
    a = base.actf.copy(); a[17] = -1; cases.append(("actneg", dict(actf=a)))
    a = base.actf.copy(); a[299] = -1; cases.append(("act_last_ignored", dict(actf=a)))
    a = base.bwd.copy(); a[5] = 1 << 61; a[280] = 1 << 61; cases.append(("overflow", dict(bwd=a)))
    a = base.bw.copy(); a[1, 1] = -9; cases.append(("diag_ignored", dict(bw=a)))
    import copy
    for name, kw in cases:
        w = copy.copy(base)
        for k, v in kw.items():
            setattr(w, k, v)
        say("prefix fault", name)
        want = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)[0]
        assert G(w).prefix() == want, name


# ------------------------------------------------------------------ partition DP

def check_dp(ppo, g, w, tables=None, gpu_tables=False):
    PF, PB, XF, XB = tables if tables is not None else oracle_tables(ppo, w)
    if not gpu_tables:
        g.set_tables(PF, PB, XF, XB)
    st, C, bounds = g.dp()
    rc, C0, b0 = ppo.partition_dp(w.L, w.D, w.S, w.N, PF, PB, XF, XB, w.orderings)
    assert rc == 0 and st == 0
    np.testing.assert_array_equal(C, C0)
    np.testing.assert_array_equal(bounds, b0)
    return C0, b0


@pytest.mark.parametrize("name", ["tiny", "transformer", "gpt"])
def test_dp_full_configs(ppo, G, name):
    w = workloads.CONFIGS[name]()
    say("partition_dp", name, "N", w.N)
    g = G(w)
    assert g.prefix() == 0
    check_dp(ppo, g, w, gpu_tables=True)


def test_dp_explicit_orderings_equal_default(ppo, G):
    w = workloads.transformer()
    say("partition_dp explicit-vs-default transformer")
    g = G(w)
    g.prefix()
    st, C, b = g.dp()
    import torch
    o = torch.from_numpy(workloads.all_orderings(w.D).reshape(-1)).to(g.dev)
    st2, C2, b2 = g.dp(orderings=o)
    assert st == 0 and st2 == 0
    np.testing.assert_array_equal(C, C2)
    np.testing.assert_array_equal(b, b2)


def test_dp_nine_devices_default_orderings(ppo, G):
    # 9! = 362880 candidates generated on the device in lexicographic order
    import math
    w = workloads.random_small(801, 14, 9, 9, 1, hi_time=30, hi_act=2000)
    w.orderings = None
    w.N = math.factorial(9)
    say("partition_dp D=9 all orderings")
    g = G(w)
    PF, PB, XF, XB = oracle_tables(ppo, w)
    g.set_tables(PF, PB, XF, XB)
    st, C, bounds = g.dp()
    rc, C0, b0 = ppo.partition_dp(w.L, w.D, w.S, w.N, PF, PB, XF, XB, workloads.all_orderings(9))
    assert st == 0 and rc == 0
    np.testing.assert_array_equal(C, C0)
    np.testing.assert_array_equal(bounds, b0)


@pytest.mark.parametrize("name,N", [("hetero", 3000), ("stress", 600)])
def test_dp_large_shapes_subset(ppo, G, name, N):
    w = workloads.CONFIGS[name](N=N)
    say("partition_dp", name, "N", N)
    g = G(w)
    assert g.prefix() == 0
    check_dp(ppo, g, w, gpu_tables=True)


SMALL = [  # seed, L, D, S, N
    (101, 1, 1, 1, 3), (102, 2, 2, 2, 5), (103, 5, 3, 1, 7), (104, 7, 7, 7, 50), (105, 9, 4, 3, 70),
    (106, 33, 5, 5, 130), (107, 64, 6, 4, 65), (108, 65, 6, 6, 64), (109, 127, 8, 8, 100),
    (110, 128, 9, 8, 129), (111, 129, 8, 8, 100), (112, 200, 12, 12, 90), (113, 257, 16, 16, 70),
    (114, 300, 20, 3, 40), (115, 513, 33, 33, 30), (116, 1000, 64, 64, 12), (117, 16, 16, 16, 200),
]


@pytest.mark.parametrize("seed,L,D,S,N", SMALL)
def test_dp_adversarial_small(ppo, G, seed, L, D, S, N):
    # narrow ranges (ties everywhere), zero-length layers, asymmetric links, S < D
    w = workloads.random_small(seed, L, D, S, N, zero_frac=0.15, hi_time=7, hi_act=500)
    say("partition_dp small", seed, L, D, S, N)
    g = G(w)
    check_dp(ppo, g, w)


@pytest.mark.parametrize("seed,L,D,S,N,shift", [(201, 40, 4, 4, 50, 26), (202, 130, 5, 5, 40, 40), (203, 300, 6, 3, 30, 50)])
def test_dp_wide_values(ppo, G, seed, L, D, S, N, shift):
    # times too large for 32-bit keys: the int64 representation must give the same answers
    w = workloads.random_small(seed, L, D, S, N, zero_frac=0.1, hi_time=9, hi_act=300)
    w.fwd = w.fwd << shift
    w.bwd = w.bwd << shift
    w.actf = w.actf << (shift - 3)
    w.actb = w.actb << (shift - 3)
    say("partition_dp wide", seed, L, D, S, N, shift)
    g = G(w)
    check_dp(ppo, g, w)


def test_dp_key_range_boundary(ppo, G):
    # total time just below / at / above the 32-bit key limit 2^(31-K) - 1
    L, D, S, N = 16, 3, 3, 6
    K = 4
    limit = (1 << (31 - K)) - 1
    for total in (limit - 1, limit, limit + 1):
        w = workloads.random_small(301, L, D, S, N)
        w.fwd[:] = 0
        w.bwd[:] = 1
        w.bwd[0] = total - (L - 1)
        say("partition_dp boundary", total)
        g = G(w)
        check_dp(ppo, g, w)


def test_dp_bad_orderings_fault(ppo, G):
    w = workloads.random_small(401, 20, 5, 4, 64)
    PF, PB, XF, XB = oracle_tables(ppo, w)
    for mutate in ("dup", "range", "neg"):
        v = sub_workload(w, np.arange(w.N))
        if mutate == "dup":
            v.orderings[13, 2] = v.orderings[13, 0]
        elif mutate == "range":
            v.orderings[63, 3] = 5
        else:
            v.orderings[0, 0] = -1
        say("partition_dp fault", mutate)
        g = G(v)
        g.set_tables(PF, PB, XF, XB)
        st, C, b = g.dp()
        rc, C0, b0 = ppo.partition_dp(v.L, v.D, v.S, v.N, PF, PB, XF, XB, v.orderings)
        assert st == rc == ppo.FAULT_ORDERING


# ---- channel times that do not depend on the cut position (the closed-form kernel)

def ran_closed_form(g):
    """Which kernel did the last DP call's work: the closed-form one computes no rows."""
    from paper_2204_10562_amd import binding as pp
    return pp.read_workspace_stats(g.ws)["rows_executed"] == 0


@pytest.mark.parametrize("seed,L,D,S,N", SMALL)
def test_dp_equal_activations_small(ppo, G, seed, L, D, S, N):
    # ties everywhere, zero-length layers (P not strictly increasing), asymmetric links, S < D
    w = workloads.random_small(seed + 1000, L, D, S, N, zero_frac=0.15, hi_time=7, hi_act=500, same_act=True)
    say("partition_dp equal activations", seed, L, D, S, N)
    g = G(w)
    check_dp(ppo, g, w)
    assert ran_closed_form(g)


@pytest.mark.parametrize("seed,L,D,S,N", [(1201, 60, 6, 6, 90), (1202, 128, 8, 8, 200), (1203, 300, 9, 9, 64),
                                           (1204, 2048, 20, 20, 10), (1205, 90, 40, 40, 30), (1206, 700, 70, 64, 9)])
def test_dp_equal_activations_wider_times(ppo, G, seed, L, D, S, N):
    # realistic spreads: few ties, long stages, S up to 64 (one wave per workgroup), D > 64
    w = workloads.random_small(seed, L, D, S, N, hi_time=3000, hi_act=10 ** 7, same_act=True)
    say("partition_dp equal activations wide spread", seed, L, D, S, N)
    g = G(w)
    check_dp(ppo, g, w)
    assert ran_closed_form(g)


@pytest.mark.parametrize("seed,L,D,S,N,shift", [(1211, 40, 4, 4, 50, 26), (1212, 130, 5, 5, 40, 40), (1213, 300, 6, 3, 30, 50)])
def test_dp_equal_activations_times_beyond_32_bits(ppo, G, seed, L, D, S, N, shift):
    w = workloads.random_small(seed, L, D, S, N, zero_frac=0.1, hi_time=9, hi_act=300, same_act=True)
    w.fwd = w.fwd << shift
    w.bwd = w.bwd << shift
    w.actf = w.actf << (shift - 3)
    w.actb = w.actb << (shift - 3)
    say("partition_dp equal activations wide", seed, L, D, S, N, shift)
    g = G(w)
    check_dp(ppo, g, w)
    assert ran_closed_form(g)


def test_dp_equal_activations_detection(ppo, G):
    # the size after the last layer is not a boundary: it may differ; any other entry decides
    base = workloads.random_small(1221, 50, 5, 5, 80, hi_time=40, hi_act=900, same_act=True)
    import copy
    for where, flat in ((None, True), (49, True), (48, False), (0, False), (17, False)):
        for arr in ("actf", "actb"):
            w = copy.copy(base)
            a = getattr(base, arr).copy()
            if where is not None:
                a[where] += 777
            setattr(w, arr, a)
            say("partition_dp detection", where, arr, flat)
            g = G(w)
            check_dp(ppo, g, w)
            assert ran_closed_form(g) == flat, (where, arr)


def test_dp_equal_activations_all_orderings_and_faults(ppo, G):
    import math
    w = workloads.random_small(1231, 30, 7, 7, 1, hi_time=60, hi_act=5000, same_act=True)
    w.orderings = None
    w.N = math.factorial(7)
    say("partition_dp equal activations, all 7! orderings")
    g = G(w)
    check_dp(ppo, g, w)
    assert ran_closed_form(g)
    # bad rows in a caller's list raise the fault and leave the other candidates alone
    w = workloads.random_small(1232, 25, 6, 5, 200, hi_time=60, hi_act=5000, same_act=True)
    tables = oracle_tables(ppo, w)
    good = ppo.partition_dp(w.L, w.D, w.S, w.N, *tables, w.orderings)
    v = sub_workload(w, np.arange(w.N))
    v.orderings[13, 2] = v.orderings[13, 0]
    v.orderings[63, 4] = 6
    v.orderings[199, 0] = -1
    say("partition_dp equal activations, faults")
    g = G(v)
    g.set_tables(*tables)
    st, C, b = g.dp()
    assert st == ppo.FAULT_ORDERING == ppo.partition_dp(v.L, v.D, v.S, v.N, *tables, v.orderings)[0]
    keep = np.array([c for c in range(w.N) if c not in (13, 63, 199)])
    np.testing.assert_array_equal(C[keep], good[1][keep])
    np.testing.assert_array_equal(b[keep], good[2][keep])


def test_dp_work_counters(ppo, G):
    from paper_2204_10562_amd import binding as pp
    # kernel for L > 128: every row of every candidate that is computed (all of them, or one per
    # group of candidates with the same transfer times); of a row's pairs the early exit may
    # leave out those that cannot matter
    w = workloads.random_small(601, 150, 6, 5, 37)
    g = G(w)
    g.set_tables(*oracle_tables(ppo, w))
    say("work counters generic")
    assert g.dp()[0] == 0
    st = pp.read_workspace_stats(g.ws)
    L, S, N = w.L, w.S, w.N
    per = sum((L - n) * (L - n + 1) // 2 for n in range(1, S - 1)) + (L - S + 1)
    done = st["share_computed"] if st["share_active"] else N
    assert 0 < done <= N
    # (where candidates are grouped, neighbours in the sorted list also share their first rows)
    assert done <= st["rows_executed"] <= done * (S - 1)
    if not st["share_active"] and not st["share_sorted"]:
        assert st["rows_executed"] == N * (S - 1)
    assert st["rows_executed"] * (L - S + 1) // 4 < st["pairs_executed"] <= done * per
    # tiled kernel, all orderings in lexicographic order: shared rows are computed once,
    # so the count lies between one row per distinct ordering prefix and the full count
    # (one activation size changed, so that the transfer times depend on the cut position
    # and the general kernel runs)
    w = workloads.transformer()
    w.actf = w.actf.copy()
    w.actf[7] += 1 << 20
    g = G(w)
    assert g.prefix() == 0
    say("work counters tiled")
    assert g.dp()[0] == 0
    st = pp.read_workspace_stats(g.ws)
    L, S, N = w.L, w.S, w.N
    full = N * (S - 1)
    import math
    trie = sum(math.factorial(8) // math.factorial(8 - n - 1) for n in range(1, S - 1)) + N
    assert trie <= st["rows_executed"] < full // 2


# ------------------------------------------------------------------ makespan

def random_bounds(rng, N, S, L):
    b = np.empty((N, S), np.int32)
    for c in range(N):
        cuts = np.sort(rng.choice(np.arange(1, L), size=S - 1, replace=False)) if S > 1 else []
        b[c, :S - 1] = cuts
        b[c, S - 1] = L
    return b


@pytest.mark.parametrize("name", ["tiny", "transformer", "gpt"])
def test_makespan_multi_full_configs(ppo, G, name):
    # several microbatch counts in one launch, on the DP's plans of every candidate
    w = workloads.CONFIGS[name]()
    g = G(w)
    assert g.prefix() == 0
    tables = oracle_tables(ppo, w)
    rc, C0, b0 = ppo.partition_dp(w.L, w.D, w.S, w.N, *tables, w.orderings)
    assert rc == 0
    Ms = tuple(w.Ms) + (1, 3, 29)
    say("makespan_multi", name, Ms)
    st, T = g.makespan_multi(Ms, b0)
    assert st == 0
    for q, M in enumerate(Ms):
        rc, T0 = ppo.schedule_makespan(w.L, w.D, w.S, w.N, M, *tables, w.orderings, b0)
        assert rc == 0
        np.testing.assert_array_equal(T[q], T0)


@pytest.mark.parametrize("seed,L,D,S,N", [(1301, 40, 5, 5, 130), (1302, 90, 12, 12, 70), (1303, 300, 20, 20, 65),
                                           (1304, 200, 40, 33, 40), (1305, 9, 3, 1, 5)])
def test_makespan_multi_arbitrary_plans(ppo, G, seed, L, D, S, N):
    # any valid plan, every kernel family (registers, 17..32 stages, LDS columns), 1..16 counts
    w = workloads.random_small(seed, L, D, S, N, zero_frac=0.1, hi_time=30, hi_act=3000)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    rng = np.random.Generator(np.random.PCG64(seed))
    bounds = random_bounds(rng, N, S, L)
    for Ms in ((7,), (2, 50), (1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 100)):
        say("makespan_multi arbitrary", seed, L, D, S, N, Ms)
        st, T = g.makespan_multi(Ms, bounds)
        assert st == 0
        for q, M in enumerate(Ms):
            rc, T0 = ppo.schedule_makespan(L, D, S, N, M, *tables, w.orderings, bounds)
            assert rc == 0
            np.testing.assert_array_equal(T[q], T0)


@pytest.mark.parametrize("name", ["tiny", "transformer", "gpt"])
def test_makespan_full_configs(ppo, G, name):
    w = workloads.CONFIGS[name]()
    g = G(w)
    assert g.prefix() == 0
    PF, PB, XF, XB = oracle_tables(ppo, w)
    rc, C0, b0 = ppo.partition_dp(w.L, w.D, w.S, w.N, PF, PB, XF, XB, None)
    for M in w.Ms:
        say("makespan", name, "M", M)
        st, T = g.makespan(M, b0)
        rc, T0 = ppo.schedule_makespan(w.L, w.D, w.S, w.N, M, PF, PB, XF, XB, None, b0)
        assert st == 0 and rc == 0
        np.testing.assert_array_equal(T, T0)


@pytest.mark.parametrize("seed,L,D,S,N", SMALL)
def test_makespan_any_valid_plan(ppo, G, seed, L, D, S, N):
    w = workloads.random_small(seed, L, D, S, N, zero_frac=0.15, hi_time=7, hi_act=500)
    rng = np.random.Generator(np.random.PCG64(seed))
    b = random_bounds(rng, N, S, L)
    PF, PB, XF, XB = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(PF, PB, XF, XB)
    for M in (1, 2, 5, 13):
        say("makespan small", seed, L, D, S, N, "M", M)
        st, T = g.makespan(M, b)
        rc, T0 = ppo.schedule_makespan(L, D, S, N, M, PF, PB, XF, XB, w.orderings, b)
        assert st == 0 and rc == 0
        np.testing.assert_array_equal(T, T0)


@pytest.mark.parametrize("S", [2, 3, 4, 5, 6, 7, 8, 11])
def test_makespan_every_microbatch_count_around_pipeline_fill(ppo, G, S):
    # M = 1 .. 4S-1: pipelines that never fill (M < 4S-4, one specialised middle phase per M
    # for S <= 8), the boundary, and full ones
    seed, L, D, N = 700 + S, 3 * S + 7, S + 1, 150
    w = workloads.random_small(seed, L, D, S, N, zero_frac=0.1, hi_time=9, hi_act=700)
    rng = np.random.Generator(np.random.PCG64(seed))
    b = random_bounds(rng, N, S, L)
    PF, PB, XF, XB = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(PF, PB, XF, XB)
    for M in range(1, 4 * S):
        say("makespan S", S, "M", M)
        st, T = g.makespan(M, b)
        rc, T0 = ppo.schedule_makespan(L, D, S, N, M, PF, PB, XF, XB, w.orderings, b)
        assert st == 0 and rc == 0
        np.testing.assert_array_equal(T, T0)


@pytest.mark.parametrize("name,N,M", [("hetero", 500, 32), ("stress", 200, 128)])
def test_makespan_large_shapes_subset(ppo, G, name, N, M):
    w = workloads.CONFIGS[name](N=N)
    rng = np.random.Generator(np.random.PCG64(5))
    b = random_bounds(rng, N, w.S, w.L)
    g = G(w)
    assert g.prefix() == 0
    PF, PB, XF, XB = oracle_tables(ppo, w)
    say("makespan", name, N, M)
    st, T = g.makespan(M, b)
    rc, T0 = ppo.schedule_makespan(w.L, w.D, w.S, N, M, PF, PB, XF, XB, w.orderings, b)
    assert st == 0 and rc == 0
    np.testing.assert_array_equal(T, T0)


def test_makespan_faults(ppo, G):
    w = workloads.random_small(501, 20, 5, 4, 40)
    PF, PB, XF, XB = oracle_tables(ppo, w)
    rng = np.random.Generator(np.random.PCG64(1))
    good = random_bounds(rng, w.N, w.S, w.L)
    g = G(w)
    g.set_tables(PF, PB, XF, XB)
    for name, row in (("zero", [0, 5, 9, 20]), ("equal", [5, 5, 9, 20]), ("short", [3, 5, 9, 19]),
                      ("long", [3, 5, 9, 21]), ("huge", [3, 5, 1 << 20, 20]), ("desc", [9, 5, 3, 20])):
        b = good.copy()
        b[7] = row
        say("makespan fault", name)
        st, T = g.makespan(3, b)
        rc, T0 = ppo.schedule_makespan(w.L, w.D, w.S, w.N, 3, PF, PB, XF, XB, w.orderings, b)
        assert st == rc == ppo.FAULT_BOUNDS, name
    # overflow guard: (M + 4S - 4) * largest block >= 2^62
    PF2 = PF.copy(); PF2[1:] += 1 << 55
    g.set_tables(PF2, PB, XF, XB)
    for M, want in ((2, 0), (200, ppo.FAULT_OVERFLOW)):
        say("makespan overflow", M)
        st, T = g.makespan(M, good)
        rc, T0 = ppo.schedule_makespan(w.L, w.D, w.S, w.N, M, PF2, PB, XF, XB, w.orderings, good)
        assert st == rc == want
        if want == 0:
            np.testing.assert_array_equal(T, T0)


# ------------------------------------------------------------------ whole path

def check_best(ppo, g, w, M, tables):
    PF, PB, XF, XB = tables
    st, res, T, C = g.best(M)
    rc, res0, T0, C0 = ppo.best_plan(w.L, w.D, w.S, w.N, M, PF, PB, XF, XB, w.orderings)
    assert st == 0 and rc == 0
    np.testing.assert_array_equal(T, T0)
    np.testing.assert_array_equal(C, C0)
    assert res == res0
    # optional outputs may be omitted
    st, res2, _, _ = g.best(M, want_all=False)
    assert st == 0 and res2 == res0


@pytest.mark.parametrize("name", ["tiny", "transformer", "gpt"])
def test_best_plan_full_configs(ppo, G, name):
    w = workloads.CONFIGS[name]()
    g = G(w)
    assert g.prefix() == 0
    tables = oracle_tables(ppo, w)
    for M in w.Ms:
        say("best_plan", name, "M", M)
        check_best(ppo, g, w, M, tables)


@pytest.mark.parametrize("seed,L,D,S,N", SMALL)
def test_best_plan_adversarial_small(ppo, G, seed, L, D, S, N):
    w = workloads.random_small(seed, L, D, S, N, zero_frac=0.15, hi_time=7, hi_act=500)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    for M in (1, 4):
        say("best_plan small", seed, L, D, S, N, "M", M)
        check_best(ppo, g, w, M, tables)


@pytest.mark.parametrize("seed,L,D,S,N", SMALL + [(1401, 128, 8, 8, 300), (1402, 100, 30, 7, 200), (1403, 64, 32, 8, 150),
                                                    (1404, 400, 6, 6, 130), (1405, 50, 40, 8, 70), (1406, 20, 9, 2, 65)])
def test_best_plan_equal_activations(ppo, G, seed, L, D, S, N):
    # transfer times that do not depend on the cut position: for 2..8 stages the makespan kernel
    # builds the plans itself from tables in LDS (where they fit), otherwise the DP kernel does
    w = workloads.random_small(seed + 3000, L, D, S, N, zero_frac=0.15 if seed % 2 else 0.0,
                               hi_time=7 if seed < 1400 else 900, hi_act=500 if seed < 1400 else 10 ** 6, same_act=True)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    for M in (1, 4, 37):
        say("best_plan equal activations", seed, L, D, S, N, "M", M)
        check_best(ppo, g, w, M, tables)
    check_best_multi(ppo, g, w, (2, 9, 33, 70), tables)
    check_best_multi(ppo, g, w, (5, 6), tables)


def test_best_plan_equal_activations_wide_and_faults(ppo, G):
    # times beyond 32 bits: the plans come from the DP kernel (int64), the schedule runs in int64
    w = workloads.random_small(1411, 60, 6, 6, 90, zero_frac=0.1, hi_time=9, hi_act=300, same_act=True)
    w.fwd = w.fwd << 30
    w.bwd = w.bwd << 30
    w.actf = w.actf << 27
    w.actb = w.actb << 27
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("best_plan equal activations, wide")
    check_best(ppo, g, w, 5, tables)
    check_best_multi(ppo, g, w, (3, 20), tables)
    # times that fit for few microbatches but not for many: the two kernels must agree on who
    # builds the plans, for every count of the list
    w = workloads.random_small(1412, 40, 5, 5, 70, hi_time=9, hi_act=300, same_act=True)
    w.fwd = w.fwd << 18
    w.bwd = w.bwd << 18
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("best_plan equal activations, near the 32-bit bound")
    for Ms in ((1,), (2, 3), (40, 1), (3000,)):
        check_best_multi(ppo, g, w, Ms, tables)
    # bad rows in a caller's list: the fault is raised, the other candidates are right
    w = workloads.random_small(1413, 25, 6, 5, 200, hi_time=60, hi_act=5000, same_act=True)
    tables = oracle_tables(ppo, w)
    rc, res0, T0, C0 = ppo.best_plan(w.L, w.D, w.S, w.N, 6, *tables, w.orderings)
    v = sub_workload(w, np.arange(w.N))
    v.orderings[13, 2] = v.orderings[13, 0]
    v.orderings[63, 4] = 6
    v.orderings[199, 0] = -1
    g = G(v)
    g.set_tables(*tables)
    say("best_plan equal activations, faults")
    st, res, T, C = g.best(6)
    assert st == ppo.FAULT_ORDERING
    keep = np.array([c for c in range(w.N) if c not in (13, 63, 199)])
    np.testing.assert_array_equal(T[keep], T0[keep])
    np.testing.assert_array_equal(C[keep], C0[keep])
    big = np.iinfo(np.int64).max
    assert (T[[13, 63, 199]] == big).all() and (C[[13, 63, 199]] == big).all()
    if res0["best_index"] in keep:
        assert res == res0


def test_best_plan_ties_lowest_index(ppo, G):
    w = workloads.tiny()
    w.bw = np.full((4, 4), 16000, np.int64)
    say("best_plan ties")
    g = G(w)
    assert g.prefix() == 0
    tables = oracle_tables(ppo, w)
    st, res, T, C = g.best(8)
    assert (T == T[0]).all() and res["best_index"] == 0 and res["order"] == [0, 1, 2, 3]
    check_best(ppo, g, w, 8, tables)
    # duplicated candidates: the first copy wins
    v = sub_workload(w, np.array([5, 3, 5, 3, 0, 0]))
    g = G(v)
    g.set_tables(*tables)
    check_best(ppo, g, v, 4, tables)


@pytest.mark.parametrize("name,N", [("hetero", 2000), ("stress", 300)])
def test_best_plan_large_shapes_subset(ppo, G, name, N):
    w = workloads.CONFIGS[name](N=N)
    g = G(w)
    assert g.prefix() == 0
    tables = oracle_tables(ppo, w)
    say("best_plan", name, N)
    check_best(ppo, g, w, w.Ms[-1], tables)


def check_best_multi(ppo, g, w, Ms, tables):
    PF, PB, XF, XB = tables
    st, res, T, C = g.best_multi(Ms)
    assert st == 0
    for q, M in enumerate(Ms):
        rc, res0, T0, C0 = ppo.best_plan(w.L, w.D, w.S, w.N, M, PF, PB, XF, XB, w.orderings)
        assert rc == 0
        np.testing.assert_array_equal(T[q], T0)
        np.testing.assert_array_equal(C, C0)
        assert res[q] == res0
    st, res2, _, _ = g.best_multi(Ms, want_all=False)
    assert st == 0 and res2 == res


@pytest.mark.parametrize("name", ["tiny", "transformer", "gpt"])
def test_best_plan_multi_full_configs(ppo, G, name):
    w = workloads.CONFIGS[name]()
    g = G(w)
    assert g.prefix() == 0
    say("best_plan_multi", name, w.Ms)
    check_best_multi(ppo, g, w, w.Ms, oracle_tables(ppo, w))


@pytest.mark.parametrize("Ms", [(7,), (3, 40), (40, 3, 9), (5, 6, 7, 8), (2, 30, 4, 50, 6),
                                (9, 8, 7, 6, 5, 4), (1, 1, 33, 33, 2, 2, 64)])
def test_best_plan_multi_list_lengths(ppo, G, Ms):
    # the waves of a workgroup share one gather for up to four counts: whole and partial groups
    w = workloads.random_small(811, 40, 7, 6, 333, zero_frac=0.1, hi_time=9, hi_act=900)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("best_plan_multi list", Ms)
    check_best_multi(ppo, g, w, Ms, tables)


@pytest.mark.parametrize("N", [16384 + 64, 16384 + 337, 3 * 16384 + 129])
def test_best_plan_multi_many_candidates_four_counts(ppo, G, N):
    # more groups of 64 candidates than compute units and four counts: workgroups of three
    # groups, the last one partly or wholly past the end of the list
    w = workloads.random_small(823, 24, 6, 5, N, zero_frac=0.1, hi_time=9, hi_act=900)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("best_plan_multi many candidates", N)
    check_best_multi(ppo, g, w, (70, 3, 30, 9), tables)


@pytest.mark.parametrize("S", [1, 2, 3, 8])
def test_best_plan_multi_many_candidates_stage_counts(ppo, G, S):
    N = 16384 + 64 * 7 + 5
    w = workloads.random_small(830 + S, 20, 8, S, N, zero_frac=0.1, hi_time=9, hi_act=900)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("best_plan_multi many candidates, S", S)
    check_best_multi(ppo, g, w, (5, 41, 2, 17), tables)


@pytest.mark.parametrize("seed,L,D,S,N", SMALL)
def test_best_plan_multi_adversarial_small(ppo, G, seed, L, D, S, N):
    w = workloads.random_small(seed, L, D, S, N, zero_frac=0.15, hi_time=7, hi_act=500)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    Ms = (1, 2, 3, 5, 8, 13, 21, 34, 55, 89, 144, 4, 6, 7, 9, 10)  # 16 = the most one call takes
    say("best_plan_multi small", seed, L, D, S, N)
    check_best_multi(ppo, g, w, Ms, tables)


def test_best_plan_multi_overflow_is_per_M(ppo, G):
    w = workloads.random_small(701, 20, 5, 4, 40)
    PF, PB, XF, XB = oracle_tables(ppo, w)
    PF2 = PF.copy(); PF2[1:] += 1 << 55
    g = G(w)
    g.set_tables(PF2, PB, XF, XB)
    say("best_plan_multi overflow")
    st, res, T, C = g.best_multi((2, 200))
    assert st == ppo.FAULT_OVERFLOW
    rc, res0, T0, C0 = ppo.best_plan(w.L, w.D, w.S, w.N, 2, PF2, PB, XF, XB, w.orderings)
    assert rc == 0 and res[0] == res0
    np.testing.assert_array_equal(T[0], T0)


# ------------------------------------------------------------------ full benchmark sizes

def plan_resource_times(w, PF, PB, XF, XB, orderings, bounds):
    """Largest per-resource time (stage f+b, channel cf+cb) of every plan, vectorised."""
    N, S = bounds.shape
    P = PF + PB
    e = np.concatenate([np.zeros((N, 1), np.int64), bounds.astype(np.int64)], axis=1)
    comp = P[e[:, 1:]] - P[e[:, :-1]]
    worst = comp.max(axis=1)
    if S > 1:
        link = orderings[:, :-1].astype(np.int64) * w.D + orderings[:, 1:].astype(np.int64)
        at = link * w.L + (e[:, 1:-1] - 1)
        chan = XF[at] + XB[at]
        worst = np.maximum(worst, chan.max(axis=1))
    return worst


@pytest.mark.parametrize("name,stride", [("gpt", 1)])
def test_whole_path_at_full_size(ppo, G, name, stride):
    """The launch configuration bench.py times: properties that hold for every candidate, and
    the oracle on every candidate.  (The two large configurations: test_gpu_full_size.py.)"""
    w = workloads.CONFIGS[name]()
    say("full size", name, "N", w.N)
    g = G(w)
    assert g.prefix() == 0
    PF, PB, XF, XB = oracle_tables(ppo, w)
    for a, b in ((g.PF, PF), (g.PB, PB), (g.XF, XF), (g.XB, XB)):
        np.testing.assert_array_equal(a.cpu().numpy(), b)
    M = w.Ms[-1]
    st, C, bounds = g.dp()
    assert st == 0
    st, res, T, C2 = g.best(M)
    assert st == 0
    np.testing.assert_array_equal(C, C2)
    orderings = w.explicit_orderings()
    N, S, L = w.N, w.S, w.L
    # every plan is a valid partition and C is its largest per-resource time
    assert (bounds[:, -1] == L).all() and (bounds[:, 0] >= 1).all()
    assert (np.diff(bounds.astype(np.int64), axis=1) >= 1).all()
    np.testing.assert_array_equal(plan_resource_times(w, PF, PB, XF, XB, orderings, bounds), C)
    total = int(PF[-1] + PB[-1])
    assert (C >= -(-total // S)).all()
    # Lemma 1: M*C <= T <= (M + 4S - 4)*C
    assert (T >= M * C).all() and (T <= (M + 4 * S - 4) * C).all()
    # the winner is the lowest index among the smallest T
    best = int(np.argmin(T))
    assert res["best_index"] == best and res["T"] == int(T[best]) and res["C"] == int(C[best])
    assert res["bounds"] == bounds[best].tolist() and res["order"] == orderings[best].tolist()
    # oracle on a sample
    idx = np.unique(np.concatenate([np.arange(0, N, stride), [best], np.argsort(T, kind="stable")[:64]]))
    sub = np.ascontiguousarray(orderings[idx])
    rc, C0, b0 = ppo.partition_dp(L, w.D, S, len(idx), PF, PB, XF, XB, sub)
    assert rc == 0
    np.testing.assert_array_equal(C[idx], C0)
    np.testing.assert_array_equal(bounds[idx], b0)
    rc, T0 = ppo.schedule_makespan(L, w.D, S, len(idx), M, PF, PB, XF, XB, sub, b0)
    assert rc == 0
    np.testing.assert_array_equal(T[idx], T0)


@pytest.mark.parametrize("seed,L,D,S,N,shift", [(811, 40, 20, 20, 70, 0), (812, 70, 32, 32, 40, 0), (813, 30, 17, 17, 65, 0),
                                                  (814, 40, 20, 20, 70, 24), (815, 64, 25, 24, 33, 30)])
def test_best_plan_between_17_and_32_stages(ppo, G, seed, L, D, S, N, shift):
    # 32-bit times: finish times in registers; larger times: the LDS kernel, chosen on the device
    w = workloads.random_small(seed, L, D, S, N, zero_frac=0.1, hi_time=9, hi_act=300)
    if shift:
        w.fwd = w.fwd << shift
        w.bwd = w.bwd << shift
        w.actf = w.actf << (shift - 3)
        w.actb = w.actb << (shift - 3)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    for M in (1, 7, 60):
        say("best_plan 17..32 stages", seed, L, D, S, N, "shift", shift, "M", M)
        check_best(ppo, g, w, M, tables)
    check_best_multi(ppo, g, w, (3, 50), tables)


@pytest.mark.parametrize("seed", range(900, 960))
def test_whole_path_random_shapes(ppo, G, seed):
    # shapes drawn at random: every tile count of the L <= 128 kernel, ragged super-rows of the
    # L > 128 kernel, S from 1 to D, caller's lists and all D! orderings
    rng = np.random.Generator(np.random.PCG64(seed))
    L = int(rng.integers(1, 129)) if seed % 3 else int(rng.integers(129, 420))
    D = int(rng.integers(1, 10))
    S = int(rng.integers(1, min(L, D) + 1))
    N = int(rng.integers(1, 160))
    w = workloads.random_small(seed, L, D, S, N, zero_frac=0.1 if seed % 2 else 0.0, hi_time=int(rng.integers(2, 200)),
                               hi_act=int(rng.integers(1, 5000)))
    if S == D and D <= 5 and seed % 4 == 0:
        import math
        w.orderings = None
        w.N = math.factorial(D)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("random shape", seed, "L", L, "D", D, "S", S, "N", w.N)
    check_dp(ppo, g, w)
    Ms = (int(rng.integers(1, 5)), int(rng.integers(5, 80)))
    check_best_multi(ppo, g, w, Ms, tables)


@pytest.mark.parametrize("seed,L,D,S,N,hi", [(1501, 60, 20, 20, 300, 2 * 10 ** 6), (1502, 90, 32, 32, 200, 10 ** 6),
                                             (1503, 40, 17, 17, 130, 4 * 10 ** 6), (1504, 50, 24, 24, 64, 50)])
def test_makespan_17_to_32_stages_without_workspace(ppo, G, seed, L, D, S, N, hi):
    # pp_schedule_makespan has no workspace header that says whether the times fit 32 bits: every
    # block of 64 candidates is scheduled by the register kernel if all of its plans fit and by
    # the 64-bit kernel otherwise.  Layer times chosen so that a launch holds both kinds.
    w = workloads.random_small(seed, L, D, S, N, hi_time=hi, hi_act=hi * 40)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    rng = np.random.Generator(np.random.PCG64(seed))
    bounds = random_bounds(rng, N, S, L)
    for Ms in ((50,), (3, 400)):
        say("makespan 17..32 stages, no workspace", seed, L, D, S, N, Ms)
        st, T = g.makespan_multi(Ms, bounds)
        assert st == 0
        fits = 0
        for q, M in enumerate(Ms):
            rc, T0 = ppo.schedule_makespan(L, D, S, N, M, *tables, w.orderings, bounds)
            assert rc == 0
            np.testing.assert_array_equal(T[q], T0)
            fits += int((T0 < 2 ** 31).sum())
        if hi > 50:
            assert 0 < fits < N * len(Ms)  # some schedules fit 32 bits and some do not
