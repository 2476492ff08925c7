"""Bit-exact parity of the stage-count search (pp_partition_dp_stages, pp_best_plan_stages)
with the CPU oracle, through the C ABI."""
import sys

import numpy as np
import pytest

from paper_2204_10562_amd import workloads
from test_gpu_parity import SMALL, oracle_tables, sub_workload

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


def check_stages(ppo, g, w, Ms, tables):
    """Every (candidate, stage count) entry and every winner against the oracle."""
    PF, PB, XF, XB = tables
    st, C, bounds = g.dp_stages()
    assert st == 0
    st, res, T, C2 = g.best_stages(Ms)
    assert st == 0
    np.testing.assert_array_equal(C, C2)
    for q, M in enumerate(Ms):
        rc, res0, T0, C0, b0 = ppo.best_plan_stages(w.L, w.D, w.S, w.N, M, PF, PB, XF, XB, w.orderings)
        assert rc == 0
        if q == 0:
            np.testing.assert_array_equal(C, C0)
            np.testing.assert_array_equal(bounds, b0)
        np.testing.assert_array_equal(T[q], T0)
        assert res[q] == res0
    st, res2, _, _ = g.best_stages(Ms, want_all=False)
    assert st == 0 and res2 == res
    return res


@pytest.mark.parametrize("name", ["tiny", "transformer", "gpt"])
def test_stages_full_configs(ppo, G, name):
    w = workloads.CONFIGS[name]()
    g = G(w)
    assert g.prefix() == 0
    Ms = w.Ms if name != "gpt" else w.Ms[:2]
    say("stages", name, Ms)
    check_stages(ppo, g, w, Ms, oracle_tables(ppo, w))


@pytest.mark.parametrize("seed,L,D,S,N", SMALL)
def test_stages_adversarial_small(ppo, G, seed, L, D, S, N):
    w = workloads.random_small(seed, L, D, S, N, zero_frac=0.15, hi_time=7, hi_act=500)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("stages small", seed, L, D, S, N)
    check_stages(ppo, g, w, (1, 5, 40), tables)


@pytest.mark.parametrize("seed,L,D,S,N", SMALL)
def test_stages_equal_activations_small(ppo, G, seed, L, D, S, N):
    # transfer times that do not depend on the cut position: the closed-form DP kernel
    w = workloads.random_small(seed + 2000, L, D, S, N, zero_frac=0.15, hi_time=7, hi_act=500, same_act=True)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("stages equal activations", seed, L, D, S, N)
    check_stages(ppo, g, w, (1, 5, 40), tables)
    from paper_2204_10562_amd import binding as pp
    assert pp.read_workspace_stats(g.ws)["rows_executed"] == 0


@pytest.mark.parametrize("seed,L,D,S,N,shift", [(211, 40, 4, 4, 50, 26), (212, 130, 5, 5, 40, 40)])
def test_stages_wide_values(ppo, G, seed, L, D, S, N, shift):
    # times too large for 32-bit keys: the int64 representation
    w = workloads.random_small(seed, L, D, S, N, zero_frac=0.1, hi_time=9, hi_act=300)
    w.fwd = w.fwd << shift
    w.bwd = w.bwd << shift
    w.actf = w.actf << (shift - 3)
    w.actb = w.actb << (shift - 3)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("stages wide", seed, L, D, S, N, shift)
    check_stages(ppo, g, w, (3,), tables)


@pytest.mark.parametrize("name,N", [("hetero", 1500), ("stress", 200)])
def test_stages_large_shapes_subset(ppo, G, name, N):
    w = workloads.CONFIGS[name](N=N)
    g = G(w)
    assert g.prefix() == 0
    say("stages", name, N)
    check_stages(ppo, g, w, w.Ms[-1:], oracle_tables(ppo, w))


def test_stages_last_column_is_the_fixed_count_result(ppo, G):
    w = workloads.transformer()
    g = G(w)
    assert g.prefix() == 0
    say("stages last column")
    st, res, T, C = g.best_stages((8,))
    st2, C1, b1 = g.dp()
    st3, Cs, bs = g.dp_stages()
    assert st == 0 and st2 == 0 and st3 == 0
    S = w.S
    np.testing.assert_array_equal(Cs[:, S - 1], C1)
    np.testing.assert_array_equal(bs[:, S * (S - 1) // 2:], b1)
    st4, fixed, T1, _ = g.best(8)
    np.testing.assert_array_equal(T[0][:, S - 1], T1)
    assert res[0]["T"] <= fixed["T"]


def test_stages_ties_lowest_candidate_then_fewest_stages(ppo, G):
    # zero-cost trailing layers and free links: every (candidate, stage count) has the same T
    L = 4
    w = workloads.random_small(901, L, 3, 3, 6)
    w.orderings = None
    w.fwd = np.array([5, 0, 0, 0], np.int64)
    w.bwd = np.array([5, 0, 0, 0], np.int64)
    w.actf = np.zeros(L, np.int64)
    w.actb = np.zeros(L, np.int64)
    w.bw = np.full((3, 3), 10, np.int64)
    g = G(w)
    assert g.prefix() == 0
    say("stages ties")
    res = check_stages(ppo, g, w, (5,), oracle_tables(ppo, w))
    assert res[0]["best_index"] == 0 and res[0]["S"] == 1 and res[0]["T"] == 50


def test_stages_bad_orderings_fault(ppo, G):
    w = workloads.random_small(402, 20, 5, 4, 64)
    tables = oracle_tables(ppo, w)
    for L2, mutate in ((20, "dup"), (20, "range")):
        v = sub_workload(w, np.arange(w.N))
        if mutate == "dup":
            v.orderings[13, 3] = v.orderings[13, 0]
        else:
            v.orderings[63, 1] = 5
        say("stages fault", mutate)
        g = G(v)
        g.set_tables(*tables)
        st, C, b = g.dp_stages()
        assert st == ppo.FAULT_ORDERING
        # the other candidates are unaffected
        rc, res0, T0, C0, b0 = ppo.best_plan_stages(w.L, w.D, w.S, w.N, 2, *tables, w.orderings)
        keep = np.array([c for c in range(w.N) if c not in (13, 63)])
        np.testing.assert_array_equal(C[keep], C0[keep])
        np.testing.assert_array_equal(b[keep], b0[keep])


@pytest.mark.parametrize("name,stride", [("hetero", 101), ("stress", 16411)])
def test_stages_at_full_size(ppo, G, name, stride):
    """Full-size launch: the oracle on every stride-th candidate and on the winner."""
    w = workloads.CONFIGS[name]()
    say("stages full size", name, "N", w.N)
    g = G(w)
    assert g.prefix() == 0
    tables = oracle_tables(ppo, w)
    Ms = w.Ms[-1:]
    st, res, T, C = g.best_stages(Ms)
    assert st == 0
    win = res[0]["best_index"]
    idx = np.unique(np.concatenate([np.arange(0, w.N, stride), [win]]))
    v = sub_workload(w, idx)
    rc, res0, T0, C0, b0 = ppo.best_plan_stages(v.L, v.D, v.S, v.N, Ms[0], *tables, v.orderings)
    assert rc == 0
    np.testing.assert_array_equal(T[0][idx], T0)
    np.testing.assert_array_equal(C[idx], C0)
    # the winner: nothing anywhere is smaller, nothing earlier is equal
    S = w.S
    flat = T[0].reshape(-1)
    at = win * S + res[0]["S"] - 1
    assert flat[at] == res[0]["T"] == flat.min()
    assert at == int(np.flatnonzero(flat == flat.min())[0])
    pos = int(np.searchsorted(idx, win))
    xi = res[0]["S"]
    assert res[0]["bounds"] == b0[pos, xi * (xi - 1) // 2: xi * (xi + 1) // 2].tolist()
    assert res[0]["order"] == v.orderings[pos, :xi].tolist()
    assert res[0]["C"] == C0[pos, xi - 1]


@pytest.mark.parametrize("seed", range(960, 990))
def test_stages_random_shapes(ppo, G, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    L = int(rng.integers(1, 129)) if seed % 3 else int(rng.integers(129, 300))
    D = int(rng.integers(1, 10))
    S = int(rng.integers(1, min(L, D) + 1))
    N = int(rng.integers(1, 120))
    w = workloads.random_small(seed, L, D, S, N, zero_frac=0.1 if seed % 2 else 0.0, hi_time=int(rng.integers(2, 200)),
                               hi_act=int(rng.integers(1, 5000)))
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    say("stages random", seed, "L", L, "D", D, "S", S, "N", N)
    check_stages(ppo, g, w, (int(rng.integers(1, 6)), int(rng.integers(6, 70))), tables)
