"""Bit-exact parity of pp_schedule_makespan_variant (comparison schedules) with the oracle."""
import sys

import numpy as np
import pytest

from paper_2204_10562_amd import workloads
from test_gpu_parity import SMALL, oracle_tables

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


def random_bounds(rng, N, S, L):
    b = np.empty((N, S), np.int32)
    for c in range(N):
        b[c, :S - 1] = np.sort(rng.choice(np.arange(1, L), size=S - 1, replace=False)) if S > 1 else []
        b[c, S - 1] = L
    return b


@pytest.mark.parametrize("seed,L,D,S,N", SMALL)
def test_variants_adversarial_small(ppo, G, seed, L, D, S, N):
    w = workloads.random_small(seed, L, D, S, N, zero_frac=0.15, hi_time=7, hi_act=500)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    bounds = random_bounds(np.random.Generator(np.random.PCG64(seed)), N, S, L)
    for variant in (0, 1, 2, 3, 4):
        for M in (1, 3, 40):
            say("variant", variant, "small", seed, L, D, S, N, "M", M)
            st, T = g.makespan_variant(variant, M, bounds)
            rc, T0 = ppo.schedule_makespan_variant(variant, L, D, S, N, M, *tables, w.orderings, bounds)
            assert st == 0 and rc == 0
            np.testing.assert_array_equal(T, T0)


@pytest.mark.parametrize("name", ["tiny", "transformer", "gpt"])
def test_variants_on_the_dp_plans(ppo, G, name):
    w = workloads.CONFIGS[name]()
    g = G(w)
    assert g.prefix() == 0
    tables = oracle_tables(ppo, w)
    st, C, bounds = g.dp()
    assert st == 0
    M = w.Ms[-1]
    st, T_pe = g.makespan(M, bounds)
    for variant in (0, 1, 2, 3, 4):
        say("variant", variant, name, "M", M)
        st, T = g.makespan_variant(variant, M, bounds)
        rc, T0 = ppo.schedule_makespan_variant(variant, w.L, w.D, w.S, w.N, M, *tables, w.orderings, bounds)
        assert st == 0 and rc == 0
        np.testing.assert_array_equal(T, T0)
        if variant == 0:
            np.testing.assert_array_equal(T, T_pe)


def test_variants_large_shapes_subset(ppo, G):
    for name, N in (("hetero", 1000), ("stress", 150)):
        w = workloads.CONFIGS[name](N=N)
        g = G(w)
        assert g.prefix() == 0
        tables = oracle_tables(ppo, w)
        st, C, bounds = g.dp()
        for variant in (1, 2, 3, 4):
            say("variant", variant, name, N)
            st, T = g.makespan_variant(variant, w.Ms[-1], bounds)
            rc, T0 = ppo.schedule_makespan_variant(variant, w.L, w.D, w.S, w.N, w.Ms[-1], *tables, w.orderings, bounds)
            assert st == 0 and rc == 0
            np.testing.assert_array_equal(T, T0)


def test_variants_faults(ppo, G):
    w = workloads.random_small(451, 20, 5, 4, 32)
    tables = oracle_tables(ppo, w)
    g = G(w)
    g.set_tables(*tables)
    bounds = random_bounds(np.random.Generator(np.random.PCG64(4)), 32, 4, 20)
    bad = bounds.copy(); bad[7, 1] = bad[7, 0]
    for variant in (1, 2, 3, 4):
        say("variant fault", variant)
        st, T = g.makespan_variant(variant, 3, bad)
        rc, T0 = ppo.schedule_makespan_variant(variant, 20, 5, 4, 32, 3, *tables, w.orderings, bad)
        assert st == rc == ppo.FAULT_BOUNDS
    from paper_2204_10562_amd import binding as pp
    import torch
    T = torch.empty(32, dtype=torch.int64, device=g.dev)
    b = torch.from_numpy(bounds.reshape(-1)).to(g.dev)
    with pytest.raises(pp.PPError):
        pp.pp_schedule_makespan_variant(9, 20, 5, 4, 32, 3, g.PF, g.PB, g.XF, g.XB, g.orderings, b, T, g.status)
