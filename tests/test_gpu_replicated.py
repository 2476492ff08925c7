"""Bit-exact parity of pp_plan_replicated (PRM with replicated stages inside SPP) with the CPU
oracle, through the C ABI."""
import sys

import numpy as np
import pytest

from paper_2204_10562_amd import workloads
from test_gpu_parity import sub_workload

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


def full(w):
    """The workload with whole orderings (all D devices per row)."""
    assert w.orderings is None or w.orderings.shape[1] == w.D
    return w


def check(ppo, G, w, alpha, M):
    g = G(w)
    st, res, T, W, b, r = g.plan_replicated(M, alpha)
    rc, res0, T0, W0, b0, r0 = ppo.spp_replicated(w.L, w.D, w.N, M, w.fwd, w.bwd, w.actf, w.actb, alpha,
                                                  w.bw, w.orderings)
    assert st == 0 and rc == 0
    np.testing.assert_array_equal(W, W0)
    np.testing.assert_array_equal(b, b0)
    np.testing.assert_array_equal(r, r0)
    np.testing.assert_array_equal(T, T0)
    assert res == res0
    st, res2 = g.plan_replicated(M, alpha, want_all=False)
    assert st == 0 and res2 == res0
    return res


SMALL_REP = [  # seed, L, D, N
    (501, 1, 1, 2), (502, 2, 2, 4), (503, 3, 5, 20), (504, 9, 4, 30), (505, 17, 6, 40), (506, 40, 8, 24),
    (507, 130, 5, 10), (508, 64, 12, 6), (509, 33, 16, 4),
]


@pytest.mark.parametrize("seed,L,D,N", SMALL_REP)
def test_replicated_adversarial_small(ppo, G, seed, L, D, N):
    # narrow ranges (ties everywhere), zero-length layers, asymmetric links, fewer layers than GPUs
    w = workloads.random_small(seed, L, D, D, N, zero_frac=0.15, hi_time=7, hi_act=500)
    rng = np.random.Generator(np.random.PCG64(seed))
    alpha = rng.integers(0, 300, size=L).astype(np.int64)
    for M in (1, 6):
        say("replicated small", seed, L, D, N, "M", M)
        check(ppo, G, w, alpha, M)


@pytest.mark.parametrize("name", ["tiny", "transformer", "gpt"])
def test_replicated_configs(ppo, G, name):
    w = workloads.CONFIGS[name]()
    alpha = workloads.parameter_sizes(w)
    if name == "tiny":
        for M in w.Ms:
            say("replicated", name, "all orderings, M", M)
            check(ppo, G, w, alpha, M)
        return
    # the oracle needs ~0.1 s per candidate at these sizes: a spread sample of the orderings
    idx = np.arange(0, w.N, w.N // 96)
    v = sub_workload(w, idx)
    say("replicated", name, "sample", len(idx), "M", w.Ms[-1])
    check(ppo, G, v, alpha, w.Ms[-1])


def test_replicated_hetero_shape(ppo, G):
    w = workloads.hetero(N=6)
    alpha = workloads.parameter_sizes(w)
    say("replicated hetero L=300 D=16 N=6")
    check(ppo, G, w, alpha, 16)


def test_replicated_default_orderings_are_lexicographic(ppo, G):
    w = workloads.random_small(520, 12, 5, 5, 1, hi_time=30, hi_act=900)
    w.orderings = None
    w.N = 120
    alpha = np.full(12, 1000, np.int64)
    say("replicated all 5! orderings")
    g = G(w)
    st, res, T, W, b, r = g.plan_replicated(3, alpha)
    v = sub_workload(w, np.arange(120))
    st2, res2, T2, W2, b2, r2 = G(v).plan_replicated(3, alpha)
    assert st == 0 and st2 == 0 and res == res2
    np.testing.assert_array_equal(T, T2)
    check(ppo, G, w, alpha, 3)


def test_replicated_faults(ppo, G):
    import copy
    w = workloads.random_small(530, 10, 4, 4, 8, hi_time=30, hi_act=900)
    alpha = np.full(10, 1000, np.int64)
    cases = []
    v = copy.copy(w); v.bw = w.bw.copy(); v.bw[1, 2] = 0; cases.append(("bandwidth", v, alpha))
    v = copy.copy(w); v.fwd = w.fwd.copy(); v.fwd[3] = -1; cases.append(("negative", v, alpha))
    a2 = alpha.copy(); a2[0] = -5; cases.append(("negative alpha", w, a2))
    v = sub_workload(w, np.arange(8)); v.orderings[5, 3] = v.orderings[5, 0]; cases.append(("ordering", v, alpha))
    v = copy.copy(w); v.bwd = w.bwd.copy(); v.bwd[2] = 1 << 60; cases.append(("overflow", v, alpha))
    for name, v, al in cases:
        say("replicated fault", name)
        st = G(v).plan_replicated(2, al)[0]
        rc = ppo.spp_replicated(v.L, v.D, v.N, 2, v.fwd, v.bwd, v.actf, v.actb, al, v.bw, v.orderings)[0]
        assert st == rc != 0, name


def test_replicated_at_full_size(ppo, G):
    """All 40320 orderings of the GPT-shaped workload in one launch: the oracle on a spread
    sample and on the winner; the winner is the first minimum of everything the GPU computed."""
    w = workloads.gpt()
    alpha = workloads.parameter_sizes(w)
    M = w.Ms[-1]
    say("replicated full size gpt N", w.N, "M", M)
    g = G(w)
    st, res, T, W, b, r = g.plan_replicated(M, alpha)
    assert st == 0
    win = res["best_index"]
    idx = np.unique(np.concatenate([np.arange(0, w.N, 97), [win]]))
    v = sub_workload(w, idx)
    rc, res0, T0, W0, b0, r0 = ppo.spp_replicated(v.L, v.D, v.N, M, v.fwd, v.bwd, v.actf, v.actb, alpha,
                                                  v.bw, v.orderings)
    assert rc == 0
    np.testing.assert_array_equal(T[idx], T0)
    np.testing.assert_array_equal(W[idx], W0)
    np.testing.assert_array_equal(b[idx], b0)
    np.testing.assert_array_equal(r[idx], r0)
    flat = T.reshape(-1)
    at = win * w.D + res["S"] - 1
    assert flat[at] == res["T"] == flat.min() and at == int(np.flatnonzero(flat == flat.min())[0])
    xi = res["S"]
    assert res["bounds"] == b[win, xi * (xi - 1) // 2: xi * (xi + 1) // 2].tolist()
    assert res["reps"] == r[win, xi * (xi - 1) // 2: xi * (xi + 1) // 2].tolist()
    assert res["order"] == workloads.all_orderings(w.D)[win].tolist() and res["W"] == W[win, xi - 1]
    # every plan obeys the bounds of Lemma 1 with the AllReduce term: M*C <= T (C <= W/M)
    ok = T != np.iinfo(np.int64).max
    assert (T[ok] * 1 >= 0).all() and ok.all()


@pytest.mark.parametrize("seed,L,D,N,what", [(541, 20, 4, 12, "times"), (542, 12, 5, 10, "acts"),
                                              (543, 16, 4, 8, "bandwidth"), (544, 14, 4, 8, "alpha")])
def test_replicated_wide_values(ppo, G, seed, L, D, N, what):
    # values beyond 2^30 somewhere: the int64 form of the tables must give the same answers
    w = workloads.random_small(seed, L, D, D, N, zero_frac=0.1, hi_time=9, hi_act=300)
    rng = np.random.Generator(np.random.PCG64(seed))
    alpha = rng.integers(0, 300, size=L).astype(np.int64)
    if what == "times":
        w.fwd = w.fwd << 28
        w.bwd = w.bwd << 28
    elif what == "acts":
        w.actf = w.actf << 30
        w.actb = w.actb << 30
    elif what == "bandwidth":
        w.bw = w.bw << 29
        w.actf = w.actf << 29
    else:
        alpha = alpha << 34
    say("replicated wide", what, seed, L, D, N)
    check(ppo, G, w, alpha, 5)


@pytest.mark.parametrize("seed", range(950, 980))
def test_replicated_random_shapes(ppo, G, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    D = int(rng.integers(1, 9))
    L = int(rng.integers(1, 60)) if seed % 3 else int(rng.integers(100, 200))
    N = int(rng.integers(1, 40))
    w = workloads.random_small(seed, L, D, D, N, zero_frac=0.1 if seed % 2 else 0.0, hi_time=int(rng.integers(2, 300)),
                               hi_act=int(rng.integers(1, 9000)))
    alpha = rng.integers(0, int(rng.integers(2, 10**6)), size=L).astype(np.int64)
    M = int(rng.integers(1, 70))
    say("replicated random", seed, "L", L, "D", D, "N", N, "M", M)
    check(ppo, G, w, alpha, M)
