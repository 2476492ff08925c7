"""The recursive device ordering (Alg. 2) as a candidate of the batched evaluation (Alg. 3
evaluates it first): pp_rdo_order's row for the cluster of every configuration, run through
pp_best_plan_multi as a one-row candidate list and as row 0 in front of a sampled list, against
ppo_rdo_order + ppo_best_plan."""
import sys

import numpy as np
import pytest

from paper_2204_10562_amd import workloads
from test_gpu_parity import oracle_tables

pytestmark = pytest.mark.gpu


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


def small(name):
    make = workloads.CONFIGS[name]
    if name in ("hetero", "stress"):
        return make(N=300)
    w = make()
    if w.N > 300:  # a spread sample of the D! orderings
        w.orderings = np.ascontiguousarray(w.explicit_orderings()[::w.N // 300])
        w.N = len(w.orderings)
    return w


@pytest.mark.parametrize("name", ["tiny", "transformer", "gpt", "hetero", "stress"])
def test_rdo_row_as_candidate(ppo, name):
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2204_10562_amd import problem
    w = small(name)
    row = problem.rdo_row(w)
    assert row.tolist() == ppo.rdo_order(w.bw)[:w.S]
    tables = oracle_tables(ppo, w)
    L, D, S = w.L, w.D, w.S
    say("rdo row", name, row.tolist())

    # the row alone
    one = problem.with_first_candidate(w, row)
    one.orderings, one.N = np.ascontiguousarray(one.orderings[:1]), 1
    g = problem.GpuProblem(one)
    assert g.prefix() == 0
    st, res, T, C = g.best_multi(w.Ms)
    assert st == 0
    st, C1, b1 = g.dp()
    assert st == 0
    for q, M in enumerate(w.Ms):
        rc, res0, T0, C0 = ppo.best_plan(L, D, S, 1, M, *tables, one.orderings)
        assert rc == 0 and res[q] == res0 and res0["best_index"] == 0 and res0["order"] == row.tolist()
        np.testing.assert_array_equal(T[q], T0)
        np.testing.assert_array_equal(C, C0)
        assert b1[0].tolist() == res0["bounds"]

    # the row in front of the candidate list
    v = problem.with_first_candidate(w, row)
    g = problem.GpuProblem(v)
    assert g.prefix() == 0
    st, res, T, C = g.best_multi(v.Ms)
    assert st == 0
    for q, M in enumerate(v.Ms):
        rc, res0, T0, C0 = ppo.best_plan(L, D, S, v.N, M, *tables, v.orderings)
        assert rc == 0 and res[q] == res0
        np.testing.assert_array_equal(T[q], T0)
        np.testing.assert_array_equal(C, C0)
    # its place among the candidates, by the helper bench.py uses
    ranks = problem.rank_among(T[:, 1:], T[:, 0])
    for q, (t, faster, tmin) in enumerate(ranks):
        assert t == T[q, 0] and faster == int((T[q, 1:] < T[q, 0]).sum()) and tmin == T[q, 1:].min()
