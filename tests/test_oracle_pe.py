"""Pins for the oracle's PE scheduler: the paper's cycle example, hand-worked schedules,
an independent event-driven simulation, Lemma 1's bounds and closed forms."""
import numpy as np
import pytest

from conftest import read_golden
from helpers import event_sim
from paper_2204_10562_amd import workloads


def test_paper_cycle_example(ppo):
    g = read_golden("cycle_example_M6_S2.txt")
    S, M = g["S"][0][0], g["M"][0][0]
    sweeps = ppo.execution_order(S, M)
    assert sweeps.shape == (g["cycles"][0][0], 4 * S - 3)
    for t, row in enumerate(g["cycle"]):
        assert sweeps[t].tolist() == row


@pytest.mark.parametrize("S,M", [(1, 1), (1, 5), (2, 1), (2, 6), (3, 2), (3, 20), (4, 8), (8, 64), (5, 3)])
def test_sweep_structure(ppo, S, M):
    sweeps = ppo.execution_order(S, M)
    J = 4 * S - 3
    # M + 4|S| - 4 cycles in total (proof of Lemma 1)
    assert sweeps.shape[0] == M + 4 * S - 4
    for t in range(sweeps.shape[0]):
        for j in range(1, J + 1):
            m = t + 1 - j + 1
            assert sweeps[t, j - 1] == (m if 1 <= m <= M else 0)


@pytest.mark.parametrize("name", ["handworked_S2_M2.txt", "handworked_S2_M6.txt"])
def test_handworked_schedules(ppo, name):
    g = read_golden(name)
    F, B, cf, cb, M = g["F"][0], g["B"][0], g["cf"][0], g["cb"][0], g["M"][0][0]
    T, st, fi = ppo.pe_makespan(F, B, cf, cb, M, want_times=True)
    assert T == g["T"][0][0]
    assert st.tolist() == g["start"]
    assert ppo.pe_makespan(F, B, cf, cb, 1) == g["T_single_microbatch"][0][0]


def _rand_pipeline(rng, S, zero=False):
    lo = 0 if zero else 1
    F = rng.integers(lo, 20, size=S)
    B = rng.integers(lo, 30, size=S)
    cf = rng.integers(lo, 25, size=S); cf[0] = 0
    cb = rng.integers(lo, 25, size=S); cb[0] = 0
    if zero:
        for a in (F, B, cf, cb):
            a[rng.random(S) < 0.3] = 0
    return F, B, cf, cb


def test_against_event_simulation(ppo):
    rng = np.random.Generator(np.random.PCG64(77))
    for trial in range(120):
        S = int(rng.integers(1, 6))
        M = int(rng.integers(1, 12))
        F, B, cf, cb = _rand_pipeline(rng, S, zero=(trial % 3 == 0))
        T, st, fi = ppo.pe_makespan(F, B, cf, cb, M, want_times=True)
        T2, start = event_sim(F.tolist(), B.tolist(), cf.tolist(), cb.tolist(), M)
        assert T == T2, (trial, S, M)
        for (j, m), s in start.items():
            assert st[j - 1, m - 1] == s, (trial, j, m)


def test_lemma1_bounds_and_critical_path(ppo):
    rng = np.random.Generator(np.random.PCG64(78))
    for trial in range(200):
        S = int(rng.integers(1, 9))
        M = int(rng.integers(1, 40))
        F, B, cf, cb = _rand_pipeline(rng, S)
        C = max(int((F + B).max()), int((cf + cb).max()))
        path = int(F.sum() + B.sum() + cf.sum() + cb.sum())
        T = ppo.pe_makespan(F, B, cf, cb, M)
        assert T >= M * C
        assert T <= (M + 4 * S - 4) * C
        assert T >= path
        assert ppo.pe_makespan(F, B, cf, cb, 1) == path


def test_single_stage(ppo):
    assert ppo.pe_makespan([7], [11], None, None, 9) == 9 * 18


def test_dominating_last_stage_closed_form(ppo):
    # the merged block never idles once started: T = sum of forwards before it
    # + M * merged + sum of backwards after it
    F = np.array([2, 3, 50]); B = np.array([4, 1, 70]); cf = np.array([0, 1, 2]); cb = np.array([0, 3, 1])
    for M in (1, 2, 7, 33):
        T = ppo.pe_makespan(F, B, cf, cb, M)
        assert T == (2 + 1 + 3 + 2) + M * 120 + (1 + 1 + 3 + 4)


def test_monotone_in_durations_and_M(ppo):
    rng = np.random.Generator(np.random.PCG64(79))
    for trial in range(60):
        S = int(rng.integers(2, 6))
        M = int(rng.integers(1, 15))
        F, B, cf, cb = _rand_pipeline(rng, S)
        T = ppo.pe_makespan(F, B, cf, cb, M)
        assert ppo.pe_makespan(F, B, cf, cb, M + 1) >= T
        which = int(rng.integers(0, 4))
        arrs = [F.copy(), B.copy(), cf.copy(), cb.copy()]
        idx = int(rng.integers(1 if which >= 2 else 0, S))
        arrs[which][idx] += int(rng.integers(1, 9))
        assert ppo.pe_makespan(*arrs, M) >= T


def test_table_driven_makespan_matches_direct_durations(ppo):
    w = workloads.random_small(21, 12, 5, 4, 40)
    rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)
    rc, C, bounds = ppo.partition_dp(w.L, w.D, w.S, w.N, PF, PB, XF, XB, w.orderings)
    assert rc == 0
    for M in (1, 3, 8):
        rc, T = ppo.schedule_makespan(w.L, w.D, w.S, w.N, M, PF, PB, XF, XB, w.orderings, bounds)
        assert rc == 0
        for c in range(w.N):
            o, e = w.orderings[c], [0] + bounds[c].tolist()
            F = [int(PF[e[i + 1]] - PF[e[i]]) for i in range(w.S)]
            B = [int(PB[e[i + 1]] - PB[e[i]]) for i in range(w.S)]
            cf = [0] + [int(XF[(o[n - 1] * w.D + o[n]) * w.L + e[n] - 1]) for n in range(1, w.S)]
            cb = [0] + [int(XB[(o[n - 1] * w.D + o[n]) * w.L + e[n] - 1]) for n in range(1, w.S)]
            assert T[c] == event_sim(F, B, cf, cb, M)[0]
            # DP plans: the schedule's bottleneck is the DP's C
            assert T[c] >= M * C[c] and T[c] <= (M + 4 * w.S - 4) * C[c]


def test_any_valid_plan_is_accepted_and_bad_bounds_fault(ppo):
    w = workloads.tiny()
    rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)
    o = workloads.all_orderings(4)[:3]
    b = np.array([[1, 2, 3, 16], [4, 8, 12, 16], [13, 14, 15, 16]], np.int32)
    rc, T = ppo.schedule_makespan(w.L, 4, 4, 3, 4, PF, PB, XF, XB, o, b)
    assert rc == 0 and (T > 0).all()
    for bad in ([0, 2, 3, 16], [4, 4, 12, 16], [4, 8, 12, 15], [4, 8, 12, 17], [8, 4, 12, 16]):
        bb = b.copy(); bb[1] = bad
        assert ppo.schedule_makespan(w.L, 4, 4, 3, 4, PF, PB, XF, XB, o, bb)[0] == ppo.FAULT_BOUNDS


def test_overflow_guard(ppo):
    L = 2
    PF = np.array([0, 1 << 58, 1 << 59], np.int64)
    PB = np.zeros(3, np.int64)
    X = np.zeros(2 * 2 * L, np.int64)
    o = np.array([[0, 1]], np.int32); b = np.array([[1, 2]], np.int32)
    assert ppo.schedule_makespan(L, 2, 2, 1, 2, PF, PB, X, X, o, b)[0] == 0
    assert ppo.schedule_makespan(L, 2, 2, 1, 100, PF, PB, X, X, o, b)[0] == ppo.FAULT_OVERFLOW
