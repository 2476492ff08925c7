"""Pins for the oracle's schedule variants (duplex channels, GPipe order, transfers added to the
stages, channels that serve by readiness): hand-worked
schedules, closed forms and an independent simulation with explicit service lists."""
import numpy as np
import pytest

from conftest import read_golden
from helpers import fifo_sim, list_sim, variant_blocks

NAMES = {0: "pe", 1: "duplex", 2: "gpipe", 3: "additive"}


def random_pipeline(seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    S = int(rng.integers(1, 6))
    M = int(rng.integers(1, 9))
    z = rng.random() < 0.3
    F = rng.integers(0 if z else 1, 20, size=S).tolist()
    B = rng.integers(0 if z else 1, 30, size=S).tolist()
    cf = [0] + rng.integers(0, 25, size=S - 1).tolist()
    cb = [0] + rng.integers(0, 25, size=S - 1).tolist()
    return S, M, F, B, cf, cb


def test_handworked(ppo):
    g = read_golden("variants_handworked.txt")
    F, B, c, M = g["A_F"][0], g["A_B"][0], g["A_c"][0], g["A_M"][0][0]
    assert ppo.variant_makespan(ppo.SCHED_PE, F, B, c, c, M) == g["A_T_pe"][0][0]
    assert ppo.variant_makespan(ppo.SCHED_DUPLEX, F, B, c, c, M) == g["A_T_duplex"][0][0]
    F, B, c, M = g["B_F"][0], g["B_B"][0], g["B_c"][0], g["B_M"][0][0]
    assert ppo.variant_makespan(ppo.SCHED_GPIPE, F, B, c, c, M) == g["B_T_gpipe"][0][0]
    assert ppo.variant_makespan(ppo.SCHED_ADDITIVE, F, B, c, c, M) == g["B_T_additive"][0][0]
    F, B, c, M = g["A_F"][0], g["A_B"][0], g["A_c"][0], g["A_M"][0][0]
    assert ppo.variant_makespan(ppo.SCHED_ADDITIVE, F, B, c, c, M) == g["A_T_additive"][0][0]
    assert ppo.variant_makespan(ppo.SCHED_FIFO, F, B, c, c, M) == g["A_T_fifo"][0][0]
    F, B, c, M = g["D_F"][0], g["D_B"][0], g["D_c"][0], g["D_M"][0][0]
    assert ppo.variant_makespan(ppo.SCHED_PE, F, B, c, c, M) == g["D_T_pe"][0][0]
    assert ppo.variant_makespan(ppo.SCHED_FIFO, F, B, c, c, M) == g["D_T_fifo"][0][0]
    assert ppo.variant_makespan(ppo.SCHED_GPIPE, [3] * 3, [5] * 3, [0] * 3, [0] * 3, 4) == g["C_T_gpipe"][0][0]


@pytest.mark.parametrize("seed", range(30))
def test_pe_variant_is_the_pe_scheduler(ppo, seed):
    S, M, F, B, cf, cb = random_pipeline(seed)
    assert ppo.variant_makespan(ppo.SCHED_PE, F, B, cf, cb, M) == ppo.pe_makespan(F, B, cf, cb, M)


@pytest.mark.parametrize("seed", range(100, 140))
@pytest.mark.parametrize("variant", [0, 1, 2, 3])
def test_against_the_list_simulation(ppo, seed, variant):
    S, M, F, B, cf, cb = random_pipeline(seed)
    T, _ = list_sim(variant_blocks(NAMES[variant], F, B, cf, cb), M)
    assert ppo.variant_makespan(variant, F, B, cf, cb, M) == T


def positive_pipeline(seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    S = int(rng.integers(1, 7))
    M = int(rng.integers(1, 12))
    hi = int(rng.choice([3, 20, 200]))   # narrow ranges give many equal times
    F = rng.integers(1, hi + 1, size=S).tolist()
    B = rng.integers(1, 2 * hi + 1, size=S).tolist()
    cf = [0] + rng.integers(1, hi + 1, size=S - 1).tolist()
    cb = [0] + rng.integers(1, hi + 1, size=S - 1).tolist()
    return S, M, F, B, cf, cb


@pytest.mark.parametrize("seed", range(300, 420))
def test_readiness_order_against_the_clock_simulation(ppo, seed):
    S, M, F, B, cf, cb = positive_pipeline(seed)
    assert ppo.variant_makespan(ppo.SCHED_FIFO, F, B, cf, cb, M) == fifo_sim(F, B, cf, cb, M)


def test_readiness_order_differs_from_list_order_sometimes(ppo):
    # the two readings of the channel rule are not the same schedule (so the test above can
    # tell them apart), and neither is always the faster one
    less = more = 0
    for seed in range(300, 420):
        S, M, F, B, cf, cb = positive_pipeline(seed)
        a = ppo.variant_makespan(ppo.SCHED_FIFO, F, B, cf, cb, M)
        b = ppo.variant_makespan(ppo.SCHED_PE, F, B, cf, cb, M)
        less += a < b
        more += a > b
    assert less > 0
    print("readiness order faster in", less, "slower in", more, "of 120")


def test_readiness_order_equals_list_order_without_shared_channels(ppo):
    # with one stage there is no channel; with one microbatch nothing ever waits
    assert ppo.variant_makespan(ppo.SCHED_FIFO, [5], [9], [0], [0], 6) == 84
    for seed in range(40):
        S, _, F, B, cf, cb = positive_pipeline(seed)
        assert ppo.variant_makespan(ppo.SCHED_FIFO, F, B, cf, cb, 1) == sum(F) + sum(B) + sum(cf) + sum(cb)


@pytest.mark.parametrize("S,M", [(1, 1), (1, 5), (2, 3), (4, 6), (6, 2)])
def test_gpipe_closed_form_without_transfers(ppo, S, M):
    # uniform stages, free links: forward wave (M + S - 1) F, then backward wave (M + S - 1) B
    assert ppo.variant_makespan(ppo.SCHED_GPIPE, [7] * S, [11] * S, [0] * S, [0] * S, M) == (M + S - 1) * 18


@pytest.mark.parametrize("S,M", [(1, 3), (3, 1), (3, 4), (5, 7), (7, 2), (9, 12)])
def test_additive_equals_pe_scheduler_on_odd_lists(ppo, S, M):
    # In the PE list every resource, stage or channel, owns block j and block 2R-j.  The additive
    # list of S = 2S'-1 stages with free links is therefore exactly the PE list of S' stages in
    # which the odd additive stages play the channels (2S-1 = 4S'-3 blocks either way).
    Sp = (S + 1) // 2
    rng = np.random.Generator(np.random.PCG64(900 + S * 31 + M))
    F = rng.integers(1, 20, size=S).tolist()
    B = rng.integers(1, 30, size=S).tolist()
    zero = [0] * S
    T = ppo.variant_makespan(ppo.SCHED_ADDITIVE, F, B, zero, zero, M)
    # PE pipeline: stage n' = additive stage 2n', channel n' (n' >= 1) = additive stage 2n'-1
    Fp, Bp = F[0::2], B[0::2]
    cfp, cbp = [0] + F[1::2], [0] + B[1::2]
    assert len(Fp) == Sp and len(cfp) == Sp
    assert T == ppo.pe_makespan(Fp, Bp, cfp, cbp, M)


def test_additive_with_free_links_and_one_microbatch_is_the_path(ppo):
    assert ppo.variant_makespan(ppo.SCHED_ADDITIVE, [3, 4, 5], [6, 7, 8], [0, 10, 20], [0, 30, 40], 1) == 133


def test_bounds(ppo):
    # every variant needs at least M times the busiest resource and one microbatch's full path
    for seed in range(200, 230):
        S, M, F, B, cf, cb = random_pipeline(seed)
        path = sum(F) + sum(B) + sum(cf) + sum(cb)
        for variant in (0, 1, 2, 3, 4):
            T = ppo.variant_makespan(variant, F, B, cf, cb, M)
            busiest = max([f + b for f, b in zip(F, B)] +
                          ([max(x, y) if variant == 1 else x + y for x, y in zip(cf[1:], cb[1:])] or [0]))
            if variant == 3:
                busiest = max(f + b + x + y for f, b, x, y in zip(F, B, cf, cb))
            assert T >= max(path, M * busiest)


def test_one_stage_all_variants_agree(ppo):
    for M in (1, 4):
        assert {ppo.variant_makespan(v, [5], [9], [0], [0], M) for v in (0, 1, 2, 3, 4)} == {14 * M}


def test_batch_function(ppo):
    from paper_2204_10562_amd import workloads
    w = workloads.tiny()
    rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)
    rc, C, bounds = ppo.partition_dp(w.L, 4, 4, 24, PF, PB, XF, XB, None)
    rc, T0 = ppo.schedule_makespan(w.L, 4, 4, 24, 8, PF, PB, XF, XB, None, bounds)
    rc, T = ppo.schedule_makespan_variant(ppo.SCHED_PE, w.L, 4, 4, 24, 8, PF, PB, XF, XB, None, bounds)
    assert rc == 0
    np.testing.assert_array_equal(T, T0)
    orders = workloads.all_orderings(4)
    for variant in (1, 2):
        rc, T = ppo.schedule_makespan_variant(variant, w.L, 4, 4, 24, 8, PF, PB, XF, XB, None, bounds)
        assert rc == 0
        for c in (0, 7, 23):
            e = [0] + bounds[c].tolist()
            o = orders[c]
            F = [int(PF[e[i + 1]] - PF[e[i]]) for i in range(4)]
            B = [int(PB[e[i + 1]] - PB[e[i]]) for i in range(4)]
            cf = [0] + [int(XF[(o[n - 1] * 4 + o[n]) * w.L + e[n] - 1]) for n in range(1, 4)]
            cb = [0] + [int(XB[(o[n - 1] * 4 + o[n]) * w.L + e[n] - 1]) for n in range(1, 4)]
            assert T[c] == list_sim(variant_blocks(NAMES[variant], F, B, cf, cb), 8)[0]
    assert ppo.schedule_makespan_variant(7, w.L, 4, 4, 24, 8, PF, PB, XF, XB, None, bounds)[0] == ppo.ERR_INVALID_ARG
