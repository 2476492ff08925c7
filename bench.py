#!/usr/bin/env python3
"""Benchmark of the batched pipeline-plan evaluator on one MI355X.

One step = one pass of the whole hot path over the GPT-shaped workload (L=128, D=S=8,
all 40320 device orderings): pp_prefix_costs, then pp_best_plan_multi (partition DP once
-- the partition does not depend on M --, then max-plus makespan and candidate arg-min
for every microbatch count of the workload, M = 8, 16, 32, 64).  A "plan evaluated" is
one (candidate, M) pair: its plan from the DP and backtrack, its schedule, its place in
the arg-min.  Inputs are resident in HBM before the timed
region.  Prints ONE JSON line on stdout; details go to stderr.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# published MI355X figures: 256 compute units x 4 SIMDs x 16 lanes at 2.4 GHz, one 32-bit
# integer operation per lane per clock
ALU_PEAK_OPS = 256 * 4 * 16 * 2.4e9
OPS_PER_PAIR = 3  # subtract, max, min on 32-bit keys per (cell, split) pair
# HBM bytes per k_dp_tile<16> launch on the GPT workload: scaled FETCH_SIZE + WRITE_SIZE from
# two rocprofv3 --pmc runs (profiles/dp_tile_gpt_hbm_traffic.txt)
DP_TRAFFIC_BYTES = {"gpt": 3.76e6}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="gpt", choices=["tiny", "transformer", "gpt", "hetero", "stress"])
    ap.add_argument("--candidates", type=int, default=0, help="override N for the sampled workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the diagnostics outside the step (stage-count search, replicated planner, "
                         "rank of the min-cut ordering), e.g. for profiling the step's kernels alone")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="instead of the workload, run 10 plain device copies of this many MiB "
                         "(reference for scaling the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
                 "use --gpus 1")

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    if args.calibrate_copy:
        n = args.calibrate_copy * (1 << 20) // 8
        src = torch.arange(n, dtype=torch.int64, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_MiB": args.calibrate_copy, "copies": 10,
                          "bytes_read_per_copy": n * 8, "bytes_written_per_copy": n * 8}))
        return
    from paper_2204_10562_amd import problem
    from paper_2204_10562_amd.problem import GpuProblem
    from paper_2204_10562_amd import binding as pp
    from paper_2204_10562_amd import workloads

    make = workloads.CONFIGS[args.workload]
    w = make(N=args.candidates) if (args.candidates and args.workload in ("hetero", "stress")) else make()
    g = GpuProblem(w)
    L, D, S, N, Ms = w.L, w.D, w.S, w.N, w.Ms
    dev = g.dev
    ws = g.workspace()
    out = torch.zeros(pp.RESULT_BYTES * len(w.Ms), dtype=torch.uint8, device=dev)
    C = torch.empty(N, dtype=torch.int64, device=dev)
    T = torch.empty(N, dtype=torch.int64, device=dev)
    bounds = torch.empty(N * S, dtype=torch.int32, device=dev)
    pairs = workloads.pair_evals_per_candidate(L, S) * N

    def step():
        pp.pp_prefix_costs(L, D, g.fwd, g.bwd, g.actf, g.actb, g.bw, g.PF, g.PB, g.XF, g.XB, g.status)
        pp.pp_best_plan_multi(L, D, S, N, Ms, g.PF, g.PB, g.XF, g.XB, g.orderings, out, None, None, ws, g.status)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    assert int(g.status.item()) == 0, "a data fault was raised"
    ms_per_step = wall / args.steps * 1e3
    plans_per_s = N * len(Ms) * args.steps / wall
    winner = pp.read_result(out, S, len(Ms) - 1)  # for the last microbatch count

    # per-entry-point durations with HIP events on the stream the kernels run on
    def timed(fn, reps):
        for _ in range(max(3, reps // 10)):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / reps * 1e-3  # seconds per call

    reps = max(10, args.steps)
    t_dp = timed(lambda: pp.pp_partition_dp(L, D, S, N, g.PF, g.PB, g.XF, g.XB, g.orderings, C, bounds, ws, g.status), reps)
    t_prefix = timed(lambda: pp.pp_prefix_costs(L, D, g.fwd, g.bwd, g.actf, g.actb, g.bw, g.PF, g.PB, g.XF, g.XB, g.status), reps)
    t_mk = {M: timed(lambda M=M: pp.pp_schedule_makespan(L, D, S, N, M, g.PF, g.PB, g.XF, g.XB, g.orderings, bounds, T, g.status), reps) for M in Ms}
    t_multi = timed(lambda: pp.pp_best_plan_multi(L, D, S, N, Ms, g.PF, g.PB, g.XF, g.XB, g.orderings, out, None, None, ws, g.status), reps)
    t_best = {M: timed(lambda M=M: pp.pp_best_plan(L, D, S, N, M, g.PF, g.PB, g.XF, g.XB, g.orderings, out, None, None, ws, g.status), reps) for M in Ms}
    t_rep = rep_winner = t_stages = None
    rdo_rank = []
    if not args.no_extras:
        # the stage-count search (Alg. 3's outer loop) over the same candidates: not part of the step
        ws_st = torch.empty(pp.pp_workspace_bytes_stages(L, D, S, N, len(Ms)), dtype=torch.uint8, device=dev)
        C_st = torch.empty(N * S, dtype=torch.int64, device=dev)
        b_st = torch.empty(N * (S * (S + 1) // 2), dtype=torch.int32, device=dev)
        out_st = torch.zeros(pp.RESULT_BYTES * len(Ms), dtype=torch.uint8, device=dev)
        t_dp_st = timed(lambda: pp.pp_partition_dp_stages(L, D, S, N, g.PF, g.PB, g.XF, g.XB, g.orderings, C_st, b_st, ws_st, g.status), reps)
        t_stages = timed(lambda: pp.pp_best_plan_stages(L, D, S, N, Ms, g.PF, g.PB, g.XF, g.XB, g.orderings, out_st, None, None, ws_st, g.status), reps)
        stage_winner = pp.read_result(out_st, None, len(Ms) - 1)
        del ws_st, C_st, b_st
        # the planner with replicated stages (Alg. 3 + Alg. 4) over the same orderings: not in the step
        if pp.pp_workspace_bytes_replicated(L, D, N) and S == D and N <= 100000:
            import numpy as np
            alpha = torch.from_numpy(workloads.parameter_sizes(w)).to(dev)
            ws_rep = torch.empty(pp.pp_workspace_bytes_replicated(L, D, N), dtype=torch.uint8, device=dev)
            out_rep = torch.zeros(pp.REP_RESULT_BYTES, dtype=torch.uint8, device=dev)
            t_rep = timed(lambda: pp.pp_plan_replicated(L, D, N, Ms[-1], g.fwd, g.bwd, g.actf, g.actb, alpha, g.bw,
                                                        g.orderings, out_rep, None, None, None, None, ws_rep, g.status), 5)
            rep_winner = pp.read_rep_result(out_rep, D)
            del ws_rep
        # the recursive device ordering (Alg. 2) as one more candidate: where does it rank?
        rdo = problem.rdo_row(w).tolist()
        T_all = torch.empty(N * len(Ms), dtype=torch.int64, device=dev)
        pp.pp_best_plan_multi(L, D, S, N, Ms, g.PF, g.PB, g.XF, g.XB, g.orderings, out, T_all, None, ws, g.status)
        o_rdo = torch.tensor(rdo, dtype=torch.int32, device=dev)
        out1 = torch.zeros(pp.RESULT_BYTES * len(Ms), dtype=torch.uint8, device=dev)
        T_rdo = torch.empty(len(Ms), dtype=torch.int64, device=dev)
        pp.pp_best_plan_multi(L, D, S, 1, Ms, g.PF, g.PB, g.XF, g.XB, o_rdo, out1, T_rdo, None, ws, g.status)
        rdo_rank = problem.rank_among(T_all.reshape(len(Ms), N), T_rdo)
        del T_all
    assert int(g.status.item()) == 0
    # what the DP really evaluated (rows shared by consecutive candidates are computed once)
    pp.pp_partition_dp(L, D, S, N, g.PF, g.PB, g.XF, g.XB, g.orderings, C, bounds, ws, g.status)
    torch.cuda.synchronize()
    stats = pp.read_workspace_stats(ws)
    pairs_exec = stats["pairs_executed"]

    achieved = OPS_PER_PAIR * pairs_exec / t_dp
    log("workload %s: L=%d D=S=%d N=%d M=%s" % (w.name, L, D, N, list(Ms)))
    log("  pp_prefix_costs        %9.1f us" % (t_prefix * 1e6))
    log("  pp_partition_dp        %9.1f us   nominal %.3e pair-evals/s  %.3e cells/s" % (t_dp * 1e6, pairs / t_dp, N * S * L / t_dp))
    log("     executed %d of %d nominal pair-evals (%d rows): %.3e executed pair-evals/s = %.1f%% of int32 VALU peak at %d ops/pair"
        % (pairs_exec, pairs, stats["rows_executed"], pairs_exec / t_dp, 100 * achieved / ALU_PEAK_OPS, OPS_PER_PAIR))
    for M in Ms:
        log("  pp_schedule_makespan M=%-3d %7.1f us   %.3e block-ops/s" % (M, t_mk[M] * 1e6, N * M * (4 * S - 3) / t_mk[M]))
    for M in Ms:
        log("  pp_best_plan M=%-3d      %9.1f us   %.3e plans/s" % (M, t_best[M] * 1e6, N / t_best[M]))
    log("  pp_best_plan_multi     %9.1f us   %.3e plans/s" % (t_multi * 1e6, N * len(Ms) / t_multi))
    log("  whole step             %9.1f us   %.3e plans/s" % (ms_per_step * 1e3, plans_per_s))
    log("  winner:", winner)
    if t_stages is not None:
        log("  stage-count search (not in the step): pp_partition_dp_stages %.1f us, pp_best_plan_stages %.1f us = %.3e (candidate, stage count, M) plans/s"
            % (t_dp_st * 1e6, t_stages * 1e6, N * S * len(Ms) / t_stages))
        log("     winner over stage counts 1..%d for M=%d:" % (S, Ms[-1]), stage_winner)
    if t_rep is not None:
        log("  planner with replicated stages (not in the step), M=%d: pp_plan_replicated %.1f ms = %.3e orderings/s"
            % (Ms[-1], t_rep * 1e3, N / t_rep))
        log("     winner:", rep_winner)
    for M, (t, better, tmin) in zip(Ms, rdo_rank):
        log("  recursive device ordering %s, M=%d: T=%d, %d of %d candidates are faster (best T=%d, +%.2f%%)"
            % (rdo[:S], M, t, better, N, tmin, 100.0 * (t - tmin) / tmin))

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ppo
        ppo.build()
        import numpy as np
        rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)
        # bounded sample: at most ~2^32 pair-evals per M (a few seconds on a handful of cores)
        n_cpu = min(N, max(1, (1 << 32) // workloads.pair_evals_per_candidate(L, S)))
        o_cpu = None if (w.orderings is None and n_cpu == N) else np.ascontiguousarray(w.explicit_orderings()[:n_cpu])
        t0 = time.perf_counter()
        for M in Ms:
            rc, res0, T0, C0 = ppo.best_plan(L, D, S, n_cpu, M, PF, PB, XF, XB, o_cpu, want_all=False)
        cpu_wall = time.perf_counter() - t0
        if n_cpu == N:
            assert res0 == winner, "GPU and oracle disagree on the best plan: %r vs %r" % (winner, res0)
        cpu = {"value": n_cpu * len(Ms) / cpu_wall, "unit": "plans/s", "cores": ppo.get_num_threads(),
               "kind": "oracle",
               "sample": "first %d of %d candidates of the %s workload, all %d microbatch counts, %.1f s wall"
                         % (n_cpu, N, w.name, len(Ms), cpu_wall)}
        log("  oracle on %d host threads: %.3e plans/s (%s)" % (cpu["cores"], cpu["value"], cpu["sample"]))

    line = {
        "metric": "candidate plans evaluated/sec (partition DP + makespan + argmin), L=%d, D=%d" % (L, D),
        "value": plans_per_s, "unit": "plans/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": "%s: L=%d, D=S=%d, N=%d orderings, M=%s" % (w.name, L, D, N, list(Ms)),
                   "plans_per_step": N * len(Ms)},
        "dp_cells_per_s": N * S * L / t_dp, "dp_nominal_pair_evals_per_s": pairs / t_dp,
        "dp_executed_pair_evals_per_s": pairs_exec / t_dp,
        "roofline": {"bound": "alu", "kernel": "pp_partition_dp", "achieved": achieved / 1e12,
                     "peak": ALU_PEAK_OPS / 1e12, "unit": "TOP/s (32-bit integer lane-ops)",
                     "frac": achieved / ALU_PEAK_OPS, "traffic": DP_TRAFFIC_BYTES.get(w.name),
                     "launch_us": t_dp * 1e6, "pair_evals_executed_per_launch": pairs_exec,
                     "pair_evals_nominal_per_launch": pairs, "ops_per_pair": OPS_PER_PAIR},
        "cpu_baseline": cpu,
    }
    if t_stages is not None:
        # measured outside the timed step: the rows built on top of the hot path
        line["extras"] = {
            "stage_search": {"entry_point": "pp_best_plan_stages", "us_per_call": t_stages * 1e6,
                             "scheduled_plans_per_s": N * S * len(Ms) / t_stages,
                             "dp_with_all_stage_counts_us": t_dp_st * 1e6},
            "replicated_planner": None if t_rep is None else {
                "entry_point": "pp_plan_replicated", "M": Ms[-1], "ms_per_call": t_rep * 1e3,
                "orderings_per_s": N / t_rep},
            "min_cut_ordering": [{"M": M, "T": t, "candidates_faster": better, "best_T": tmin}
                                 for M, (t, better, tmin) in zip(Ms, rdo_rank)],
        }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
