#!/usr/bin/env python3
"""Benchmark of the batched pipeline-plan evaluator on one MI355X.

One step = one pass of the whole hot path over the GPT-shaped workload (L=128, D=S=8,
all 40320 device orderings): pp_prefix_costs, then pp_best_plan_multi (partition DP once
-- the partition does not depend on M --, then max-plus makespan and candidate arg-min
for every microbatch count of the workload, M = 8, 16, 32, 64).  A "plan evaluated" is
one (candidate, M) pair: its plan from the DP and backtrack, its schedule, its place in
the arg-min.  Inputs are resident in HBM before the timed region.  Prints ONE JSON line
on stdout; details go to stderr.

Objects of the line beside the contract's fields:
  roofline          the kernel that dominates the step (the makespan launch over all
                    microbatch counts), timed alone through pp_schedule_makespan_multi
  roofline_dp       the general partition-DP kernel, timed on the same shape with activation
                    sizes that differ per boundary (on the GPT workload itself the transfer
                    times do not depend on the cut position and the DP runs in closed form:
                    see "dp")
  calibration       the integer vector rate measured on this GPU by the calibration kernel
  cpu_baseline      the oracle on the host cores, as it stands
"""
import argparse
import ctypes
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# published MI355X figures: 256 compute units x 4 SIMDs x 16 lanes at 2.4 GHz, one 32-bit
# integer operation per lane per clock
ALU_PEAK_OPS = 256 * 4 * 16 * 2.4e9
OPS_PER_PAIR = 3      # subtract, max, min on 32-bit keys per (cell, split) pair of the DP
OPS_PER_BLOCK_OP = 2  # max, add per (block, microbatch) update of the schedule


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def profile_figures():
    """Figures that only a counter run can give (HBM bytes, issued instructions), read from
    the rocprofv3 summaries under profiles/: lines of the form 'bench.<key> = <number>'."""
    out = {}
    d = os.path.join(ROOT, "profiles")
    if os.path.isdir(d):
        for name in sorted(os.listdir(d)):
            if name.endswith(".txt"):
                for m in re.finditer(r"^bench\.([\w.]+)\s*=\s*([0-9.eE+-]+)\s*$", open(os.path.join(d, name)).read(), re.M):
                    out[m.group(1)] = float(m.group(2))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="gpt", choices=["tiny", "transformer", "gpt", "gpt_varied", "hetero", "stress"])
    ap.add_argument("--candidates", type=int, default=0, help="override N for the sampled workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip everything outside the step and its entry points (general DP kernel on the "
                         "varied workload, calibration, stage-count search, replicated planner, rank of the "
                         "min-cut ordering, channel-order comparison), e.g. for profiling the step's kernels alone")
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
    from paper_2204_10562_amd import build as pp_build
    calib = ctypes.CDLL(pp_build.CALIB_PATH)
    calib.pp_calib_valu.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    calib.pp_calib_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    if args.calibrate_copy:
        n = args.calibrate_copy * (1 << 20) // 8
        src = torch.arange(n, dtype=torch.int64, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(10):
            assert calib.pp_calib_copy(src.data_ptr(), dst.data_ptr(), n * 8, torch.cuda.current_stream().cuda_stream) == 0
        torch.cuda.synchronize()
        assert bool((dst == src).all())
        print(json.dumps({"calibrate_copy_MiB": args.calibrate_copy, "copies": 10, "kernel": "k_calib_copy",
                          "bytes_read_per_copy": n * 8, "bytes_written_per_copy": n * 8}))
        return
    from paper_2204_10562_amd import problem
    from paper_2204_10562_amd.problem import GpuProblem
    from paper_2204_10562_amd import binding as pp
    from paper_2204_10562_amd import workloads

    make = workloads.WORKLOADS[args.workload]
    w = make(N=args.candidates) if (args.candidates and args.workload in ("hetero", "stress")) else make()
    g = GpuProblem(w)
    L, D, S, N, Ms = w.L, w.D, w.S, w.N, w.Ms
    dev = g.dev
    ws = g.workspace()
    out = torch.zeros(pp.RESULT_BYTES * len(w.Ms), dtype=torch.uint8, device=dev)
    C = torch.empty(N, dtype=torch.int64, device=dev)
    T = torch.empty(N, dtype=torch.int64, device=dev)
    T_multi = torch.empty(N * len(Ms), dtype=torch.int64, device=dev)
    bounds = torch.empty(N * S, dtype=torch.int32, device=dev)
    pairs = workloads.pair_evals_per_candidate(L, S) * N
    figures = profile_figures()

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

    # durations with HIP events on the stream the kernels run on: one event between any two
    # calls, so that every launch has a duration of its own (median and minimum besides the mean)
    def timed(fn, reps):
        for _ in range(max(3, reps // 10)):
            fn()
        # mean: the calls back to back between two events.  Taken twice, the smaller kept: once
        # per process, a few thousand launches in, the host stalls for about 30 ms inside the
        # runtime, and whichever loop that falls into would report it as kernel time.
        mean = None
        for _ in range(2):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            e1.synchronize()
            m = e0.elapsed_time(e1) * 1e-3 / reps
            mean = m if mean is None or m < mean else mean
        # median and minimum: once more with an event after every call (the events themselves
        # add about 3 us per call, so these lie above the mean)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        ev[0].record()
        for i in range(reps):
            fn()
            ev[i + 1].record()
        ev[-1].synchronize()
        each = [ev[i].elapsed_time(ev[i + 1]) * 1e-3 for i in range(reps)]
        return {"mean": mean, "median": statistics.median(each), "min": min(each), "launches": reps}

    def us(t):
        return {"mean_us": t["mean"] * 1e6, "median_us_with_event_per_call": t["median"] * 1e6,
                "min_us_with_event_per_call": t["min"] * 1e6, "launches": t["launches"]}

    # (the large sampled workloads run for tens of milliseconds per call: fewer launches there)
    reps = max(100, args.steps) if pairs < 1e10 else max(3, min(args.steps, 10))
    t_step = timed(step, reps)
    t_dp = timed(lambda: pp.pp_partition_dp(L, D, S, N, g.PF, g.PB, g.XF, g.XB, g.orderings, C, bounds, ws, g.status), reps)
    torch.cuda.synchronize()
    stats = pp.read_workspace_stats(ws)  # what the DP really evaluated in its last call
    t_prefix = timed(lambda: pp.pp_prefix_costs(L, D, g.fwd, g.bwd, g.actf, g.actb, g.bw, g.PF, g.PB, g.XF, g.XB, g.status), reps)
    t_mk = {M: timed(lambda M=M: pp.pp_schedule_makespan(L, D, S, N, M, g.PF, g.PB, g.XF, g.XB, g.orderings, bounds, T, g.status), reps) for M in Ms}
    t_mkm = timed(lambda: pp.pp_schedule_makespan_multi(L, D, S, N, Ms, g.PF, g.PB, g.XF, g.XB, g.orderings, bounds, T_multi, g.status), reps)
    t_multi = timed(lambda: pp.pp_best_plan_multi(L, D, S, N, Ms, g.PF, g.PB, g.XF, g.XB, g.orderings, out, None, None, ws, g.status), reps)
    t_best = {M: timed(lambda M=M: pp.pp_best_plan(L, D, S, N, M, g.PF, g.PB, g.XF, g.XB, g.orderings, out, None, None, ws, g.status), reps) for M in Ms}
    assert int(g.status.item()) == 0
    closed_form = stats["rows_executed"] == 0 and S > 1
    block_ops = N * sum(Ms) * (4 * S - 3)
    prefix_bytes = 4 * L * 8 + (2 * (L + 1) + 2 * D * D * L) * 8

    log("workload %s: L=%d D=S=%d N=%d M=%s" % (w.name, L, D, N, list(Ms)))
    log("  pp_prefix_costs        %9.1f us   %.2f GB/s of %d algorithmic bytes (HBM peak 8000 GB/s: launch-bound)"
        % (t_prefix["mean"] * 1e6, prefix_bytes / t_prefix["mean"] / 1e9, prefix_bytes))
    log("  pp_partition_dp        %9.1f us (median %.1f, min %.1f)   nominal %.3e pair-evals/s  %.3e cells/s%s"
        % (t_dp["mean"] * 1e6, t_dp["median"] * 1e6, t_dp["min"] * 1e6, pairs / t_dp["mean"], N * S * L / t_dp["mean"],
           "   [closed form: transfer times do not depend on the cut position]" if closed_form else ""))
    log("     executed %d of %d nominal pair-evals (%d rows)" % (stats["pairs_executed"], pairs, stats["rows_executed"]))
    if L > 128 and stats["share_active"]:
        log("     %d link classes: %d of the %d candidates computed, the others share their results"
            % (stats["share_classes"], stats["share_computed"], N))
    for M in Ms:
        log("  pp_schedule_makespan M=%-3d %7.1f us   %.3e block-ops/s" % (M, t_mk[M]["mean"] * 1e6, N * M * (4 * S - 3) / t_mk[M]["mean"]))
    log("  pp_schedule_makespan_multi %6.1f us (median %.1f, min %.1f)   %.3e block-ops/s = %.1f%% of int32 VALU peak at %d ops/block-op"
        % (t_mkm["mean"] * 1e6, t_mkm["median"] * 1e6, t_mkm["min"] * 1e6, block_ops / t_mkm["mean"],
           100 * OPS_PER_BLOCK_OP * block_ops / t_mkm["mean"] / ALU_PEAK_OPS, OPS_PER_BLOCK_OP))
    for M in Ms:
        log("  pp_best_plan M=%-3d      %9.1f us   %.3e plans/s" % (M, t_best[M]["mean"] * 1e6, N / t_best[M]["mean"]))
    log("  pp_best_plan_multi     %9.1f us   %.3e plans/s" % (t_multi["mean"] * 1e6, N * len(Ms) / t_multi["mean"]))
    log("  whole step             %9.1f us   %.3e plans/s   (events per step: median %.1f us, min %.1f us)"
        % (ms_per_step * 1e3, plans_per_s, t_step["median"] * 1e6, t_step["min"] * 1e6))
    log("  winner:", winner)

    extras = None
    roofline_dp = None
    calibration = None
    if not args.no_extras:
        extras = {}
        stream = torch.cuda.current_stream().cuda_stream
        # --- the integer vector rate this GPU sustains (calibration kernel: the DP's instruction mix)
        cus = calib.pp_calib_compute_units()
        per_iter = calib.pp_calib_valu_insts_per_iter()
        sink = torch.zeros(1, dtype=torch.int32, device=dev)
        calibration = {"kernel": "k_calib_valu: 16 v_max_i32 + 8 v_min3_i32 per round on independent registers",
                       "compute_units": cus, "clock_khz_reported": calib.pp_calib_clock_khz(), "unit": "T wave64-lane instructions/s"}
        for wps in (1, 2, 4, 8):
            iters = 5000
            tc = timed(lambda: calib.pp_calib_valu(cus * wps, iters, 7, sink.data_ptr(), stream), 5)
            calibration["waves_per_simd_%d" % wps] = cus * wps * 4 * iters * per_iter * 64 / tc["min"] / 1e12
        log("  calibration (T lane-instructions/s at 1/2/4/8 waves per SIMD): %s   spec %.2f"
            % (", ".join("%.2f" % calibration["waves_per_simd_%d" % k] for k in (1, 2, 4, 8)), ALU_PEAK_OPS / 1e12))

        # --- the general DP kernel on the same shape with position-dependent transfer times
        if w.name == "gpt":
            wv = workloads.gpt_varied()
            gv = GpuProblem(wv)
            assert gv.prefix() == 0
            wsv = gv.workspace()
            t_dpv = timed(lambda: pp.pp_partition_dp(L, D, S, N, gv.PF, gv.PB, gv.XF, gv.XB, gv.orderings, C, bounds, wsv, gv.status), reps)
            torch.cuda.synchronize()
            sv = pp.read_workspace_stats(wsv)
            assert int(gv.status.item()) == 0 and sv["rows_executed"] > 0
            ach = OPS_PER_PAIR * sv["pairs_executed"] / t_dpv["mean"]
            peak2 = calibration["waves_per_simd_2"] * 1e12
            roofline_dp = {
                "bound": "alu", "kernel": "pp_partition_dp = k_prep + k_dp_tile<16> (general path)",
                "workload": "gpt_varied: the GPT shape with activation sizes 16 MiB x U[0.5, 2) per boundary",
                "achieved": ach / 1e12, "peak": ALU_PEAK_OPS / 1e12, "unit": "TOP/s (32-bit integer lane-ops)",
                "frac": ach / ALU_PEAK_OPS, "ops_per_pair": OPS_PER_PAIR,
                "peak_measured": peak2 / 1e12, "peak_measured_at": "2 waves per SIMD (the kernel's occupancy)",
                "launch": us(t_dpv), "pair_evals_executed_per_launch": sv["pairs_executed"],
                "pair_evals_nominal_per_launch": pairs, "rows_executed_per_launch": sv["rows_executed"],
                "dp_cells_per_s": N * S * L / t_dpv["mean"], "dp_nominal_pair_evals_per_s": pairs / t_dpv["mean"],
                "traffic": figures.get("dp_general.traffic_bytes_per_launch"),
            }
            # instruction view: what the kernel issued (counter run) against one instruction per
            # lane and clock; cannot exceed 1 whatever one instruction does
            vi = figures.get("dp_general.valu_insts_per_launch")
            if vi:
                roofline_dp["issue_view"] = {
                    "valu_wave_insts_per_launch": vi, "valu_insts_per_executed_pair_lane": vi * 64 / sv["pairs_executed"],
                    "frac_of_spec_issue_rate": vi * 64 / t_dpv["mean"] / ALU_PEAK_OPS,
                    "frac_of_measured_issue_rate": vi * 64 / t_dpv["mean"] / peak2,
                    "valu_busy_frac": figures.get("dp_general.valu_busy_frac"), "source": "profiles/ (rocprofv3 --pmc)"}
            log("  general DP kernel on gpt_varied: pp_partition_dp %.1f us (median %.1f, min %.1f); executed %d pairs (%d rows): "
                "%.1f%% of spec peak at %d ops/pair, %.1f%% of the measured rate"
                % (t_dpv["mean"] * 1e6, t_dpv["median"] * 1e6, t_dpv["min"] * 1e6, sv["pairs_executed"], sv["rows_executed"],
                   100 * ach / ALU_PEAK_OPS, OPS_PER_PAIR, 100 * ach / peak2))
            del gv, wsv

        # --- the stage-count search (Alg. 3's outer loop) over the same candidates
        ws_st = torch.empty(pp.pp_workspace_bytes_stages(L, D, S, N, len(Ms)), dtype=torch.uint8, device=dev)
        C_st = torch.empty(N * S, dtype=torch.int64, device=dev)
        b_st = torch.empty(N * (S * (S + 1) // 2), dtype=torch.int32, device=dev)
        out_st = torch.zeros(pp.RESULT_BYTES * len(Ms), dtype=torch.uint8, device=dev)
        t_dp_st = timed(lambda: pp.pp_partition_dp_stages(L, D, S, N, g.PF, g.PB, g.XF, g.XB, g.orderings, C_st, b_st, ws_st, g.status), reps)
        t_stages = timed(lambda: pp.pp_best_plan_stages(L, D, S, N, Ms, g.PF, g.PB, g.XF, g.XB, g.orderings, out_st, None, None, ws_st, g.status), reps)
        stage_winner = pp.read_result(out_st, None, len(Ms) - 1)
        del ws_st, C_st, b_st
        extras["stage_search"] = {"entry_point": "pp_best_plan_stages", "us_per_call": t_stages["mean"] * 1e6,
                                  "scheduled_plans_per_s": N * S * len(Ms) / t_stages["mean"],
                                  "dp_with_all_stage_counts_us": t_dp_st["mean"] * 1e6}
        log("  stage-count search (not in the step): pp_partition_dp_stages %.1f us, pp_best_plan_stages %.1f us = %.3e (candidate, stage count, M) plans/s"
            % (t_dp_st["mean"] * 1e6, t_stages["mean"] * 1e6, N * S * len(Ms) / t_stages["mean"]))
        log("     winner over stage counts 1..%d for M=%d:" % (S, Ms[-1]), stage_winner)

        # --- the planner with replicated stages (Alg. 3 + Alg. 4) over the same orderings
        extras["replicated_planner"] = None
        if pp.pp_workspace_bytes_replicated(L, D, N) and S == D and N <= 100000:
            alpha = torch.from_numpy(workloads.parameter_sizes(w)).to(dev)
            ws_rep = torch.empty(pp.pp_workspace_bytes_replicated(L, D, N), dtype=torch.uint8, device=dev)
            out_rep = torch.zeros(pp.REP_RESULT_BYTES, dtype=torch.uint8, device=dev)
            t_rep = timed(lambda: pp.pp_plan_replicated(L, D, N, Ms[-1], g.fwd, g.bwd, g.actf, g.actb, alpha, g.bw,
                                                        g.orderings, out_rep, None, None, None, None, ws_rep, g.status), 5)
            rep_winner = pp.read_rep_result(out_rep, D)
            del ws_rep
            extras["replicated_planner"] = {"entry_point": "pp_plan_replicated", "M": Ms[-1], "ms_per_call": t_rep["mean"] * 1e3,
                                            "orderings_per_s": N / t_rep["mean"]}
            log("  planner with replicated stages (not in the step), M=%d: pp_plan_replicated %.1f ms = %.3e orderings/s"
                % (Ms[-1], t_rep["mean"] * 1e3, N / t_rep["mean"]))
            log("     winner:", rep_winner)

        # --- the recursive device ordering (Alg. 2) as one more candidate: where does it rank?
        rdo = problem.rdo_row(w).tolist()
        T_all = torch.empty(N * len(Ms), dtype=torch.int64, device=dev)
        pp.pp_best_plan_multi(L, D, S, N, Ms, g.PF, g.PB, g.XF, g.XB, g.orderings, out, T_all, None, ws, g.status)
        o_rdo = torch.tensor(rdo, dtype=torch.int32, device=dev)
        out1 = torch.zeros(pp.RESULT_BYTES * len(Ms), dtype=torch.uint8, device=dev)
        T_rdo = torch.empty(len(Ms), dtype=torch.int64, device=dev)
        pp.pp_best_plan_multi(L, D, S, 1, Ms, g.PF, g.PB, g.XF, g.XB, o_rdo, out1, T_rdo, None, ws, g.status)
        rdo_rank = problem.rank_among(T_all.reshape(len(Ms), N), T_rdo)
        extras["min_cut_ordering"] = [{"M": M, "T": t, "candidates_faster": better, "best_T": tmin}
                                      for M, (t, better, tmin) in zip(Ms, rdo_rank)]
        for M, (t, better, tmin) in zip(Ms, rdo_rank):
            log("  recursive device ordering %s, M=%d: T=%d, %d of %d candidates are faster (best T=%d, +%.2f%%)"
                % (rdo[:S], M, t, better, N, tmin, 100.0 * (t - tmin) / tmin))

        # --- Alg. 1 read strictly (channels serve by readiness) against the list-order reading
        # the library takes, on the DP's plans: how many T differ, does the winner change?
        # (the event simulation is slow: on the large sampled workloads only the first 2^16
        # candidates, which are a uniform sample, and the default's winner)
        pp.pp_partition_dp(L, D, S, N, g.PF, g.PB, g.XF, g.XB, g.orderings, C, bounds, ws, g.status)
        T_all = T_all.reshape(len(Ms), N)
        n_r = N if g.orderings is None else min(N, 1 << 16)
        T_fifo = torch.empty(n_r, dtype=torch.int64, device=dev)
        readings = []
        for q, M in enumerate(Ms):
            pp.pp_schedule_makespan_variant(pp.PP_SCHED_FIFO, L, D, S, n_r, M, g.PF, g.PB, g.XF, g.XB, g.orderings, bounds, T_fifo, g.status)
            rd = {"M": M, "plans_compared": n_r, "plans_with_different_T": int((T_fifo != T_all[q, :n_r]).sum().item()),
                  "same_winner_among_compared": int(torch.argmin(T_fifo).item()) == int(torch.argmin(T_all[q, :n_r]).item())}
            if n_r < N:
                # the default reading's winner over all N, re-timed under the strict reading
                best = int(torch.argmin(T_all[q]).item())
                t1 = torch.empty(1, dtype=torch.int64, device=dev)
                pp.pp_schedule_makespan_variant(pp.PP_SCHED_FIFO, L, D, S, 1, M, g.PF, g.PB, g.XF, g.XB,
                                                g.orderings[best * S:(best + 1) * S].contiguous(),
                                                bounds[best * S:(best + 1) * S].contiguous(), t1, g.status)
                rd["winner_T_default"], rd["winner_T_by_readiness"] = int(T_all[q, best].item()), int(t1.item())
            readings.append(rd)
        extras["channel_order_readings"] = {"compared": "PP_SCHED_FIFO against the default on the DP plans", "per_M": readings}
        log("  channels by readiness against list order: %s" % readings)
        del T_all
        assert int(g.status.item()) == 0

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
        threads = ppo.get_num_threads()
        cpu = {"value": n_cpu * len(Ms) / cpu_wall, "unit": "plans/s", "cores": threads, "kind": "oracle",
               "sample": "first %d of %d candidates of the %s workload, all %d microbatch counts, %.1f s wall"
                         % (n_cpu, N, w.name, len(Ms), cpu_wall)}
        log("  oracle on %d host threads: %.3e plans/s (%s)" % (cpu["cores"], cpu["value"], cpu["sample"]))
        # one thread, on a sample an eighth of that
        n_one = max(1, n_cpu // 8)
        ppo.set_num_threads(1)
        o_one = np.ascontiguousarray(w.explicit_orderings()[:n_one])
        t0 = time.perf_counter()
        for M in Ms:
            ppo.best_plan(L, D, S, n_one, M, PF, PB, XF, XB, o_one, want_all=False)
        one_wall = time.perf_counter() - t0
        ppo.set_num_threads(threads)
        cpu["single_thread"] = {"value": n_one * len(Ms) / one_wall, "unit": "plans/s", "cores": 1,
                                "sample": "first %d candidates, all %d microbatch counts, %.1f s wall" % (n_one, len(Ms), one_wall)}
        log("  oracle on 1 host thread: %.3e plans/s (%s)" % (cpu["single_thread"]["value"], cpu["single_thread"]["sample"]))

    achieved = OPS_PER_BLOCK_OP * block_ops / t_mkm["mean"]
    line = {
        "metric": "candidate plans evaluated/sec (partition DP + makespan + argmin), L=%d, D=%d" % (L, D),
        "value": plans_per_s, "unit": "plans/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": "%s: L=%d, D=S=%d, N=%d orderings, M=%s" % (w.name, L, D, N, list(Ms)),
                   "plans_per_step": N * len(Ms)},
        "step": us(t_step),
        "dp": {"entry_point": "pp_partition_dp", "closed_form": closed_form, "call": us(t_dp),
               "dp_cells_per_s": N * S * L / t_dp["mean"], "dp_nominal_pair_evals_per_s": pairs / t_dp["mean"],
               "pair_evals_executed_per_launch": stats["pairs_executed"], "pair_evals_nominal_per_launch": pairs,
               "rows_executed_per_launch": stats["rows_executed"],
               # candidates whose links have the same transfer times share one DP (L > 128)
               "shared": ({"link_classes": stats["share_classes"], "candidates_computed": stats["share_computed"]}
                          if L > 128 and stats["share_active"] else None)},
        "dp_cells_per_s": N * S * L / t_dp["mean"],
        "prefix": {"entry_point": "pp_prefix_costs", "call": us(t_prefix), "algorithmic_bytes": prefix_bytes,
                   "GB_per_s": prefix_bytes / t_prefix["mean"] / 1e9, "hbm_peak_GB_per_s": 8000},
        "makespan": {"per_M": [{"M": M, "us": t_mk[M]["mean"] * 1e6, "block_ops_per_s": N * M * (4 * S - 3) / t_mk[M]["mean"]} for M in Ms],
                     "all_M_one_launch_block_ops_per_s": block_ops / t_mkm["mean"]},
        "roofline": {"bound": "alu", "kernel": ("pp_schedule_makespan_multi (the makespan launch of the step: all %d microbatch counts)" % len(Ms)
                                               if not (L > 128 and stats["share_active"]) else
                                               "pp_schedule_makespan_multi over all %d candidates, stand-alone (inside the step only the "
                                               "%d representatives are scheduled)" % (N, stats["share_computed"])),
                     "achieved": achieved / 1e12, "peak": ALU_PEAK_OPS / 1e12, "unit": "TOP/s (32-bit integer lane-ops)",
                     "frac": achieved / ALU_PEAK_OPS, "traffic": figures.get("makespan.traffic_bytes_per_launch"),
                     "launch": us(t_mkm), "launch_us": t_mkm["mean"] * 1e6, "block_ops_per_launch": block_ops,
                     "ops_per_block_op": OPS_PER_BLOCK_OP,
                     "peak_measured": None if calibration is None else calibration["waves_per_simd_2"]},
        "roofline_dp": roofline_dp,
        "calibration": calibration,
        "cpu_baseline": cpu,
    }
    if extras is not None:
        line["extras"] = extras
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
