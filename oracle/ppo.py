"""ctypes front end of the CPU oracle (oracle/ppo.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
cpu_baseline leg of the benchmark.  The product package never imports it.
All arrays are numpy host arrays; nothing here touches a GPU.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libppo.so")
_lib = None

MAX_STAGES = 64

FAULT_BANDWIDTH = 1
FAULT_NEGATIVE = 2
FAULT_ORDERING = 4
FAULT_BOUNDS = 8
FAULT_OVERFLOW = 16
ERR_INVALID_ARG = -1


class Result(ctypes.Structure):
    _fields_ = [
        ("best_index", ctypes.c_int64),
        ("T", ctypes.c_int64),
        ("C", ctypes.c_int64),
        ("S", ctypes.c_int32),
        ("bounds", ctypes.c_int32 * MAX_STAGES),
        ("order", ctypes.c_int32 * MAX_STAGES),
    ]


def build(force=False):
    """Compile oracle/ppo.c into oracle/libppo.so with gcc."""
    src = os.path.join(_HERE, "ppo.c")
    hdr = os.path.join(_HERE, "ppo.h")
    if (not force and os.path.exists(_SO)
            and os.path.getmtime(_SO) >= max(os.path.getmtime(src), os.path.getmtime(hdr))):
        return _SO
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", _SO, src]
    subprocess.run(cmd, check=True, cwd=_HERE)
    return _SO


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        _lib = ctypes.CDLL(_SO)
        _lib.ppo_pe_makespan.restype = ctypes.c_int64
        _lib.ppo_variant_makespan.restype = ctypes.c_int64
        _lib.ppo_get_num_threads.restype = ctypes.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


class RepResult(ctypes.Structure):
    _fields_ = [
        ("best_index", ctypes.c_int64),
        ("T", ctypes.c_int64),
        ("W", ctypes.c_int64),
        ("S", ctypes.c_int32),
        ("bounds", ctypes.c_int32 * MAX_STAGES),
        ("reps", ctypes.c_int32 * MAX_STAGES),
        ("order", ctypes.c_int32 * MAX_STAGES),
    ]


def set_num_threads(n):
    lib().ppo_set_num_threads(ctypes.c_int(int(n)))


def get_num_threads():
    return int(lib().ppo_get_num_threads())


def prefix_costs(fwd, bwd, actf, actb, bw):
    """-> (status, PF, PB, XF, XB); bw is a D x D matrix in bytes/us."""
    fwd, bwd, actf = _i64(fwd), _i64(bwd), _i64(actf)
    actb = None if actb is None else _i64(actb)
    bw = _i64(bw)
    L, D = fwd.shape[0], bw.shape[0]
    PF = np.empty(L + 1, np.int64)
    PB = np.empty(L + 1, np.int64)
    XF = np.empty(D * D * L, np.int64)
    XB = np.empty(D * D * L, np.int64)
    rc = lib().ppo_prefix_costs(L, D, _p(fwd), _p(bwd), _p(actf), _p(actb), _p(bw),
                                _p(PF), _p(PB), _p(XF), _p(XB))
    return rc, PF, PB, XF, XB


def partition_dp(L, D, S, N, PF, PB, XF, XB, orderings):
    """-> (status, C[N], bounds[N,S])"""
    orderings = _i32(orderings)
    C = np.empty(N, np.int64)
    bounds = np.empty((N, S), np.int32)
    rc = lib().ppo_partition_dp(L, D, S, ctypes.c_int64(N), _p(_i64(PF)), _p(_i64(PB)),
                                _p(_i64(XF)), _p(_i64(XB)), _p(orderings), _p(C), _p(bounds))
    return rc, C, bounds


def schedule_makespan(L, D, S, N, M, PF, PB, XF, XB, orderings, bounds):
    """-> (status, T[N])"""
    orderings = _i32(orderings)
    bounds = _i32(bounds)
    T = np.empty(N, np.int64)
    rc = lib().ppo_schedule_makespan(L, D, S, ctypes.c_int64(N), M, _p(_i64(PF)), _p(_i64(PB)),
                                     _p(_i64(XF)), _p(_i64(XB)), _p(orderings), _p(bounds), _p(T))
    return rc, T


def best_plan(L, D, S, N, M, PF, PB, XF, XB, orderings, want_all=True):
    """-> (status, dict(best_index, T, C, bounds, order), T_all, C_all)"""
    orderings = _i32(orderings)
    res = Result()
    T_all = np.empty(N, np.int64) if want_all else None
    C_all = np.empty(N, np.int64) if want_all else None
    rc = lib().ppo_best_plan(L, D, S, ctypes.c_int64(N), M, _p(_i64(PF)), _p(_i64(PB)),
                             _p(_i64(XF)), _p(_i64(XB)), _p(orderings), ctypes.byref(res),
                             _p(T_all), _p(C_all))
    out = dict(best_index=int(res.best_index), T=int(res.T), C=int(res.C), S=int(res.S),
               bounds=[int(res.bounds[i]) for i in range(S)],
               order=[int(res.order[i]) for i in range(S)])
    return rc, out, T_all, C_all


def best_plan_stages(L, D, S, N, M, PF, PB, XF, XB, orderings):
    """-> (status, dict(best_index, T, C, S, bounds, order), T_all[N,S], C_all[N,S],
    bounds_all[N, S(S+1)/2])"""
    orderings = _i32(orderings)
    res = Result()
    tri = S * (S + 1) // 2
    T_all = np.empty((N, S), np.int64)
    C_all = np.empty((N, S), np.int64)
    b_all = np.empty((N, tri), np.int32)
    rc = lib().ppo_best_plan_stages(L, D, S, ctypes.c_int64(N), M, _p(_i64(PF)), _p(_i64(PB)),
                                    _p(_i64(XF)), _p(_i64(XB)), _p(orderings), ctypes.byref(res),
                                    _p(T_all), _p(C_all), _p(b_all))
    xi = int(res.S)
    out = dict(best_index=int(res.best_index), T=int(res.T), C=int(res.C), S=xi,
               bounds=[int(res.bounds[i]) for i in range(xi)],
               order=[int(res.order[i]) for i in range(xi)])
    return rc, out, T_all, C_all, b_all


def spp_replicated(L, D, N, M, fwd, bwd, actf, actb, alpha, bw, orderings):
    """-> (status, dict(best_index, T, W, S, bounds, reps, order), T_all[N,D], W_all[N,D],
    bounds_all[N, D(D+1)/2], reps_all[N, D(D+1)/2])"""
    orderings = _i32(orderings)
    res = RepResult()
    tri = D * (D + 1) // 2
    T_all = np.empty((N, D), np.int64)
    W_all = np.empty((N, D), np.int64)
    b_all = np.empty((N, tri), np.int32)
    r_all = np.empty((N, tri), np.int32)
    actb = None if actb is None else _i64(actb)
    rc = lib().ppo_spp_replicated(L, D, ctypes.c_int64(N), M, _p(_i64(fwd)), _p(_i64(bwd)),
                                  _p(_i64(actf)), _p(actb), _p(_i64(alpha)), _p(_i64(bw)),
                                  _p(orderings), ctypes.byref(res), _p(T_all), _p(W_all),
                                  _p(b_all), _p(r_all))
    xi = int(res.S)
    out = dict(best_index=int(res.best_index), T=int(res.T), W=int(res.W), S=xi,
               bounds=[int(res.bounds[i]) for i in range(xi)],
               reps=[int(res.reps[i]) for i in range(xi)],
               order=[int(res.order[i]) for i in range(D)])
    return rc, out, T_all, W_all, b_all, r_all


def execution_order(S, M):
    """-> array [sweeps, 4S-3]: microbatch handled by each block per sweep (0 = none)."""
    J = 4 * S - 3
    cap = M + 4 * S + 8
    buf = np.zeros((cap, J), np.int32)
    n = lib().ppo_execution_order(S, M, _p(buf), cap)
    if n < 0:
        raise RuntimeError("ppo_execution_order failed: %d" % n)
    if n > cap:
        raise RuntimeError("more sweeps than expected: %d" % n)
    return buf[:n].copy()


def pe_makespan(F, B, cf, cb, M, want_times=False):
    """Makespan of one pipeline from its durations.

    F, B: per stage (length S); cf, cb: per channel, length S with entry 0 unused.
    """
    F, B = _i64(F), _i64(B)
    S = F.shape[0]
    cf = _i64(cf) if cf is not None else np.zeros(S, np.int64)
    cb = _i64(cb) if cb is not None else np.zeros(S, np.int64)
    J = 4 * S - 3
    st = np.full((J, M), -1, np.int64) if want_times else None
    fi = np.full((J, M), -1, np.int64) if want_times else None
    T = int(lib().ppo_pe_makespan(S, M, _p(F), _p(B), _p(cf), _p(cb), _p(st), _p(fi)))
    return (T, st, fi) if want_times else T


SCHED_PE, SCHED_DUPLEX, SCHED_GPIPE, SCHED_ADDITIVE, SCHED_FIFO = 0, 1, 2, 3, 4


def variant_makespan(variant, F, B, cf, cb, M):
    """Makespan of one pipeline under a schedule variant, from its durations."""
    F, B = _i64(F), _i64(B)
    S = F.shape[0]
    cf = _i64(cf) if cf is not None else np.zeros(S, np.int64)
    cb = _i64(cb) if cb is not None else np.zeros(S, np.int64)
    return int(lib().ppo_variant_makespan(int(variant), S, M, _p(F), _p(B), _p(cf), _p(cb)))


def schedule_makespan_variant(variant, L, D, S, N, M, PF, PB, XF, XB, orderings, bounds):
    """-> (status, T[N])"""
    orderings = _i32(orderings)
    bounds = _i32(bounds)
    T = np.empty(N, np.int64)
    rc = lib().ppo_schedule_makespan_variant(int(variant), L, D, S, ctypes.c_int64(N), M, _p(_i64(PF)),
                                             _p(_i64(PB)), _p(_i64(XF)), _p(_i64(XB)), _p(orderings),
                                             _p(bounds), _p(T))
    return rc, T


def rdo_order(bw):
    """Recursive device ordering of a D x D bandwidth matrix -> list of devices by rank."""
    bw = _i64(bw)
    D = bw.shape[0]
    order = np.empty(D, np.int32)
    rc = lib().ppo_rdo_order(D, _p(bw), _p(order))
    if rc != 0:
        raise RuntimeError("ppo_rdo_order failed: %d" % rc)
    return order.tolist()
