"""Thin Python binding of libpp (include/pp.h): argument marshalling only.

Every function takes torch tensors that already live on the GPU, checks dtype, device
and contiguity, and passes raw pointers plus the current HIP stream to the C entry
point of the same name.  No step of the method runs in Python and there is no CPU
fallback: if libpp.so is missing the import of the library fails loudly.
"""
import ctypes
import os

import torch

from .build import LIB_PATH

PP_OK = 0
PP_ERR_INVALID_ARG = -1
PP_ERR_WORKSPACE = -2
PP_ERR_HIP = -3
PP_FAULT_BANDWIDTH = 1
PP_FAULT_NEGATIVE = 2
PP_FAULT_ORDERING = 4
PP_FAULT_BOUNDS = 8
PP_FAULT_OVERFLOW = 16
PP_MAX_STAGES = 64

EXPORTS = ("pp_prefix_costs", "pp_workspace_bytes", "pp_partition_dp", "pp_schedule_makespan",
           "pp_schedule_makespan_multi", "pp_schedule_makespan_variant",
           "pp_best_plan", "pp_best_plan_static", "pp_best_plan_multi", "pp_workspace_bytes_stages", "pp_partition_dp_stages",
           "pp_best_plan_stages", "pp_workspace_bytes_replicated", "pp_plan_replicated", "pp_rdo_order",
           "pp_strerror")


class PPResult(ctypes.Structure):
    _fields_ = [
        ("best_index", ctypes.c_int64),
        ("T", ctypes.c_int64),
        ("C", ctypes.c_int64),
        ("S", ctypes.c_int32),
        ("bounds", ctypes.c_int32 * PP_MAX_STAGES),
        ("order", ctypes.c_int32 * PP_MAX_STAGES),
    ]


class PPRepResult(ctypes.Structure):
    _fields_ = [
        ("best_index", ctypes.c_int64),
        ("T", ctypes.c_int64),
        ("W", ctypes.c_int64),
        ("S", ctypes.c_int32),
        ("bounds", ctypes.c_int32 * PP_MAX_STAGES),
        ("reps", ctypes.c_int32 * PP_MAX_STAGES),
        ("order", ctypes.c_int32 * PP_MAX_STAGES),
    ]


RESULT_BYTES = ctypes.sizeof(PPResult)
REP_RESULT_BYTES = ctypes.sizeof(PPRepResult)
_lib = None


class PPError(RuntimeError):
    def __init__(self, code):
        self.code = code
        super().__init__("libpp: %s (%d)" % (lib().pp_strerror(code).decode(), code))


def lib():
    """The loaded C library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libpp.so is not built (%s); run __graft_entry__.build() or "
                               "python -m paper_2204_10562_amd.build" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
        L.pp_prefix_costs.argtypes = [i32, i32] + [vp] * 9 + [vp, vp]
        L.pp_prefix_costs.restype = i32
        L.pp_workspace_bytes.argtypes = [i32, i32, i32, i64]
        L.pp_workspace_bytes.restype = sz
        L.pp_partition_dp.argtypes = [i32, i32, i32, i64] + [vp] * 7 + [vp, sz, vp, vp]
        L.pp_partition_dp.restype = i32
        L.pp_schedule_makespan.argtypes = [i32, i32, i32, i64, i32] + [vp] * 7 + [vp, vp]
        L.pp_schedule_makespan.restype = i32
        L.pp_schedule_makespan_multi.argtypes = [i32, i32, i32, i64, i32] + [vp] * 8 + [vp, vp]
        L.pp_schedule_makespan_multi.restype = i32
        L.pp_schedule_makespan_variant.argtypes = [i32, i32, i32, i32, i64, i32] + [vp] * 7 + [vp, vp]
        L.pp_schedule_makespan_variant.restype = i32
        L.pp_best_plan.argtypes = [i32, i32, i32, i64, i32] + [vp] * 8 + [vp, sz, vp, vp]
        L.pp_best_plan.restype = i32
        L.pp_best_plan_static.argtypes = [i32, i32, i32, i64, i32] + [vp] * 8 + [vp, vp]
        L.pp_best_plan_static.restype = i32
        L.pp_best_plan_multi.argtypes = [i32, i32, i32, i64, i32] + [vp] * 9 + [vp, sz, vp, vp]
        L.pp_best_plan_multi.restype = i32
        L.pp_workspace_bytes_stages.argtypes = [i32, i32, i32, i64, i32]
        L.pp_workspace_bytes_stages.restype = sz
        L.pp_partition_dp_stages.argtypes = L.pp_partition_dp.argtypes
        L.pp_partition_dp_stages.restype = i32
        L.pp_best_plan_stages.argtypes = L.pp_best_plan_multi.argtypes
        L.pp_best_plan_stages.restype = i32
        L.pp_workspace_bytes_replicated.argtypes = [i32, i32, i64]
        L.pp_workspace_bytes_replicated.restype = sz
        L.pp_plan_replicated.argtypes = [i32, i32, i64, i32] + [vp] * 12 + [vp, sz, vp, vp]
        L.pp_plan_replicated.restype = i32
        L.pp_rdo_order.argtypes = [i32, vp, vp]
        L.pp_rdo_order.restype = i32
        L.pp_strerror.argtypes = [i32]
        L.pp_strerror.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _ptr(t, dtype, numel=None, name="tensor", optional=False):
    if t is None:
        if optional:
            return None
        raise ValueError(name + " is required")
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError("%s must be a contiguous %s tensor on the GPU" % (name, dtype))
    if numel is not None and t.numel() < numel:
        raise ValueError("%s has %d elements, needs %d" % (name, t.numel(), numel))
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _check(rc):
    if rc != PP_OK:
        raise PPError(rc)


def pp_workspace_bytes(L, D, S, N):
    return int(lib().pp_workspace_bytes(L, D, S, N))


def pp_prefix_costs(L, D, fwd_us, bwd_us, act_fwd_bytes, act_bwd_bytes, bw_bytes_per_us,
                    PF, PB, XF, XB, status):
    i64 = torch.int64
    _check(lib().pp_prefix_costs(
        L, D, _ptr(fwd_us, i64, L, "fwd_us"), _ptr(bwd_us, i64, L, "bwd_us"),
        _ptr(act_fwd_bytes, i64, L, "act_fwd_bytes"),
        _ptr(act_bwd_bytes, i64, L, "act_bwd_bytes", optional=True),
        _ptr(bw_bytes_per_us, i64, D * D, "bw_bytes_per_us"),
        _ptr(PF, i64, L + 1, "PF"), _ptr(PB, i64, L + 1, "PB"),
        _ptr(XF, i64, D * D * L, "XF"), _ptr(XB, i64, D * D * L, "XB"),
        _ptr(status, torch.int32, 1, "status"), _stream()))


def pp_partition_dp(L, D, S, N, PF, PB, XF, XB, orderings, C_out, bounds_out, workspace, status):
    i64, i32 = torch.int64, torch.int32
    _check(lib().pp_partition_dp(
        L, D, S, N, _ptr(PF, i64, L + 1, "PF"), _ptr(PB, i64, L + 1, "PB"),
        _ptr(XF, i64, D * D * L, "XF"), _ptr(XB, i64, D * D * L, "XB"),
        _ptr(orderings, i32, N * S, "orderings", optional=True),
        _ptr(C_out, i64, N, "C_out"), _ptr(bounds_out, i32, N * S, "bounds_out"),
        _ptr(workspace, torch.uint8, None, "workspace"), workspace.numel(),
        _ptr(status, i32, 1, "status"), _stream()))


def pp_schedule_makespan(L, D, S, N, M, PF, PB, XF, XB, orderings, bounds, T_out, status):
    i64, i32 = torch.int64, torch.int32
    _check(lib().pp_schedule_makespan(
        L, D, S, N, M, _ptr(PF, i64, L + 1, "PF"), _ptr(PB, i64, L + 1, "PB"),
        _ptr(XF, i64, D * D * L, "XF"), _ptr(XB, i64, D * D * L, "XB"),
        _ptr(orderings, i32, N * S, "orderings", optional=True),
        _ptr(bounds, i32, N * S, "bounds"), _ptr(T_out, i64, N, "T_out"),
        _ptr(status, i32, 1, "status"), _stream()))


def pp_schedule_makespan_multi(L, D, S, N, M_list, PF, PB, XF, XB, orderings, bounds, T_out, status):
    """M_list is a host sequence of ints; T_out holds len(M_list) * N values."""
    i64, i32 = torch.int64, torch.int32
    nM = len(M_list)
    Ms = (ctypes.c_int32 * nM)(*[int(m) for m in M_list])
    _check(lib().pp_schedule_makespan_multi(
        L, D, S, N, nM, ctypes.cast(Ms, ctypes.c_void_p), _ptr(PF, i64, L + 1, "PF"),
        _ptr(PB, i64, L + 1, "PB"), _ptr(XF, i64, D * D * L, "XF"), _ptr(XB, i64, D * D * L, "XB"),
        _ptr(orderings, i32, N * S, "orderings", optional=True),
        _ptr(bounds, i32, N * S, "bounds"), _ptr(T_out, i64, N * nM, "T_out"),
        _ptr(status, i32, 1, "status"), _stream()))


PP_SCHED_PE, PP_SCHED_DUPLEX, PP_SCHED_GPIPE, PP_SCHED_ADDITIVE, PP_SCHED_FIFO = 0, 1, 2, 3, 4


def pp_schedule_makespan_variant(variant, L, D, S, N, M, PF, PB, XF, XB, orderings, bounds, T_out, status):
    i64, i32 = torch.int64, torch.int32
    _check(lib().pp_schedule_makespan_variant(
        variant, L, D, S, N, M, _ptr(PF, i64, L + 1, "PF"), _ptr(PB, i64, L + 1, "PB"),
        _ptr(XF, i64, D * D * L, "XF"), _ptr(XB, i64, D * D * L, "XB"),
        _ptr(orderings, i32, N * S, "orderings", optional=True),
        _ptr(bounds, i32, N * S, "bounds"), _ptr(T_out, i64, N, "T_out"),
        _ptr(status, i32, 1, "status"), _stream()))


def pp_best_plan(L, D, S, N, M, PF, PB, XF, XB, orderings, out, T_all, C_all, workspace, status):
    i64, i32 = torch.int64, torch.int32
    _check(lib().pp_best_plan(
        L, D, S, N, M, _ptr(PF, i64, L + 1, "PF"), _ptr(PB, i64, L + 1, "PB"),
        _ptr(XF, i64, D * D * L, "XF"), _ptr(XB, i64, D * D * L, "XB"),
        _ptr(orderings, i32, N * S, "orderings", optional=True),
        _ptr(out, torch.uint8, RESULT_BYTES, "out"),
        _ptr(T_all, i64, N, "T_all", optional=True), _ptr(C_all, i64, N, "C_all", optional=True),
        _ptr(workspace, torch.uint8, None, "workspace"), workspace.numel(),
        _ptr(status, i32, 1, "status"), _stream()))


PP_STATIC_WORKSPACE_BYTES = 32 << 20


def pp_best_plan_static(L, D, S, N, M, PF, PB, XF, XB, orderings, out, T_all, C_all, status):
    """pp_best_plan with the library's own static device array as workspace."""
    i64, i32 = torch.int64, torch.int32
    _check(lib().pp_best_plan_static(
        L, D, S, N, M, _ptr(PF, i64, L + 1, "PF"), _ptr(PB, i64, L + 1, "PB"),
        _ptr(XF, i64, D * D * L, "XF"), _ptr(XB, i64, D * D * L, "XB"),
        _ptr(orderings, i32, N * S, "orderings", optional=True),
        _ptr(out, torch.uint8, RESULT_BYTES, "out"),
        _ptr(T_all, i64, N, "T_all", optional=True), _ptr(C_all, i64, N, "C_all", optional=True),
        _ptr(status, i32, 1, "status"), _stream()))


def pp_best_plan_multi(L, D, S, N, M_list, PF, PB, XF, XB, orderings, out, T_all, C_all, workspace,
                       status):
    """M_list is a host sequence of ints; out holds len(M_list) pp_result records."""
    i64, i32 = torch.int64, torch.int32
    nM = len(M_list)
    Ms = (ctypes.c_int32 * nM)(*[int(m) for m in M_list])
    _check(lib().pp_best_plan_multi(
        L, D, S, N, nM, ctypes.cast(Ms, ctypes.c_void_p), _ptr(PF, i64, L + 1, "PF"),
        _ptr(PB, i64, L + 1, "PB"), _ptr(XF, i64, D * D * L, "XF"), _ptr(XB, i64, D * D * L, "XB"),
        _ptr(orderings, i32, N * S, "orderings", optional=True),
        _ptr(out, torch.uint8, RESULT_BYTES * nM, "out"),
        _ptr(T_all, i64, N * nM, "T_all", optional=True), _ptr(C_all, i64, N, "C_all", optional=True),
        _ptr(workspace, torch.uint8, None, "workspace"), workspace.numel(),
        _ptr(status, i32, 1, "status"), _stream()))


def pp_workspace_bytes_stages(L, D, S, N, nM):
    return int(lib().pp_workspace_bytes_stages(L, D, S, N, nM))


def pp_partition_dp_stages(L, D, S, N, PF, PB, XF, XB, orderings, C_out, bounds_out, workspace,
                           status):
    i64, i32 = torch.int64, torch.int32
    _check(lib().pp_partition_dp_stages(
        L, D, S, N, _ptr(PF, i64, L + 1, "PF"), _ptr(PB, i64, L + 1, "PB"),
        _ptr(XF, i64, D * D * L, "XF"), _ptr(XB, i64, D * D * L, "XB"),
        _ptr(orderings, i32, N * S, "orderings", optional=True),
        _ptr(C_out, i64, N * S, "C_out"),
        _ptr(bounds_out, i32, N * (S * (S + 1) // 2), "bounds_out"),
        _ptr(workspace, torch.uint8, None, "workspace"), workspace.numel(),
        _ptr(status, i32, 1, "status"), _stream()))


def pp_best_plan_stages(L, D, S, N, M_list, PF, PB, XF, XB, orderings, out, T_all, C_all,
                        workspace, status):
    """M_list is a host sequence of ints; out holds len(M_list) pp_result records."""
    i64, i32 = torch.int64, torch.int32
    nM = len(M_list)
    Ms = (ctypes.c_int32 * nM)(*[int(m) for m in M_list])
    _check(lib().pp_best_plan_stages(
        L, D, S, N, nM, ctypes.cast(Ms, ctypes.c_void_p), _ptr(PF, i64, L + 1, "PF"),
        _ptr(PB, i64, L + 1, "PB"), _ptr(XF, i64, D * D * L, "XF"), _ptr(XB, i64, D * D * L, "XB"),
        _ptr(orderings, i32, N * S, "orderings", optional=True),
        _ptr(out, torch.uint8, RESULT_BYTES * nM, "out"),
        _ptr(T_all, i64, N * S * nM, "T_all", optional=True),
        _ptr(C_all, i64, N * S, "C_all", optional=True),
        _ptr(workspace, torch.uint8, None, "workspace"), workspace.numel(),
        _ptr(status, i32, 1, "status"), _stream()))


def pp_workspace_bytes_replicated(L, D, N):
    return int(lib().pp_workspace_bytes_replicated(L, D, N))


def pp_plan_replicated(L, D, N, M, fwd_us, bwd_us, act_fwd_bytes, act_bwd_bytes, alpha_bytes,
                       bw_bytes_per_us, orderings, out, T_all, W_all, bounds_all, reps_all, workspace,
                       status):
    i64, i32 = torch.int64, torch.int32
    tri = D * (D + 1) // 2
    _check(lib().pp_plan_replicated(
        L, D, N, M, _ptr(fwd_us, i64, L, "fwd_us"), _ptr(bwd_us, i64, L, "bwd_us"),
        _ptr(act_fwd_bytes, i64, L, "act_fwd_bytes"),
        _ptr(act_bwd_bytes, i64, L, "act_bwd_bytes", optional=True),
        _ptr(alpha_bytes, i64, L, "alpha_bytes"), _ptr(bw_bytes_per_us, i64, D * D, "bw_bytes_per_us"),
        _ptr(orderings, i32, N * D, "orderings", optional=True),
        _ptr(out, torch.uint8, REP_RESULT_BYTES, "out"),
        _ptr(T_all, i64, N * D, "T_all", optional=True), _ptr(W_all, i64, N * D, "W_all", optional=True),
        _ptr(bounds_all, i32, N * tri, "bounds_all", optional=True),
        _ptr(reps_all, i32, N * tri, "reps_all", optional=True),
        _ptr(workspace, torch.uint8, None, "workspace"), workspace.numel(),
        _ptr(status, i32, 1, "status"), _stream()))


def read_rep_result(out, D):
    """Copy a device pp_rep_result (uint8 tensor) to the host and unpack it."""
    r = PPRepResult.from_buffer_copy(bytes(out.cpu().numpy().tobytes()[:REP_RESULT_BYTES]))
    S = int(r.S)
    return dict(best_index=int(r.best_index), T=int(r.T), W=int(r.W), S=S,
                bounds=[int(r.bounds[i]) for i in range(S)], reps=[int(r.reps[i]) for i in range(S)],
                order=[int(r.order[i]) for i in range(D)])


def pp_rdo_order(D, bw_bytes_per_us):
    """Host function: bw is a host sequence/array of D*D ints; returns the devices by rank."""
    bw = (ctypes.c_int64 * (D * D))(*[int(x) for x in bw_bytes_per_us])
    order = (ctypes.c_int32 * D)()
    _check(lib().pp_rdo_order(D, ctypes.cast(bw, ctypes.c_void_p), ctypes.cast(order, ctypes.c_void_p)))
    return list(order)


PP_WS_WORK = 1024
PP_WS_WORK_STRIDE = 128
PP_WS_SHARE = 768


def read_workspace_stats(workspace):
    """Diagnostic counters the last DP call left in the workspace header (see pp.h)."""
    import numpy as np
    rec = workspace[PP_WS_WORK:PP_WS_WORK + 64 * PP_WS_WORK_STRIDE].cpu().numpy().view(np.uint64)
    rec = rec.reshape(64, PP_WS_WORK_STRIDE // 8)
    sh = workspace[PP_WS_SHARE:PP_WS_SHARE + 32].cpu().numpy().view(np.uint32)
    return dict(pairs_executed=int(rec[:, 0].sum()), rows_executed=int(rec[:, 1].sum()),
                share_active=int(sh[0]), share_classes=int(sh[1]), share_keys=int(sh[2]),
                share_computed=int(sh[3]), share_sorted=int(sh[6]), share_sort_devices=int(sh[7]))


def read_result(out, S=None, index=0):
    """Copy a device pp_result (uint8 tensor, record number `index`) to the host and unpack it
    (S entries of bounds and order; S = None: as many as the record's own stage count)."""
    raw = bytes(out.cpu().numpy().tobytes()[index * RESULT_BYTES:(index + 1) * RESULT_BYTES])
    r = PPResult.from_buffer_copy(raw)
    if S is None:
        S = int(r.S)
    return dict(best_index=int(r.best_index), T=int(r.T), C=int(r.C), S=int(r.S),
                bounds=[int(r.bounds[i]) for i in range(S)],
                order=[int(r.order[i]) for i in range(S)])
