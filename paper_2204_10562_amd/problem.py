"""Uploads a workload, runs libpp through the Python binding, downloads results."""
import numpy as np
import torch

from . import binding as pp


class GpuProblem:
    def __init__(self, w, device="cuda:0"):
        self.w = w
        self.dev = torch.device(device)
        t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)
        self.fwd, self.bwd = t(w.fwd), t(w.bwd)
        self.actf, self.actb = t(w.actf), t(w.actb)
        self.bw = t(w.bw.reshape(-1))
        self.orderings = None if w.orderings is None else t(w.orderings.reshape(-1))
        L, D = w.L, w.D
        self.PF = torch.empty(L + 1, dtype=torch.int64, device=self.dev)
        self.PB = torch.empty(L + 1, dtype=torch.int64, device=self.dev)
        self.XF = torch.empty(D * D * L, dtype=torch.int64, device=self.dev)
        self.XB = torch.empty(D * D * L, dtype=torch.int64, device=self.dev)
        self.status = torch.zeros(1, dtype=torch.int32, device=self.dev)
        self.ws = None

    def workspace(self, N=None, S=None):
        w = self.w
        need = pp.pp_workspace_bytes(w.L, w.D, S or w.S, N or w.N)
        assert need > 0
        if self.ws is None or self.ws.numel() < need:
            self.ws = torch.empty(need, dtype=torch.uint8, device=self.dev)
        assert self.ws.data_ptr() % 256 == 0
        return self.ws

    def take_status(self):
        s = int(self.status.item())
        self.status.zero_()
        return s

    def prefix(self, actb_none=False):
        w = self.w
        pp.pp_prefix_costs(w.L, w.D, self.fwd, self.bwd, self.actf, None if actb_none else self.actb,
                           self.bw, self.PF, self.PB, self.XF, self.XB, self.status)
        return self.take_status()

    def set_tables(self, PF, PB, XF, XB):
        for dst, src in ((self.PF, PF), (self.PB, PB), (self.XF, XF), (self.XB, XB)):
            dst.copy_(torch.from_numpy(np.ascontiguousarray(src)))

    def dp(self, orderings="default", N=None, S=None):
        w = self.w
        N, S = N or w.N, S or w.S
        o = self.orderings if isinstance(orderings, str) else orderings
        C = torch.empty(N, dtype=torch.int64, device=self.dev)
        bounds = torch.empty(N * S, dtype=torch.int32, device=self.dev)
        pp.pp_partition_dp(w.L, w.D, S, N, self.PF, self.PB, self.XF, self.XB, o, C, bounds,
                           self.workspace(N, S), self.status)
        return self.take_status(), C.cpu().numpy(), bounds.cpu().numpy().reshape(N, S)

    def makespan(self, M, bounds, orderings="default", N=None, S=None):
        w = self.w
        N, S = N or w.N, S or w.S
        o = self.orderings if isinstance(orderings, str) else orderings
        b = torch.from_numpy(np.ascontiguousarray(bounds, dtype=np.int32).reshape(-1)).to(self.dev)
        T = torch.empty(N, dtype=torch.int64, device=self.dev)
        pp.pp_schedule_makespan(w.L, w.D, S, N, M, self.PF, self.PB, self.XF, self.XB, o, b, T,
                                self.status)
        return self.take_status(), T.cpu().numpy()

    def makespan_multi(self, Ms, bounds, orderings="default", N=None, S=None):
        w = self.w
        N, S = N or w.N, S or w.S
        o = self.orderings if isinstance(orderings, str) else orderings
        b = torch.from_numpy(np.ascontiguousarray(bounds, dtype=np.int32).reshape(-1)).to(self.dev)
        T = torch.empty(N * len(Ms), dtype=torch.int64, device=self.dev)
        pp.pp_schedule_makespan_multi(w.L, w.D, S, N, list(Ms), self.PF, self.PB, self.XF, self.XB, o, b, T,
                                      self.status)
        return self.take_status(), T.cpu().numpy().reshape(len(Ms), N)

    def best(self, M, orderings="default", N=None, S=None, want_all=True):
        w = self.w
        N, S = N or w.N, S or w.S
        o = self.orderings if isinstance(orderings, str) else orderings
        out = torch.zeros(pp.RESULT_BYTES, dtype=torch.uint8, device=self.dev)
        T = torch.empty(N, dtype=torch.int64, device=self.dev) if want_all else None
        C = torch.empty(N, dtype=torch.int64, device=self.dev) if want_all else None
        pp.pp_best_plan(w.L, w.D, S, N, M, self.PF, self.PB, self.XF, self.XB, o, out, T, C,
                        self.workspace(N, S), self.status)
        res = pp.read_result(out, S)
        return (self.take_status(), res, None if T is None else T.cpu().numpy(),
                None if C is None else C.cpu().numpy())

    def best_multi(self, Ms, orderings="default", N=None, S=None, want_all=True):
        w = self.w
        N, S = N or w.N, S or w.S
        o = self.orderings if isinstance(orderings, str) else orderings
        nM = len(Ms)
        out = torch.zeros(pp.RESULT_BYTES * nM, dtype=torch.uint8, device=self.dev)
        T = torch.empty(N * nM, dtype=torch.int64, device=self.dev) if want_all else None
        C = torch.empty(N, dtype=torch.int64, device=self.dev) if want_all else None
        pp.pp_best_plan_multi(w.L, w.D, S, N, list(Ms), self.PF, self.PB, self.XF, self.XB, o, out, T, C,
                              self.workspace(N, S), self.status)
        res = [pp.read_result(out, S, q) for q in range(nM)]
        return (self.take_status(), res, None if T is None else T.cpu().numpy().reshape(nM, N),
                None if C is None else C.cpu().numpy())

    def dp_stages(self, orderings="default", N=None, S=None):
        w = self.w
        N, S = N or w.N, S or w.S
        tri = S * (S + 1) // 2
        o = self.orderings if isinstance(orderings, str) else orderings
        C = torch.empty(N * S, dtype=torch.int64, device=self.dev)
        bounds = torch.empty(N * tri, dtype=torch.int32, device=self.dev)
        pp.pp_partition_dp_stages(w.L, w.D, S, N, self.PF, self.PB, self.XF, self.XB, o, C, bounds,
                                  self.workspace(N, S), self.status)
        return self.take_status(), C.cpu().numpy().reshape(N, S), bounds.cpu().numpy().reshape(N, tri)

    def best_stages(self, Ms, orderings="default", N=None, S=None, want_all=True):
        w = self.w
        N, S = N or w.N, S or w.S
        o = self.orderings if isinstance(orderings, str) else orderings
        nM = len(Ms)
        need = pp.pp_workspace_bytes_stages(w.L, w.D, S, N, nM)
        assert need > 0
        if self.ws is None or self.ws.numel() < need:
            self.ws = torch.empty(need, dtype=torch.uint8, device=self.dev)
        out = torch.zeros(pp.RESULT_BYTES * nM, dtype=torch.uint8, device=self.dev)
        T = torch.empty(N * S * nM, dtype=torch.int64, device=self.dev) if want_all else None
        C = torch.empty(N * S, dtype=torch.int64, device=self.dev) if want_all else None
        pp.pp_best_plan_stages(w.L, w.D, S, N, list(Ms), self.PF, self.PB, self.XF, self.XB, o, out,
                               T, C, self.ws, self.status)
        res = [pp.read_result(out, None, q) for q in range(nM)]
        return (self.take_status(), res, None if T is None else T.cpu().numpy().reshape(nM, N, S),
                None if C is None else C.cpu().numpy().reshape(N, S))

    def plan_replicated(self, M, alpha, orderings="default", N=None, want_all=True):
        w = self.w
        N = N or w.N
        L, D = w.L, w.D
        tri = D * (D + 1) // 2
        o = self.orderings if isinstance(orderings, str) else orderings
        need = pp.pp_workspace_bytes_replicated(L, D, N)
        assert need > 0
        ws = torch.empty(need, dtype=torch.uint8, device=self.dev)
        al = torch.from_numpy(np.ascontiguousarray(alpha, dtype=np.int64)).to(self.dev)
        out = torch.zeros(pp.REP_RESULT_BYTES, dtype=torch.uint8, device=self.dev)
        T = torch.empty(N * D, dtype=torch.int64, device=self.dev) if want_all else None
        W = torch.empty(N * D, dtype=torch.int64, device=self.dev) if want_all else None
        b = torch.empty(N * tri, dtype=torch.int32, device=self.dev) if want_all else None
        r = torch.empty(N * tri, dtype=torch.int32, device=self.dev) if want_all else None
        pp.pp_plan_replicated(L, D, N, M, self.fwd, self.bwd, self.actf, self.actb, al, self.bw, o, out,
                              T, W, b, r, ws, self.status)
        res = pp.read_rep_result(out, D)
        if not want_all:
            return self.take_status(), res
        return (self.take_status(), res, T.cpu().numpy().reshape(N, D), W.cpu().numpy().reshape(N, D),
                b.cpu().numpy().reshape(N, tri), r.cpu().numpy().reshape(N, tri))

    def makespan_variant(self, variant, M, bounds, orderings="default", N=None, S=None):
        w = self.w
        N, S = N or w.N, S or w.S
        o = self.orderings if isinstance(orderings, str) else orderings
        b = torch.from_numpy(np.ascontiguousarray(bounds, dtype=np.int32).reshape(-1)).to(self.dev)
        T = torch.empty(N, dtype=torch.int64, device=self.dev)
        pp.pp_schedule_makespan_variant(variant, w.L, w.D, S, N, M, self.PF, self.PB, self.XF, self.XB, o, b,
                                        T, self.status)
        return self.take_status(), T.cpu().numpy()


def rdo_row(w):
    """The recursive device ordering (Alg. 2) of the workload's cluster, cut to the S devices
    a candidate row holds: the row Alg. 3 evaluates before anything else."""
    return np.asarray(pp.pp_rdo_order(w.D, w.bw.reshape(-1).tolist())[:w.S], dtype=np.int32)


def with_first_candidate(w, row):
    """A copy of the workload whose candidate list is `row` followed by the workload's own
    candidates (explicit list, N + 1 rows), so that index 0 is the extra candidate and ties
    with a later copy of the same ordering go to it."""
    import copy
    v = copy.copy(w)
    v.orderings = np.ascontiguousarray(np.vstack([np.asarray(row, np.int32)[None, :], w.explicit_orderings()]))
    v.N = w.N + 1
    return v


def rank_among(T_all, T_one):
    """How many candidates of T_all ([nM, N] tensor or array) are strictly faster than the
    candidate with times T_one ([nM]), and the best time, per microbatch count."""
    T_all = torch.as_tensor(T_all)
    T_one = torch.as_tensor(T_one).to(T_all.device)
    faster = (T_all < T_one[:, None]).sum(dim=1)
    return [(int(T_one[q]), int(faster[q]), int(T_all[q].min())) for q in range(T_all.shape[0])]
