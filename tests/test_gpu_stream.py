"""The entry points are asynchronous on the caller's stream: enqueued on a non-default stream
behind work that is still pending, they return at once, and their outputs are right after
that stream alone has been synchronised."""
import sys
import time

import numpy as np
import pytest

from paper_2204_10562_amd import workloads
from test_gpu_parity import oracle_tables

pytestmark = pytest.mark.gpu


def test_best_plan_on_a_side_stream_behind_pending_work(ppo):
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2204_10562_amd import binding as pp
    from paper_2204_10562_amd.problem import GpuProblem
    w = workloads.gpt()
    g = GpuProblem(w)
    L, D, S, N, M = w.L, w.D, w.S, w.N, w.Ms[2]
    ws = g.workspace()
    out = torch.zeros(pp.RESULT_BYTES, dtype=torch.uint8, device=g.dev)
    T = torch.full((N,), -1, dtype=torch.int64, device=g.dev)
    C = torch.full((N,), -1, dtype=torch.int64, device=g.dev)
    torch.cuda.synchronize()
    side = torch.cuda.Stream(device=g.dev)
    gate = torch.cuda.Event()
    # about 0.2 s of work on the default stream that the side stream has to wait for
    a = torch.randn(8192, 8192, device=g.dev)
    for _ in range(40):
        a = (a @ a).clamp_(-1, 1)
    gate.record()
    side.wait_event(gate)
    done = torch.cuda.Event()
    t0 = time.perf_counter()
    with torch.cuda.stream(side):
        pp.pp_prefix_costs(L, D, g.fwd, g.bwd, g.actf, g.actb, g.bw, g.PF, g.PB, g.XF, g.XB, g.status)
        pp.pp_best_plan(L, D, S, N, M, g.PF, g.PB, g.XF, g.XB, None, out, T, C, ws, g.status)
        done.record()
    enqueue_s = time.perf_counter() - t0
    still_pending = not gate.query()
    print("[case] enqueue took %.3f ms, gate pending afterwards: %s" % (enqueue_s * 1e3, still_pending), flush=True)
    sys.stdout.flush()
    # the calls came back while the work in front of them had not finished: nothing in them waited
    assert still_pending and not done.query()
    side.synchronize()  # only the side stream
    assert done.query()
    res = pp.read_result(out, S)
    assert int(g.status.item()) == 0
    tables = oracle_tables(ppo, w)
    rc, res0, T0, C0 = ppo.best_plan(L, D, S, N, M, *tables, None)
    assert rc == 0 and res == res0
    np.testing.assert_array_equal(T.cpu().numpy(), T0)
    np.testing.assert_array_equal(C.cpu().numpy(), C0)
