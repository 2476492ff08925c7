"""The entry points only enqueue kernels (no allocation, no memset, no synchronisation), so a
caller can record them into a HIP graph: a captured call is replayed several times, with eager
work and synchronisations between the replays, and every replay is compared with the eager
result and with the oracle."""
import sys

import numpy as np
import pytest

from paper_2204_10562_amd import workloads
from test_gpu_parity import oracle_tables

pytestmark = pytest.mark.gpu


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("entry", ["pp_best_plan_static", "pp_best_plan_multi"])
def test_captured_call_replays(ppo, entry):
    import torch
    from paper_2204_10562_amd import binding as pp
    from paper_2204_10562_amd.problem import GpuProblem
    w = workloads.transformer()
    tables = oracle_tables(ppo, w)
    g = GpuProblem(w)
    assert g.prefix() == 0
    L, D, S, N, M = w.L, w.D, w.S, w.N, 16
    out = torch.zeros(pp.RESULT_BYTES, dtype=torch.uint8, device=g.dev)
    T = torch.empty(N, dtype=torch.int64, device=g.dev)
    C = torch.empty(N, dtype=torch.int64, device=g.dev)
    ws = g.workspace()

    def call():
        if entry == "pp_best_plan_static":
            pp.pp_best_plan_static(L, D, S, N, M, g.PF, g.PB, g.XF, g.XB, g.orderings, out, T, C, g.status)
        else:
            pp.pp_best_plan_multi(L, D, S, N, [M], g.PF, g.PB, g.XF, g.XB, g.orderings, out, T, C, ws, g.status)

    say("graph capture of", entry)
    rc, res0, T0, C0 = ppo.best_plan(L, D, S, N, M, *tables, None)
    assert rc == 0
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        call()  # (the first call on a device looks up the static workspace: not under capture)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            call()
    torch.cuda.synchronize()
    for replay in range(3):
        T.zero_(); C.zero_(); out.zero_()
        x = torch.randn(256, 256, device=g.dev)
        (x @ x).sum().item()  # eager work and a synchronisation of the program's own
        graph.replay()
        torch.cuda.synchronize()
        assert int(g.status.item()) == 0
        assert pp.read_result(out, S) == res0, replay
        np.testing.assert_array_equal(T.cpu().numpy(), T0)
        np.testing.assert_array_equal(C.cpu().numpy(), C0)
