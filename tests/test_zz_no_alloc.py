"""pp_best_plan_static (the entry point that allocates nothing: workspace in a device array
of the library) against pp_best_plan, through the C ABI: two calls in a row on the same GPU,
the second with a smaller input, so that whatever the first call left in the shared array is
still there; every output compared element by element, and both against the oracle."""
import sys

import numpy as np
import pytest

from paper_2204_10562_amd import workloads

pytestmark = pytest.mark.gpu


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


def run_both(ppo, w, M):
    import torch
    from paper_2204_10562_amd import binding as pp
    from paper_2204_10562_amd.problem import GpuProblem
    g = GpuProblem(w)
    assert g.prefix() == 0
    L, D, S, N = w.L, w.D, w.S, w.N
    st, res, T, C = g.best(M)
    assert st == 0
    out = torch.zeros(pp.RESULT_BYTES, dtype=torch.uint8, device=g.dev)
    T2 = torch.full((N,), -7, dtype=torch.int64, device=g.dev)
    C2 = torch.full((N,), -7, dtype=torch.int64, device=g.dev)
    before = torch.cuda.memory_allocated()
    pp.pp_best_plan_static(L, D, S, N, M, g.PF, g.PB, g.XF, g.XB, g.orderings, out, T2, C2, g.status)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert g.take_status() == 0
    res2 = pp.read_result(out, S)
    np.testing.assert_array_equal(T2.cpu().numpy(), T)
    np.testing.assert_array_equal(C2.cpu().numpy(), C)
    assert res2 == res
    # winner only (no T_all / C_all)
    out.zero_()
    pp.pp_best_plan_static(L, D, S, N, M, g.PF, g.PB, g.XF, g.XB, g.orderings, out, None, None, g.status)
    assert g.take_status() == 0 and pp.read_result(out, S) == res
    # and the oracle
    rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)
    rc, res0, T0, C0 = ppo.best_plan(L, D, S, N, M, PF, PB, XF, XB, w.orderings)
    assert rc == 0 and res2 == res0
    np.testing.assert_array_equal(T, T0)
    np.testing.assert_array_equal(C, C0)


def test_static_workspace_two_calls_in_a_row(ppo):
    big = workloads.gpt()            # 19.4 MiB of the 32 MiB array, the tiled kernel
    say("pp_best_plan_static gpt", big.N)
    run_both(ppo, big, big.Ms[1])
    small = workloads.hetero(N=500)  # then a smaller problem in the same array, the L > 128 kernel
    say("pp_best_plan_static hetero", small.N)
    run_both(ppo, small, small.Ms[0])
    tiny = workloads.tiny()
    say("pp_best_plan_static tiny", tiny.N)
    run_both(ppo, tiny, tiny.Ms[0])


def test_static_workspace_rejects_large_problems():
    import torch
    from paper_2204_10562_amd import binding as pp
    from paper_2204_10562_amd.problem import GpuProblem
    w = workloads.hetero(N=200000)   # needs more than the array holds
    assert pp.pp_workspace_bytes(w.L, w.D, w.S, w.N) > pp.PP_STATIC_WORKSPACE_BYTES
    g = GpuProblem(w)
    out = torch.zeros(pp.RESULT_BYTES, dtype=torch.uint8, device=g.dev)
    with pytest.raises(pp.PPError) as e:
        pp.pp_best_plan_static(w.L, w.D, w.S, w.N, 4, g.PF, g.PB, g.XF, g.XB, g.orderings, out, None, None, g.status)
    assert e.value.code == pp.PP_ERR_WORKSPACE
