"""Pins for the oracle's prefix sums and transfer-time tables (CPU only)."""
import numpy as np
import pytest

from conftest import read_golden
from paper_2204_10562_amd import workloads


def test_transfer_values_from_fixture(ppo):
    g = read_golden("transfer_values.txt")
    for nbytes, bw, us in g["case"]:
        bwm = np.array([[0, bw], [bw, 0]], np.int64)
        rc, PF, PB, XF, XB = ppo.prefix_costs([1, 1], [1, 1], [nbytes, 0], None, bwm)
        assert rc == 0
        # link 0 -> 1, boundary 1 is entry 0
        assert XF[(0 * 2 + 1) * 2 + 0] == us
        assert XB[(0 * 2 + 1) * 2 + 0] == us
        assert XF[(0 * 2 + 1) * 2 + 1] == 0  # entry L-1 unused
        assert XF[0] == 0 and XF[(1 * 2 + 1) * 2] == 0  # diagonal rows


def test_prefix_matches_numpy_cumsum(ppo):
    for make in (workloads.tiny, workloads.transformer, workloads.gpt):
        w = make()
        rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)
        assert rc == 0
        assert PF[0] == 0 and PB[0] == 0
        np.testing.assert_array_equal(PF[1:], np.cumsum(w.fwd))
        np.testing.assert_array_equal(PB[1:], np.cumsum(w.bwd))
        assert PF[-1] + PB[-1] == int(w.fwd.sum() + w.bwd.sum())


def test_transfer_is_directional(ppo):
    # forward u->v uses bw[u][v]; backward (v->u) uses bw[v][u]
    bw = np.array([[0, 10, 3], [7, 0, 5], [2, 11, 0]], np.int64)
    actf = np.array([100, 55, 0], np.int64)
    actb = np.array([31, 200, 0], np.int64)
    rc, PF, PB, XF, XB = ppo.prefix_costs([1, 2, 3], [4, 5, 6], actf, actb, bw)
    assert rc == 0
    L, D = 3, 3
    for u in range(D):
        for v in range(D):
            for k in range(L - 1):
                ef = 0 if u == v else -(-int(actf[k]) // int(bw[u, v]))
                eb = 0 if u == v else -(-int(actb[k]) // int(bw[v, u]))
                assert XF[(u * D + v) * L + k] == ef
                assert XB[(u * D + v) * L + k] == eb


def test_backward_sizes_default_to_forward(ppo):
    w = workloads.tiny()
    a = ppo.prefix_costs(w.fwd, w.bwd, w.actf, None, w.bw)
    b = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actf.copy(), w.bw)
    for x, y in zip(a[1:], b[1:]):
        np.testing.assert_array_equal(x, y)


def test_faults(ppo):
    bw = np.array([[0, 10], [10, 0]], np.int64)
    assert ppo.prefix_costs([1, 1], [1, 1], [5, 0], None, bw)[0] == 0
    bad = bw.copy(); bad[0, 1] = 0
    assert ppo.prefix_costs([1, 1], [1, 1], [5, 0], None, bad)[0] & ppo.FAULT_BANDWIDTH
    assert ppo.prefix_costs([1, -1], [1, 1], [5, 0], None, bw)[0] & ppo.FAULT_NEGATIVE
    assert ppo.prefix_costs([1, 1], [1, 1], [-5, 0], None, bw)[0] & ppo.FAULT_NEGATIVE
    # the last activation entry is ignored, even if negative
    assert ppo.prefix_costs([1, 1], [1, 1], [5, -7], None, bw)[0] == 0
    big = 1 << 61
    assert ppo.prefix_costs([big, big], [1, 1], [5, 0], None, bw)[0] & ppo.FAULT_OVERFLOW
    # the diagonal of the bandwidth matrix is ignored
    diag = bw.copy(); diag[0, 0] = -3
    assert ppo.prefix_costs([1, 1], [1, 1], [5, 0], None, diag)[0] == 0
