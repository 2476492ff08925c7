"""The identity the closed-form DP kernel rests on, checked on the CPU against the oracle.

When every link's channel time is the same at every cut position, the recursion for
W(l, xi, r, i) of Sec. IV-B (one replica per stage) collapses: W[n][l] = max(x_1..x_n, B[n][l])
with B the same recursion without channel costs, and the lowest minimising split of cell
(n, l) is the first k >= n with P[k] >= P[l] - W[n][l].  The model below is that statement in
plain Python (the kernel's arithmetic, not its code); the oracle knows nothing of it."""
import bisect

import numpy as np
import pytest

from paper_2204_10562_amd import workloads

INF = 1 << 62


def channel_free_table(P, S):
    L = len(P) - 1
    B = [[INF] * (L + 1) for _ in range(S)]
    B[0] = list(P)
    for n in range(1, S):
        for l in range(n + 1, L + 1):
            B[n][l] = min(max(B[n - 1][k], P[l] - P[k]) for k in range(n, l))
    return B


def closed_form_plan(P, B, x, S):
    """x[n] = channel time between stages n-1 and n (any cut position)."""
    L = len(P) - 1
    m = [0] * S
    for n in range(1, S):
        m[n] = max(m[n - 1], x[n])
    C = max(m[S - 1], B[S - 1][L])
    bounds = [0] * S
    e = L
    for n in range(S - 1, -1, -1):
        bounds[n] = e
        if n:
            v = max(m[n], B[n][e])
            e = max(n, bisect.bisect_left(P, P[e] - v))
    return C, bounds


@pytest.mark.parametrize("seed", range(60))
def test_closed_form_equals_the_recursion(ppo, seed):
    rng = np.random.Generator(np.random.PCG64(5000 + seed))
    L = int(rng.integers(1, 40))
    D = int(rng.integers(1, 7))
    S = int(rng.integers(1, min(L, D) + 1))
    N = 40
    w = workloads.random_small(5000 + seed, L, D, S, N, zero_frac=0.2 if seed % 2 else 0.0,
                               hi_time=int(rng.integers(1, 12)), hi_act=3000, same_act=True)
    rc, PF, PB, XF, XB = ppo.prefix_costs(w.fwd, w.bwd, w.actf, w.actb, w.bw)
    assert rc == 0
    rc, C0, b0 = ppo.partition_dp(L, D, S, N, PF, PB, XF, XB, w.orderings)
    assert rc == 0
    P = [int(v) for v in PF + PB]
    B = channel_free_table(P, S)
    X = (XF + XB).reshape(D, D, L)
    if L > 1:
        assert (X[:, :, :L - 1] == X[:, :, :1]).all()  # the premise
    for c in range(N):
        o = w.orderings[c]
        x = [0] + [int(X[o[n - 1], o[n], 0]) for n in range(1, S)]
        C, bounds = closed_form_plan(P, B, x, S)
        assert C == C0[c] and bounds == b0[c].tolist(), (seed, c)
