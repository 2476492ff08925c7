"""pp_rdo_order (host function of libpp) against the oracle's ordering, element by element.
Needs no GPU: the function runs on the host.  The binding is loaded without touching CUDA."""
import numpy as np
import pytest

from paper_2204_10562_amd import binding, workloads


def both(ppo, bw):
    bw = np.asarray(bw, dtype=np.int64)
    D = bw.shape[0]
    return binding.pp_rdo_order(D, bw.reshape(-1).tolist()), ppo.rdo_order(bw)


@pytest.mark.parametrize("seed", range(40))
def test_random_graphs(ppo, seed):
    rng = np.random.Generator(np.random.PCG64(1000 + seed))
    D = int(rng.integers(1, 25))
    kind = seed % 4
    if kind == 0:      # asymmetric, wide values
        bw = rng.integers(0, 10**6, size=(D, D))
    elif kind == 1:    # few distinct values: many equal cuts and equal adjacencies
        bw = rng.integers(0, 3, size=(D, D))
        bw = np.minimum(bw, bw.T)
    elif kind == 2:    # islands: strong inside, weak across
        isl = rng.integers(0, 3, size=D)
        bw = np.where(isl[:, None] == isl[None, :], 25000, 1250)
    else:              # sparse: most pairs not connected at all
        bw = rng.integers(1, 100, size=(D, D)) * (rng.random((D, D)) < 0.2)
    np.fill_diagonal(bw, 0)
    got, want = both(ppo, bw)
    assert got == want


@pytest.mark.parametrize("name", ["tiny", "transformer", "gpt", "hetero", "stress"])
def test_config_clusters(ppo, name):
    gen = getattr(workloads, name)
    w = gen(N=4) if name in ("hetero", "stress") else gen()
    got, want = both(ppo, w.bw)
    assert got == want
    assert sorted(got) == list(range(w.D))


def test_rejects_bad_arguments():
    with pytest.raises(binding.PPError):
        binding.pp_rdo_order(2, [0, -1, 5, 0])
    with pytest.raises(binding.PPError):
        binding.pp_rdo_order(2, [0, 1 << 61, 5, 0])
    assert binding.pp_rdo_order(1, [0]) == [0]
