"""GPU parity of prefix routing against the oracle's fp64 argmin."""
import numpy as np
import pytest
import torch

import dipaco_inputs as gen
import paper_2403_10616_amd as dp
from oracle import dipaco_oracle as orc
from gpu_util import DEV, dev, host

pytestmark = pytest.mark.gpu

TIE = 1e-4   # squared-distance gap below which fp32 and fp64 may legitimately order two centroids differently


def _run(z, c):
    N, D = z.shape
    K = c.shape[0]
    idx = torch.full((max(N, 1),), -1, dtype=torch.int32, device=DEV)
    hist = torch.full((K,), -7, dtype=torch.int64, device=DEV)
    margin = torch.zeros(max(N, 1), dtype=torch.float32, device=DEV)
    zd = dev(z) if N else torch.zeros((1, D), dtype=torch.float32, device=DEV)
    dp.dipaco_route_prefix(zd, dev(c), N, D, K, idx, hist, margin)
    return host(idx)[:N], host(hist), host(margin)[:N]


def _check(z, c, scale=1.0):
    idx, hist, margin = _run(z, c)
    o_idx, o_hist, o_margin = orc.route_prefix(z, c)
    clear = o_margin > TIE * scale
    assert np.array_equal(idx[clear], o_idx[clear])
    for n in np.nonzero(~clear)[0]:           # near-ties: the GPU's pick must be one of the oracle's two best
        d = ((z[n].astype(np.float64) - c.astype(np.float64)) ** 2).sum(1)
        assert idx[n] in np.argsort(d, kind="stable")[:2], (n, o_margin[n])
    assert hist.sum() == len(z) and np.array_equal(hist, np.bincount(idx, minlength=len(c)))
    moved = int((idx != o_idx).sum())
    assert np.abs(hist - o_hist).sum() <= 2 * moved
    fin = clear & np.isfinite(o_margin)
    assert np.abs(margin[fin] - o_margin[fin]).max(initial=0.0) <= 2e-4 * scale
    assert np.array_equal(np.isinf(margin), np.isinf(o_margin))
    return moved, int((~clear).sum())


@pytest.mark.parametrize("N,D,K", [(1000, 768, 256), (129, 64, 8), (4096, 32, 300), (777, 100, 1), (5, 4, 3),
                                   (2500, 768, 1000)])
def test_route_matches_oracle(N, D, K):
    print(f"route N={N} D={D} K={K}", flush=True)
    z, c, _ = gen.gaussian_mixture(N, D, K, 0.3, seed=4)
    _check(z, c)


def test_route_exact_ties_pick_lowest_index_and_empty_input():
    rng = np.random.default_rng(0)
    c = rng.integers(-3, 4, size=(16, 8)).astype(np.float32)
    c[11] = c[4]
    z = rng.integers(-3, 4, size=(300, 8)).astype(np.float32)
    z[:16] = c
    idx, hist, margin = _run(z, c)                   # small integers: fp32 scores are exact
    o_idx, o_hist, o_margin = orc.route_prefix(z, c)
    assert np.array_equal(idx, o_idx) and np.array_equal(hist, o_hist)
    assert np.array_equal(margin.astype(np.float64), o_margin)
    assert idx[11] == 4 and hist[11] == 0
    idx, hist, _ = _run(np.zeros((0, 8), np.float32), c)
    assert len(idx) == 0 and np.array_equal(hist, np.zeros(16, np.int64))
