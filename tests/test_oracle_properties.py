"""Randomised property tests of the oracle (hypothesis): each property is fixed by the mathematics of the operation,
not by the oracle's own code, and a dropped term, a wrong sign or a swapped index breaks one of them.  CPU only."""
import itertools

import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import dipaco_oracle as orc

SET = dict(max_examples=40, deadline=None, derandomize=True)   # the same examples on every run


@settings(**SET)
@given(st.lists(st.integers(1, 5), min_size=1, max_size=4), st.data())
def test_path_number_is_a_bijection_with_level_one_most_significant(K, data):
    P = int(np.prod(K))
    mods = tuple(data.draw(st.integers(0, k - 1)) for k in K)
    j = orc.path_index(mods, K)
    assert 0 <= j < P and orc.modules_of_path(j, K) == mods
    # raising the last level's choice by one raises the path number by one; the first level's by P / K_1
    if mods[-1] + 1 < K[-1]:
        assert orc.path_index(mods[:-1] + (mods[-1] + 1,), K) == j + 1
    if mods[0] + 1 < K[0]:
        assert orc.path_index((mods[0] + 1,) + mods[1:], K) == j + P // K[0]


@settings(**SET)
@given(st.integers(1, 12), st.integers(1, 5), st.integers(1, 6), st.integers(0, 2 ** 31 - 1))
def test_routing_against_python_loops_on_integer_points(N, D, K, seed):
    """Small integers: every distance is exact in any precision, ties are frequent and must go to the lowest index."""
    rng = np.random.default_rng(seed)
    z = rng.integers(-2, 3, size=(N, D)).astype(np.float64)
    c = rng.integers(-2, 3, size=(K, D)).astype(np.float64)
    idx, hist, margin = orc.route_prefix(z, c)
    idx2, hist2 = orc.route_prefix_top2(z, c)
    for n in range(N):
        d = [sum((z[n][j] - c[k][j]) ** 2 for j in range(D)) for k in range(K)]
        order = sorted(range(K), key=lambda k: (d[k], k))
        assert idx[n] == order[0] and idx2[n, 0] == order[0]
        if K > 1:
            assert margin[n] == d[order[1]] - d[order[0]] and idx2[n, 1] == order[1]
        else:
            assert np.isinf(margin[n]) and idx2[n, 1] == -1
    assert hist.sum() == N and all(hist[k] == int((idx == k).sum()) for k in range(K))
    assert hist2.sum() == N * min(K, 2)
    # the linear router with w_k = 2 c_k, b_k = -|c_k|^2 is the same decision (scores differ by |z|^2 only)
    lin, lhist, _ = orc.route_linear(z, 2 * c, -(c * c).sum(1))
    assert np.array_equal(lin, idx) and np.array_equal(lhist, hist)


@settings(**SET)
@given(st.integers(1, 6), st.integers(1, 20), st.booleans(), st.integers(0, 2 ** 31 - 1))
def test_outer_step_closed_form_of_the_first_two_steps(n_paths, n, weighted, seed):
    rng = np.random.default_rng(seed)
    theta = rng.standard_normal(n)
    copies = [theta + 0.1 * rng.standard_normal(n) for _ in range(n_paths)]
    w = rng.uniform(0.5, 1.5, n_paths) if weighted else None
    alpha = (w / w.sum()) if weighted else np.full(n_paths, 1.0 / n_paths)
    delta = sum(a * (theta - x) for a, x in zip(alpha, copies))
    lr, mu = 0.7, 0.9
    t1, b1 = orc.outer_step(theta, np.zeros(n), copies, w, False, lr, mu)
    assert np.allclose(b1, delta, rtol=0, atol=1e-14)
    assert np.allclose(t1, theta - lr * (1 + mu) * delta, rtol=0, atol=1e-14)       # first step from a zero buffer
    # a second step with the same delta: buffer (1 + mu) delta, step lr (1 + mu + mu^2) delta
    t2, b2 = orc.outer_step(t1, b1, [delta], None, True, lr, mu)
    assert np.allclose(b2, (1 + mu) * delta, atol=1e-14)
    assert np.allclose(t2, t1 - lr * (1 + mu + mu * mu) * delta, atol=1e-14)
    # the average of the copies is where lr = 1, mu = 0 lands
    t, _ = orc.outer_step(theta, np.zeros(n), copies, w, False, 1.0, 0.0)
    assert np.allclose(t, sum(a * x for a, x in zip(alpha, copies)), atol=1e-14)


@settings(**SET)
@given(st.integers(1, 30), st.floats(1e-4, 1e-1), st.floats(0.0, 0.5), st.integers(0, 2 ** 31 - 1))
def test_adamw_first_step_is_a_signed_step_plus_decay(n, lr, wd, seed):
    rng = np.random.default_rng(seed)
    theta, g = rng.standard_normal(n), rng.standard_normal(n)
    mask = rng.integers(0, 2, n).astype(bool)
    eps = 1e-8
    t, m, v = orc.adamw_step(theta, g, np.zeros(n), np.zeros(n), 1, lr, 0.9, 0.95, eps, wd, mask)
    # bias correction makes m_hat = g and v_hat = g^2 at step 1
    want = theta - lr * (g / (np.abs(g) + eps) + wd * mask * theta)
    assert np.allclose(t, want, rtol=1e-12, atol=1e-15)
    assert np.allclose(m, 0.1 * g, rtol=1e-12) and np.allclose(v, 0.05 * g * g, rtol=1e-12)


@settings(**SET)
@given(st.integers(1, 4), st.integers(1, 3), st.integers(1, 12), st.integers(1, 14), st.integers(0, 2 ** 31 - 1))
def test_window_targets_and_chunk_scores_against_python_loops(P, n, length, window, seed):
    rng = np.random.default_rng(seed)
    S = rng.integers(-3, 4, size=(P, n, length)).astype(np.float64)      # exact sums, frequent ties
    T = orc.window_targets(S, window)
    for i, j in itertools.product(range(n), range(length)):
        sums = [sum(S[p, i, jj] for jj in range(j, min(length, j + window))) for p in range(P)]
        assert T[i, j] == min(range(P), key=lambda p: (-sums[p], p))
    chunk = window
    n_chunks = -(-length // chunk)
    paths = rng.integers(0, P, size=(n, n_chunks))
    got = orc.chunk_routed_scores(S, paths, chunk)
    for i in range(n):
        assert got[i] == sum(S[paths[i][jj // chunk], i, jj] for jj in range(length))
    # one path for every chunk: the document's score under that path
    same = orc.chunk_routed_scores(S, np.zeros((n, n_chunks), dtype=int), chunk)
    assert np.array_equal(same, S[0].sum(axis=1))


@settings(**SET)
@given(st.integers(1, 20), st.integers(1, 4), st.integers(1, 5), st.integers(0, 2 ** 31 - 1))
def test_kmeans_update_is_the_mean_of_the_members(N, D, K, seed):
    rng = np.random.default_rng(seed)
    z = rng.integers(-4, 5, size=(N, D)).astype(np.float64)
    idx = rng.integers(0, K, N)
    prev = rng.standard_normal((K, D))
    c, counts = orc.kmeans_update(z, idx, prev)
    for k in range(K):
        members = [z[n] for n in range(N) if idx[n] == k]
        assert counts[k] == len(members)
        if members:
            assert np.allclose(c[k], sum(members) / len(members), atol=1e-13)
        else:
            assert np.array_equal(c[k], prev[k])                    # an empty cluster keeps its centroid
    # the update never raises the k-means objective for the assignment it was given
    assert orc.kmeans_objective(z, idx, c) <= orc.kmeans_objective(z, idx, prev) + 1e-9
