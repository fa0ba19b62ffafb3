"""Pins for the oracle's AdamW, outer step, path composition and routing (CPU only).

Expected values come from closed forms, hand expansions with python floats, special cases the paper names
(a path-specific module still takes the outer step; all-shared modules reduce to DiLoCo) and brute force.
"""
import itertools
import math

import numpy as np
import pytest

import dipaco_inputs as gen
from oracle import dipaco_oracle as orc


# ------------------------------------------------------------------------------------------- AdamW
def test_adamw_first_step_closed_form():
    rng = np.random.default_rng(0)
    theta = rng.standard_normal(50)
    g = rng.standard_normal(50)
    g[:3] = [0.0, 1e-12, -1e-12]
    mask = (np.arange(50) % 2).astype(float)
    lr, eps, wd = 1e-3, 1e-8, 0.1
    new, m, v = orc.adamw_step(theta, g, np.zeros(50), np.zeros(50), 1, lr, 0.9, 0.95, eps, wd, mask)
    # from zero state the bias corrections cancel the (1-beta) factors exactly: mhat = g, vhat = g^2
    want = theta - lr * (g / (np.abs(g) + eps) + wd * mask * theta)
    assert np.allclose(new, want, rtol=1e-13, atol=1e-18)
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 0.05 * g * g)
    # no decay: the step has size lr*|g|/(|g|+eps) and opposes the gradient
    new2, _, _ = orc.adamw_step(theta, g, np.zeros(50), np.zeros(50), 1, lr, 0.9, 0.95, eps, 0.0, mask)
    assert np.allclose(np.abs(new2 - theta), lr * np.abs(g) / (np.abs(g) + eps), rtol=1e-9, atol=1e-20)
    assert np.all((new2 - theta) * g <= 0)


def test_adamw_two_steps_scalar_by_hand():
    th, m, v = 0.5, 0.0, 0.0
    b1, b2, lr, eps, wd = 0.9, 0.95, 0.01, 1e-8, 0.1
    want = th
    mm = vv = 0.0
    for t, g in enumerate([0.3, -0.7], start=1):
        mm = b1 * mm + (1 - b1) * g
        vv = b2 * vv + (1 - b2) * g * g
        want = want - lr * ((mm / (1 - b1 ** t)) / (math.sqrt(vv / (1 - b2 ** t)) + eps) + wd * want)
    T, M, V = np.array([th]), np.array([m]), np.array([v])
    for t, g in enumerate([0.3, -0.7], start=1):
        T, M, V = orc.adamw_step(T, np.array([g]), M, V, t, lr, b1, b2, eps, wd, np.ones(1))
    assert abs(T[0] - want) < 1e-15
    assert abs(M[0] - mm) < 1e-16 and abs(V[0] - vv) < 1e-16


def test_adamw_mask_switches_decay_off():
    theta = np.array([2.0, 2.0]); g = np.array([1.0, 1.0])
    new, _, _ = orc.adamw_step(theta, g, np.zeros(2), np.zeros(2), 1, 0.1, 0.9, 0.95, 0.0, 0.5, np.array([1.0, 0.0]))
    assert np.allclose(new, [2.0 - 0.1 * (1 + 0.5 * 2.0), 2.0 - 0.1])


def test_decay_mask_covers_matrices_only():
    a = orc.Arch((1, 1), 8, 2, 4, 16, 11, 6)
    lay = orc.param_layout(a)
    mask = orc.decay_mask(a)
    for name, (off, shape, _) in lay.items():
        seg = mask[off:off + int(np.prod(shape))]
        assert np.all(seg == (1.0 if len(shape) == 2 else 0.0)), name


# ------------------------------------------------------------------------------------------- outer step
def _mod(n=40, seed=0):
    rng = np.random.default_rng(seed)
    return rng.standard_normal(n), rng.standard_normal(n) * 0.1


def test_outer_one_path_no_momentum_is_sgd_on_delta():
    theta, _ = _mod()
    local = theta + np.random.default_rng(1).standard_normal(40) * 0.01
    new, buf = orc.outer_step(theta, np.zeros(40), [local], None, False, 0.3, 0.0)
    assert np.allclose(new, theta - 0.3 * (theta - local), rtol=1e-14)
    assert np.allclose(buf, theta - local)
    new1, _ = orc.outer_step(theta, np.zeros(40), [local], None, False, 1.0, 0.0)
    assert np.allclose(new1, local, rtol=1e-14)            # lr 1: the module becomes the path's copy


def test_outer_equal_inputs_equal_single_input_and_delta_form():
    theta, buf = _mod()
    local = theta - 0.02
    a, ba = orc.outer_step(theta, buf, [local] * 5, gen.shard_weights(5, 1), False, 0.7, 0.9)
    b, bb = orc.outer_step(theta, buf, [local], None, False, 0.7, 0.9)
    c, bc = orc.outer_step(theta, buf, [theta - local], None, True, 0.7, 0.9)
    assert np.allclose(a, b, rtol=1e-13) and np.allclose(ba, bb, rtol=1e-13)
    assert np.allclose(b, c, rtol=1e-15) and np.allclose(bb, bc, rtol=1e-15)


def test_outer_weights_scale_and_permutation_invariance_and_uniform_mean():
    theta, buf = _mod(seed=2)
    rng = np.random.default_rng(3)
    locs = [theta + rng.standard_normal(40) * 0.01 for _ in range(6)]
    w = gen.shard_weights(6, 5).astype(np.float64)
    a, ba = orc.outer_step(theta, buf, locs, w, False, 0.7, 0.9)
    b, bb = orc.outer_step(theta, buf, locs, 17.0 * w, False, 0.7, 0.9)
    assert np.allclose(a, b, rtol=1e-13) and np.allclose(ba, bb, rtol=1e-13)
    perm = [3, 0, 5, 1, 4, 2]
    c, bc = orc.outer_step(theta, buf, [locs[i] for i in perm], w[perm], False, 0.7, 0.9)
    assert np.allclose(a, c, rtol=1e-13) and np.allclose(ba, bc, rtol=1e-13)
    # uniform weights: Delta is the plain mean of Algorithm 1
    u, bu = orc.outer_step(theta, np.zeros(40), locs, None, False, 1.0, 0.0)
    assert np.allclose(bu, theta - np.mean(locs, axis=0), rtol=1e-12, atol=1e-15)
    # weighted: Delta = sum w_i (theta - theta_i) / sum w_i, written out
    _, bw = orc.outer_step(theta, np.zeros(40), locs, w, False, 1.0, 0.0)
    want = sum(w[i] * (theta - locs[i]) for i in range(6)) / w.sum()
    assert np.allclose(bw, want, rtol=1e-12, atol=1e-15)


def test_outer_two_steps_match_hand_expanded_momentum():
    th, lr, mu = 1.25, 0.7, 0.9
    d1, d2 = 0.04, -0.03
    b1 = d1
    t1 = th - lr * (d1 + mu * b1)
    b2 = mu * b1 + d2
    t2 = t1 - lr * (d2 + mu * b2)
    T, B = np.array([th]), np.zeros(1)
    T, B = orc.outer_step(T, B, [np.array([d1])], None, True, lr, mu)
    assert abs(T[0] - (th - lr * (1 + mu) * d1)) < 1e-15   # first step from zero buffer
    T, B = orc.outer_step(T, B, [np.array([d2])], None, True, lr, mu)
    assert abs(T[0] - t2) < 1e-15 and abs(B[0] - b2) < 1e-16


# ------------------------------------------------------------------------------------------- paths / compose
def test_path_index_round_trip_and_sharing_counts():
    for K in [(2, 2), (16, 16), (3, 1, 4), (5,)]:
        P = int(np.prod(K))
        seen = set()
        for mods in itertools.product(*[range(k) for k in K]):
            j = orc.path_index(mods, K)
            assert orc.modules_of_path(j, K) == mods
            seen.add(j)
        assert seen == set(range(P))
        for l, kl in enumerate(K):
            for e in range(kl):
                assert len(orc.paths_through_module(l, e, K)) == P // kl
    assert orc.path_index((1, 0), (2, 2)) == 2               # level 1 is the most significant digit
    assert orc.paths_through_module(0, 3, (16, 16)) == list(range(48, 64))


def test_compose_round_trip():
    a = orc.Arch((2, 1), 8, 2, 4, 16, 11, 6)
    bounds = orc.segment_bounds(a)
    assert bounds[0][0] == 0 and bounds[-1][1] == orc.param_count(a)
    assert all(bounds[i][1] == bounds[i + 1][0] for i in range(len(bounds) - 1))
    rng = np.random.default_rng(0)
    segs = [rng.standard_normal(e - s) for s, e in bounds]
    flat = orc.compose_path(segs)
    for (s, e), seg in zip(bounds, segs):
        assert np.array_equal(flat[s:e], seg)
    lay = orc.param_layout(a)
    assert lay["blk0.ln1_g"][0] == bounds[1][0] and lay["blk2.ln1_g"][0] == bounds[2][0]
    assert lay["lnf_g"][0] == bounds[3][0]


# ------------------------------------------------------------------------------------------- routing
def test_route_brute_force_with_constructed_ties():
    rng = np.random.default_rng(0)
    N, K, D = 64, 8, 5
    c = rng.integers(-3, 4, size=(K, D)).astype(np.float64)
    c[5] = c[2]                                            # duplicate centroid: exact ties, lowest index wins
    z = rng.integers(-3, 4, size=(N, D)).astype(np.float64)
    z[:8] = c                                              # points sitting on centroids
    idx, hist, margin = orc.route_prefix(z, c)
    for n in range(N):
        best, best_k, second = None, -1, None
        ds = []
        for k in range(K):
            d = 0.0
            for j in range(D):
                d += (z[n, j] - c[k, j]) ** 2
            ds.append(d)
            if best is None or d < best:
                best, best_k = d, k
        rest = sorted(ds[:best_k] + ds[best_k + 1:])
        assert idx[n] == best_k
        assert margin[n] == rest[0] - best
    assert idx[2] == 2 and idx[5] == 2 and margin[2] == 0.0
    assert hist.sum() == N and np.array_equal(hist, np.bincount(idx, minlength=K))
    assert hist[5] == 0


def test_route_point_on_centroid_and_translation_invariance():
    z, c, _ = gen.gaussian_mixture(200, 16, 12, 0.3, seed=4, dtype=np.float64)
    idx, hist, margin = orc.route_prefix(c, c)
    assert np.array_equal(idx, np.arange(12))
    idx0, hist0, m0 = orc.route_prefix(z, c)
    shift = np.random.default_rng(1).standard_normal(16)
    idx1, hist1, m1 = orc.route_prefix(z + shift, c + shift)
    assert np.array_equal(idx0, idx1) and np.array_equal(hist0, hist1)
    assert np.allclose(m0, m1, rtol=1e-9, atol=1e-12)
    assert np.all(m0 >= 0)


def test_route_matches_expanded_square_form_away_from_ties():
    z, c, _ = gen.gaussian_mixture(500, 32, 20, 0.3, seed=9, dtype=np.float64)
    idx, _, margin = orc.route_prefix(z, c)
    score = (c * c).sum(1)[None, :] - 2.0 * z @ c.T          # same argmin, ||z||^2 dropped
    alt = score.argmin(1)
    far = margin > 1e-9
    assert far.sum() > 400 and np.array_equal(idx[far], alt[far])


# ---- top-2 assignment and the k-means update ------------------------------------------------------------------
def test_top2_brute_force_ties_and_relation_to_argmin():
    rng = np.random.default_rng(5)
    c = rng.integers(-2, 3, size=(6, 3)).astype(np.float64)
    c[4] = c[1]                                   # an exact duplicate: ties everywhere it matters
    z = rng.integers(-2, 3, size=(40, 3)).astype(np.float64)
    idx2, hist = orc.route_prefix_top2(z, c)
    for n in range(len(z)):                       # plain loops, (distance, index) pairs sorted as tuples
        pairs = sorted((sum((z[n][j] - c[k][j]) ** 2 for j in range(3)), k) for k in range(6))
        assert (idx2[n, 0], idx2[n, 1]) == (pairs[0][1], pairs[1][1])
    first, _, _ = orc.route_prefix(z, c)
    assert np.array_equal(idx2[:, 0], first)
    assert np.all(idx2[:, 0] != idx2[:, 1])
    assert hist.sum() == 2 * len(z)
    assert np.array_equal(hist, np.bincount(idx2.ravel(), minlength=6))
    # the duplicate pair: whenever centroid 1 is closest, the second choice is as close (its copy 4, or another
    # centroid at that very distance with a lower index)
    for n in np.nonzero(idx2[:, 0] == 1)[0]:
        d = ((z[n] - c) ** 2).sum(1)
        assert d[idx2[n, 1]] == d[1] and idx2[n, 1] <= 4


def test_top2_single_centroid_and_point_on_centroid():
    idx2, hist = orc.route_prefix_top2(np.ones((3, 2)), np.zeros((1, 2)))
    assert np.array_equal(idx2, [[0, -1]] * 3) and np.array_equal(hist, [3])
    c = np.array([[0.0, 0.0], [10.0, 0.0], [0.0, 1.0]])
    idx2, _ = orc.route_prefix_top2(c, c)         # a point on a centroid: itself first, then its nearest neighbour
    assert np.array_equal(idx2, [[0, 2], [1, 0], [2, 0]])


def test_kmeans_update_by_hand_and_empty_cluster():
    z = np.array([[0.0, 0.0], [2.0, 0.0], [0.0, 4.0], [10.0, 10.0], [1.0, 1.0]])
    idx = np.array([0, 0, 0, 2, 2])
    prev = np.array([[9.0, 9.0], [7.0, -7.0], [5.0, 5.0]])
    c, counts = orc.kmeans_update(z, idx, prev)
    assert np.array_equal(c[0], [2.0 / 3.0, 4.0 / 3.0])
    assert np.array_equal(c[1], [7.0, -7.0])       # no rows: keeps its value
    assert np.array_equal(c[2], [5.5, 5.5])
    assert np.array_equal(counts, [3, 0, 2])
    c1, _ = orc.kmeans_update(z[:1], idx[:1], prev)
    assert np.array_equal(c1[0], z[0])             # one member: the member itself


def test_kmeans_update_invariants():
    rng = np.random.default_rng(6)
    z = rng.standard_normal((200, 5))
    idx = rng.integers(0, 7, size=200)
    prev = rng.standard_normal((7, 5))
    c, counts = orc.kmeans_update(z, idx, prev)
    for k in range(7):                             # residuals of a cluster sum to zero (definition of the mean)
        assert np.abs((z[idx == k] - c[k]).sum(axis=0)).max() < 1e-12
    assert counts.sum() == 200
    perm = rng.permutation(200)                    # order of the points is irrelevant
    c_p, _ = orc.kmeans_update(z[perm], idx[perm], prev)
    assert np.abs(c_p - c).max() < 1e-13
    shift = rng.standard_normal(5)                 # translation equivariance
    c_s, _ = orc.kmeans_update(z + shift, idx, prev + shift)
    assert np.abs(c_s - (c + shift)).max() < 1e-12
    # the mean minimises the within-cluster squared error: any other centre is worse
    assert orc.kmeans_objective(z, idx, c) <= orc.kmeans_objective(z, idx, c + 1e-3 * rng.standard_normal(c.shape))


def test_kmeans_objective_hand_value():
    """Section 2.4.1 (k-means on the prefix features): the within-cluster squared error of three points in the plane,
    worked by hand: (0,0) and (2,0) around (1,0) cost 1 each, (0,4) around (0,3) costs 1, (5,5) around (1,0) costs 41."""
    z = np.array([[0.0, 0.0], [2.0, 0.0], [0.0, 4.0], [5.0, 5.0]])
    c = np.array([[1.0, 0.0], [0.0, 3.0]])
    assert orc.kmeans_objective(z, [0, 0, 1, 0], c) == 44.0
    assert orc.kmeans_objective(z[:3], [0, 0, 1], c) == 3.0
    # it is the sum over points of eq. (1)'s minimum when every point sits with its closest centroid
    idx, _, _ = orc.route_prefix(z, c)
    direct = sum(min((zn[0] - ck[0]) ** 2 + (zn[1] - ck[1]) ** 2 for ck in c) for zn in z)
    assert orc.kmeans_objective(z, idx, c) == direct


def test_lloyd_iterations_never_raise_the_objective():
    z, c0, _ = gen.gaussian_mixture(600, 16, 12, 0.3, seed=7, dtype=np.float64)
    c = c0 + 0.2 * np.random.default_rng(8).standard_normal(c0.shape)
    prev = np.inf
    for _ in range(5):
        idx, _, _ = orc.route_prefix(z, c)
        after_assign = orc.kmeans_objective(z, idx, c)
        assert after_assign <= prev + 1e-9
        c, _ = orc.kmeans_update(z, idx, c)
        prev = orc.kmeans_objective(z, idx, c)
        assert prev <= after_assign + 1e-9


# ---- streaming outer step and norm rescaling ------------------------------------------------------------------------
def test_streaming_outer_equals_batch_form_in_any_arrival_order():
    rng = np.random.default_rng(9)
    theta, buf = rng.standard_normal(50), rng.standard_normal(50)
    locals_ = [theta + 1e-2 * rng.standard_normal(50) for _ in range(5)]
    w = rng.uniform(0.5, 1.5, size=5)
    want = orc.outer_step(theta, buf, locals_, w, False, 0.7, 0.9)
    got = orc.outer_step_streaming(theta, buf, locals_, w, False, 0.7, 0.9)
    assert np.abs(got[0] - want[0]).max() < 1e-14 and np.abs(got[1] - want[1]).max() < 1e-14
    perm = [3, 0, 4, 2, 1]
    got_p = orc.outer_step_streaming(theta, buf, [locals_[i] for i in perm], w[perm], False, 0.7, 0.9)
    assert np.abs(got_p[0] - want[0]).max() < 1e-14
    deltas = [theta - x for x in locals_]
    got_d = orc.outer_step_streaming(theta, buf, deltas, w, True, 0.7, 0.9)
    assert np.abs(got_d[0] - want[0]).max() < 1e-14


def test_norm_rescaling_closed_forms():
    theta, buf0 = np.array([1.0, -2.0, 0.5]), np.zeros(3)
    d = np.array([0.1, 0.2, -0.4])
    P = 16
    th, buf = orc.outer_step_streaming(theta, buf0, [d] * P, None, True, 0.5, 0.0, norm_scale=np.sqrt(P))
    assert np.allclose(th, theta - 0.5 * 4.0 * d, atol=1e-15)      # P equal deltas: mean d, times sqrt(16) = 4
    assert np.allclose(buf, 4.0 * d, atol=1e-15)
    # without momentum the step is linear in the scale; with it, theta - theta_prev = -lr (1 + mu) s d on the first step
    th2, _ = orc.outer_step_streaming(theta, buf0, [d], None, True, 0.7, 0.9, norm_scale=3.0)
    assert np.allclose(th2, theta - 0.7 * 1.9 * 3.0 * d, atol=1e-15)
    th1, b1 = orc.outer_step_streaming(theta, buf0, [d], None, True, 0.7, 0.9, norm_scale=1.0)
    ref = orc.outer_step(theta, buf0, [d], None, True, 0.7, 0.9)
    assert np.array_equal(th1, ref[0]) and np.array_equal(b1, ref[1])


def test_module_table_path_specific_module_and_independence():
    """Section 2.6: a path-specific module (one path, no averaging) still takes the outer optimiser.  First step
    from zero momentum in closed form; shared modules equal the single-module rule; modules do not interact."""
    rng = np.random.default_rng(21)
    th_a, th_b = rng.standard_normal(7), rng.standard_normal(11)
    local_a = th_a + 0.01 * rng.standard_normal(7)
    locals_b = [th_b + 0.01 * rng.standard_normal(11) for _ in range(4)]
    w_b = rng.uniform(0.5, 1.5, size=4)
    mods = [dict(theta=th_a, momentum=np.zeros(7), inputs=[local_a], weights=None, is_delta=False),
            dict(theta=th_b, momentum=rng.standard_normal(11), inputs=locals_b, weights=w_b, is_delta=False)]
    out = orc.outer_step_modules(mods, 0.7, 0.9)
    # one path, zero momentum: theta - lr (1 + mu) (theta - theta_local); momentum = the delta itself
    assert np.allclose(out[0][0], th_a - 0.7 * 1.9 * (th_a - local_a), atol=1e-15)
    assert np.allclose(out[0][1], th_a - local_a, atol=1e-15)
    # hand-expanded weighted mean for the shared module
    alpha = w_b / w_b.sum()
    delta = sum(alpha[i] * (th_b - locals_b[i]) for i in range(4))
    buf = 0.9 * mods[1]["momentum"] + delta
    assert np.allclose(out[1][1], buf, atol=1e-15)
    assert np.allclose(out[1][0], th_b - 0.7 * (delta + 0.9 * buf), atol=1e-15)
    # independence: changing module a leaves module b's result bit-identical
    mods2 = [dict(mods[0], inputs=[local_a + 1.0]), mods[1]]
    out2 = orc.outer_step_modules(mods2, 0.7, 0.9)
    assert np.array_equal(out2[1][0], out[1][0]) and not np.array_equal(out2[0][0], out[0][0])
    # norm rescaling multiplies the averaged delta: with zero momentum coefficient the step is linear in it
    m3 = [dict(mods[1], momentum=np.zeros(11), norm_scale=2.0)]
    m1 = [dict(mods[1], momentum=np.zeros(11))]
    s3, s1 = orc.outer_step_modules(m3, 0.5, 0.0), orc.outer_step_modules(m1, 0.5, 0.0)
    assert np.allclose(th_b - s3[0][0], 2.0 * (th_b - s1[0][0]), atol=1e-15)


# ---- discriminative router: linear logistic classifier --------------------------------------------------------------
def test_logistic_closed_forms_at_zero_weights_and_two_classes():
    rng = np.random.default_rng(31)
    N, D, K = 40, 6, 5
    z = rng.standard_normal((N, D))
    y = rng.integers(0, K, size=N)
    loss, dW, db = orc.logistic_loss_grad(z, y, np.zeros((K, D)), np.zeros(K))
    q = np.bincount(y, minlength=K) / N
    assert abs(loss - math.log(K)) < 1e-14                       # uniform prediction
    assert np.allclose(db, 1.0 / K - q, atol=1e-15)              # mean softmax minus label frequencies
    want = np.full((K, D), 1.0 / K) * z.mean(0)[None, :]
    for k in range(K):
        want[k] -= z[y == k].sum(0) / N
    assert np.allclose(dW, want, atol=1e-14)
    # two classes: softmax over (a, -a) is the logistic sigmoid of 2a -- the textbook binary model
    w, b0 = rng.standard_normal(D), 0.3
    W2, b2 = np.stack([w, -w]), np.array([b0, -b0])
    y2 = rng.integers(0, 2, size=N)
    loss2, dW2, db2 = orc.logistic_loss_grad(z, y2, W2, b2)
    s = 1.0 / (1.0 + np.exp(-2.0 * (z @ w + b0)))                # P(class 0)
    assert abs(loss2 + np.mean(np.where(y2 == 0, np.log(s), np.log1p(-s)))) < 1e-13
    assert np.allclose(db2, [np.mean(s - (y2 == 0)), -np.mean(s - (y2 == 0))], atol=1e-14)
    assert np.allclose(dW2[0], ((s - (y2 == 0))[:, None] * z).mean(0), atol=1e-14)
    assert np.allclose(dW2.sum(0), 0.0, atol=1e-14) and abs(db2.sum()) < 1e-15   # rows of p - e sum to zero


def test_logistic_gradients_match_finite_differences_and_ignore_bad_labels():
    rng = np.random.default_rng(32)
    N, D, K = 25, 4, 3
    z = rng.standard_normal((N, D))
    y = rng.integers(0, K, size=N)
    W, b = 0.5 * rng.standard_normal((K, D)), 0.2 * rng.standard_normal(K)
    loss, dW, db = orc.logistic_loss_grad(z, y, W, b)
    h = 1e-6
    for (k, d) in [(0, 0), (2, 3), (1, 2)]:
        Wp, Wm = W.copy(), W.copy()
        Wp[k, d] += h
        Wm[k, d] -= h
        fd = (orc.logistic_loss_grad(z, y, Wp, b)[0] - orc.logistic_loss_grad(z, y, Wm, b)[0]) / (2 * h)
        assert abs(fd - dW[k, d]) < 1e-8
    for k in range(K):
        bp, bm = b.copy(), b.copy()
        bp[k] += h
        bm[k] -= h
        fd = (orc.logistic_loss_grad(z, y, W, bp)[0] - orc.logistic_loss_grad(z, y, W, bm)[0]) / (2 * h)
        assert abs(fd - db[k]) < 1e-8
    y_bad = y.copy()
    y_bad[:5] = [-1, K, 7, -3, K + 1]
    l2, dW2, db2 = orc.logistic_loss_grad(z, y_bad, W, b)
    l3, dW3, db3 = orc.logistic_loss_grad(z[5:], y[5:], W, b)
    assert abs(l2 * N - l3 * (N - 5)) < 1e-12 and np.allclose(dW2 * N, dW3 * (N - 5), atol=1e-12)


def test_bias_only_descent_matches_the_label_distribution():
    """The appendix's remedy for under-represented paths: a bias trained (weights frozen) until the router's mean
    predicted distribution equals the labels' -- the stationary point of the cross-entropy in the bias."""
    rng = np.random.default_rng(33)
    N, D, K = 400, 5, 4
    z = rng.standard_normal((N, D))
    W = rng.standard_normal((K, D))
    y = rng.choice(K, size=N, p=[0.55, 0.3, 0.1, 0.05])          # an unbalanced target
    q = np.bincount(y, minlength=K) / N
    b = np.zeros(K)
    for _ in range(3000):
        _, _, db = orc.logistic_loss_grad(z, y, W, b)
        b -= 2.0 * db
    _, _, db = orc.logistic_loss_grad(z, y, W, b)
    assert np.abs(db).max() < 1e-9                               # mean softmax = q
    logit = z @ W.T + b
    p = np.exp(logit - logit.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    assert np.allclose(p.mean(0), q, atol=1e-8)


def test_route_linear_brute_force_and_relation_to_kmeans():
    rng = np.random.default_rng(34)
    W = rng.integers(-2, 3, size=(6, 4)).astype(np.float64)
    W[4] = W[1]
    b = rng.integers(-1, 2, size=6).astype(np.float64)
    b[4] = b[1]                                                   # class 4 duplicates class 1: ties go to 1
    z = rng.integers(-3, 4, size=(50, 4)).astype(np.float64)
    idx, hist, margin = orc.route_linear(z, W, b)
    for n in range(50):
        logits = [sum(W[k][d] * z[n][d] for d in range(4)) + b[k] for k in range(6)]
        best = max(logits)
        assert idx[n] == logits.index(best)
        assert margin[n] == best - sorted(logits)[-2]
    assert hist[4] == 0 and hist.sum() == 50
    # with w_k = 2 c_k and b_k = -||c_k||^2 the linear router is the k-means router of eq. 1
    c = rng.standard_normal((7, 5))
    x = rng.standard_normal((60, 5))
    i_lin, h_lin, _ = orc.route_linear(x, 2.0 * c, -(c * c).sum(1))
    i_km, h_km, _ = orc.route_prefix(x, c)
    assert np.array_equal(i_lin, i_km) and np.array_equal(h_lin, h_km)
    i1, h1, m1 = orc.route_linear(x, c[:1], np.zeros(1))
    assert np.all(i1 == 0) and np.all(np.isinf(m1))


# ---- routing more often at evaluation -------------------------------------------------------------------------------
def test_window_targets_and_chunk_scores_special_cases():
    rng = np.random.default_rng(41)
    P, n, L = 3, 4, 12
    S = -rng.uniform(0.5, 6.0, size=(P, n, L))                    # log-likelihoods
    # a window of one token: the per-token best path; a window past the end: the best path for the rest of the text
    assert np.array_equal(orc.window_targets(S, 1), np.argmax(S, axis=0))
    suffix = np.cumsum(S[:, :, ::-1], axis=2)[:, :, ::-1]
    assert np.array_equal(orc.window_targets(S, L + 5), np.argmax(suffix, axis=0))
    T3 = orc.window_targets(S, 3)
    assert T3[2, 4] == int(np.argmax([S[p, 2, 4] + S[p, 2, 5] + S[p, 2, 6] for p in range(P)]))
    assert T3[1, L - 1] == int(np.argmax(S[:, 1, L - 1]))
    # exact ties go to the lowest path
    S2 = S.copy()
    S2[2] = S2[0]
    assert not np.any(orc.window_targets(S2, 4) == 2)
    # one chunk, one path per document: that path's document score; chunks of one token routed by the per-token
    # best path: no worse than any single path and equal to the sum of per-token maxima
    one = orc.chunk_routed_scores(S, [[1]] * n, L)
    assert np.allclose(one, S[1].sum(1), atol=1e-13)
    per_tok = orc.chunk_routed_scores(S, np.argmax(S, axis=0), 1)
    assert np.allclose(per_tok, S.max(0).sum(1), atol=1e-13) and np.all(per_tok >= S.sum(2).max(0) - 1e-13)
    # ragged last chunk, by hand
    ch = [[0, 2, 1]] * n                                           # chunks [0,5) [5,10) [10,12)
    got = orc.chunk_routed_scores(S, ch, 5)
    assert np.allclose(got, S[0, :, :5].sum(1) + S[2, :, 5:10].sum(1) + S[1, :, 10:].sum(1), atol=1e-13)


def test_route_rows_of_nan_distances_take_the_first_centroid():
    """What eq. (1) written out with numpy gives for a document whose features hold a NaN (every distance is NaN):
    the first centroid, a NaN margin, and (first, second) centroid in the top-2 form.  The library documents the same
    rule for such rows; rows of finite features are not affected by their presence."""
    rng = np.random.default_rng(3)
    c = rng.standard_normal((6, 5))
    z = rng.standard_normal((9, 5))
    clean_idx, _, clean_margin = orc.route_prefix(z, c)
    z_bad = z.copy()
    z_bad[4, 2] = np.nan
    with np.errstate(invalid="ignore"):
        idx, hist, margin = orc.route_prefix(z_bad, c)
        idx2, _ = orc.route_prefix_top2(z_bad, c)
    assert idx[4] == 0 and np.isnan(margin[4]) and tuple(idx2[4]) == (0, 1)
    keep = np.arange(9) != 4
    assert np.array_equal(idx[keep], clean_idx[keep]) and np.array_equal(margin[keep], clean_margin[keep])
    assert hist.sum() == 9
