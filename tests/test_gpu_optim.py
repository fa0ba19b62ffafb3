"""GPU parity of compose, AdamW and the module outer step against the oracle."""
import numpy as np
import pytest
import torch

import dipaco_inputs as gen
import paper_2403_10616_amd as dp
from oracle import dipaco_oracle as orc
from gpu_util import DEV, dev, host, make_arch, rel_l2

pytestmark = pytest.mark.gpu

SMALL = dict(layers_per_level=(2, 1), d_model=64, n_heads=2, d_head=32, d_mlp=136, vocab=264, max_seq=40)


@pytest.mark.parametrize("compute", [dp.F32, dp.BF16])
def test_compose_path_round_trip_and_bf16_image(compute):
    a, ctx = make_arch(SMALL, compute)
    bounds = orc.segment_bounds(a)
    rng = np.random.default_rng(0)
    segs = [rng.standard_normal(hi - lo).astype(np.float32) for lo, hi in bounds]
    want = orc.compose_path(segs)
    n = dp.dipaco_path_param_count(ctx)
    master = torch.zeros(n, dtype=torch.float32, device=DEV)
    lowp = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    dp.dipaco_compose_path(ctx, [dev(s) for s in segs], master, lowp)
    assert np.array_equal(host(master).astype(np.float64), want)
    # bf16 image: round-to-nearest-even of every element, bit-exact against torch's cast
    assert torch.equal(lowp.cpu(), torch.from_numpy(want.astype(np.float32)).to(torch.bfloat16))
    master.zero_()
    dp.dipaco_compose_path(ctx, [dev(s) for s in segs], master, None)
    assert np.array_equal(host(master).astype(np.float64), want)


@pytest.mark.parametrize("compute", [dp.F32, dp.BF16])
def test_adamw_three_steps_match_oracle(compute):
    a, ctx = make_arch(SMALL, compute)
    n = orc.param_count(a)
    mask = orc.decay_mask(a)
    rng = np.random.default_rng(1)
    theta = rng.standard_normal(n).astype(np.float32)
    th_d = dev(theta)
    m_d = torch.zeros(n, dtype=torch.float32, device=DEV)
    v_d = torch.zeros(n, dtype=torch.float32, device=DEV)
    lowp = torch.zeros(n, dtype=torch.bfloat16, device=DEV) if compute == dp.BF16 else None
    th_o, m_o, v_o = theta.astype(np.float64), np.zeros(n), np.zeros(n)
    for step in (1, 2, 3):
        g = (rng.standard_normal(n) * 10.0 ** rng.integers(-6, 1, size=n)).astype(np.float32)
        g[::97] = 0.0
        dp.dipaco_inner_adamw(ctx, th_d, dev(g), m_d, v_d, lowp, step, 1e-3, 0.9, 0.95, 1e-8, 0.1)
        th_o, m_o, v_o = orc.adamw_step(th_o, g, m_o, v_o, step, 1e-3, 0.9, 0.95, 1e-8, 0.1, mask)
        assert np.abs(host(th_d) - th_o).max() <= 2e-6 * np.abs(th_o).max()
        assert rel_l2(host(th_d), th_o) <= 1e-6 and rel_l2(host(m_d), m_o) <= 1e-6 and rel_l2(host(v_d), v_o) <= 1e-6
    # decay really is confined to the matrices: a zero-gradient step moves only decayed entries
    before = host(th_d).copy()
    m_d.zero_(); v_d.zero_()
    dp.dipaco_inner_adamw(ctx, th_d, torch.zeros_like(th_d), m_d, v_d, lowp, 1, 1e-2, 0.9, 0.95, 1e-8, 0.5)
    moved = host(th_d) != before
    assert np.array_equal(moved, (mask > 0) & (before != 0))
    if lowp is not None:
        assert torch.equal(lowp.cpu(), th_d.cpu().to(torch.bfloat16))


@pytest.mark.parametrize("n_paths,n_elems,weighted,is_delta", [
    (1, 1000, False, False), (2, 4096 + 3, True, False), (16, 70_001, True, True), (16, 1 << 20, True, False),
    (5, 12_345, False, True), (37, 9_999, True, False), (256, 2_048, True, False)])
def test_outer_step_matches_oracle_over_two_steps(n_paths, n_elems, weighted, is_delta):
    rng = np.random.default_rng(n_paths)
    theta = (rng.standard_normal(n_elems) * 0.02).astype(np.float32)
    th_d, buf_d = dev(theta), torch.zeros(n_elems, dtype=torch.float32, device=DEV)
    th_o, buf_o = theta.astype(np.float64), np.zeros(n_elems)
    w = gen.shard_weights(n_paths, 3) if weighted else None
    for step in range(2):
        eps = [gen.perturbation(n_elems, 1e-3, 300 + 16 * step + i) for i in range(n_paths)]
        cur = host(th_d).copy()
        ins = [(-e if is_delta else cur + e) for e in eps]         # theta_i = theta + eps  =>  delta_i = -eps
        ins = [np.asarray(x, dtype=np.float32) for x in ins]
        dp.dipaco_module_outer_step(th_d, buf_d, [dev(x) for x in ins], w, n_elems, is_delta, 0.7, 0.9)
        th_o, buf_o = orc.outer_step(cur, buf_o, ins, w, is_delta, 0.7, 0.9)
        assert rel_l2(host(th_d), th_o) <= 1e-6
        assert rel_l2(host(buf_d), buf_o) <= 2e-5      # delta is a small difference of fp32 numbers
        buf_o = host(buf_d).astype(np.float64)          # continue from the device state, as th does


def test_outer_step_special_cases():
    n = 5000
    rng = np.random.default_rng(0)
    theta = rng.standard_normal(n).astype(np.float32)
    local = (theta + rng.standard_normal(n).astype(np.float32) * 0.01).astype(np.float32)
    # one path, no momentum, lr 1: the module becomes the path's copy (plain SGD on the delta)
    th_d, buf_d = dev(theta), torch.zeros(n, dtype=torch.float32, device=DEV)
    dp.dipaco_module_outer_step(th_d, buf_d, [dev(local)], None, n, False, 1.0, 0.0)
    assert np.abs(host(th_d) - local).max() <= 1e-6
    # permutation of the inputs changes nothing beyond fp32 reassociation
    ins = [(theta + gen.perturbation(n, 1e-3, i)).astype(np.float32) for i in range(8)]
    w = gen.shard_weights(8, 1)
    outs = []
    for perm in (list(range(8)), [3, 1, 7, 0, 2, 6, 5, 4]):
        th_d, buf_d = dev(theta), torch.zeros(n, dtype=torch.float32, device=DEV)
        dp.dipaco_module_outer_step(th_d, buf_d, [dev(ins[i]) for i in perm], w[perm], n, False, 0.7, 0.9)
        outs.append(host(th_d).copy())
    assert np.abs(outs[0] - outs[1]).max() <= 1e-6
    # rejected inputs
    with pytest.raises(dp.DipacoError):
        dp.dipaco_module_outer_step(th_d, buf_d, [dev(ins[0])], [0.0], n, False, 0.7, 0.9)


@pytest.mark.parametrize("n_paths,n_elems,weighted,is_delta,scale", [
    (1, 1000, False, False, 1.0), (3, 4096 + 3, True, False, 1.0), (16, 70_001, True, True, 4.0),
    (16, 1 << 20, True, False, 4.0), (5, 2, False, True, 2.0)])
def test_streaming_outer_step_matches_oracle_and_one_shot_form(n_paths, n_elems, weighted, is_delta, scale):
    rng = np.random.default_rng(40 + n_paths)
    theta = (rng.standard_normal(n_elems) * 0.02).astype(np.float32)
    buf0 = (rng.standard_normal(n_elems) * 1e-3).astype(np.float32)
    w = gen.shard_weights(n_paths, 3) if weighted else np.ones(n_paths)
    eps = [gen.perturbation(n_elems, 1e-3, 700 + i) for i in range(n_paths)]
    ins = [np.asarray(-e if is_delta else theta + e, dtype=np.float32) for e in eps]
    th_d, buf_d = dev(theta), dev(buf0)
    prev_d = dev(theta)                                          # theta_prev stays untouched while paths arrive
    acc = torch.full((n_elems,), 123.0, dtype=torch.float32, device=DEV)   # garbage: the first call overwrites
    for i, x in enumerate(ins):
        dp.dipaco_module_delta_accumulate(acc, None if is_delta else prev_d, dev(x), float(w[i]), n_elems, is_delta,
                                          i == 0)
    dp.dipaco_module_outer_apply(th_d, buf_d, acc, float(np.sum(w.astype(np.float64))), scale, n_elems, 0.7, 0.9)
    th_o, buf_o = orc.outer_step_streaming(theta, buf0, ins, w, is_delta, 0.7, 0.9, norm_scale=scale)
    assert rel_l2(host(th_d), th_o) <= 1e-6
    assert rel_l2(host(buf_d), buf_o) <= 2e-5
    if scale == 1.0:                                              # same numbers as the one-shot entry point
        th1, buf1 = dev(theta), dev(buf0)
        dp.dipaco_module_outer_step(th1, buf1, [dev(x) for x in ins], w if weighted else None, n_elems, is_delta, 0.7,
                                    0.9)
        assert np.abs(host(th1) - host(th_d)).max() <= 1e-6


def test_streaming_outer_step_rejects_bad_arguments():
    t = torch.zeros(16, dtype=torch.float32, device=DEV)
    with pytest.raises(dp.DipacoError):
        dp.dipaco_module_delta_accumulate(t, t, t, 0.0, 16, False, True)
    with pytest.raises(dp.DipacoError):
        dp.dipaco_module_delta_accumulate(t, None, t, 1.0, 16, False, True)    # theta_prev needed for local copies
    with pytest.raises(dp.DipacoError):
        dp.dipaco_module_outer_apply(t, t, t, 0.0, 1.0, 16, 0.7, 0.9)
    with pytest.raises(dp.DipacoError):
        dp.dipaco_module_outer_apply(t, t, t, 1.0, float("nan"), 16, 0.7, 0.9)


def _grid_modules(seed, sizes, path_counts, weighted, is_delta, scales):
    """host arrays of a table of modules: sizes / path counts / norm scales per module"""
    rng = np.random.default_rng(seed)
    mods = []
    for m, (n, P) in enumerate(zip(sizes, path_counts)):
        theta = (rng.standard_normal(n) * 0.02).astype(np.float32)
        buf = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        eps = [gen.perturbation(n, 1e-3, 900 + 17 * m + i) for i in range(P)]
        ins = [np.asarray(-e if is_delta[m] else theta + e, dtype=np.float32) for e in eps]
        w = gen.shard_weights(P, 5 + m) if weighted[m] else None
        mods.append(dict(theta=theta, momentum=buf, inputs=ins, weights=w, is_delta=is_delta[m], norm_scale=scales[m],
                         n_elems=n))
    return mods


@pytest.mark.parametrize("case", ["mixed", "many_small", "single"])
def test_table_outer_step_matches_oracle_and_per_module_calls(case):
    """Shared modules of different sizes and path counts and path-specific modules (one path) in one launch."""
    if case == "mixed":
        sizes = [70_001, 4096, 0, 3, 1 << 20, 4097, 12_288]
        paths = [16, 1, 2, 5, 4, 1, 256]
    elif case == "many_small":
        sizes = [1 + (37 * i) % 9000 for i in range(300)]
        paths = [1 + i % 3 for i in range(300)]
    else:
        sizes, paths = [123_457], [16]
    M = len(sizes)
    weighted = [i % 2 == 0 for i in range(M)]
    is_delta = [i % 3 == 0 for i in range(M)]
    scales = [1.0 if i % 4 else float(np.sqrt(paths[i])) for i in range(M)]
    mods = _grid_modules(77, sizes, paths, weighted, is_delta, scales)
    # every buffer is a view into one arena at a 16-byte aligned offset (n_elems = 3 leaves odd sizes behind)
    dmods = []
    for m in mods:
        dmods.append(dict(m, theta=dev(m["theta"]) if m["n_elems"] else torch.zeros(4, device=DEV),
                          momentum=dev(m["momentum"]) if m["n_elems"] else torch.zeros(4, device=DEV),
                          inputs=[dev(x) if m["n_elems"] else torch.zeros(4, device=DEV) for x in m["inputs"]]))
    image = dp.dipaco_outer_table_pack(dmods)
    table = torch.frombuffer(bytearray(image), dtype=torch.uint8).to(DEV)
    dp.dipaco_outer_step_table(image, table, 0.7, 0.9)
    want = orc.outer_step_modules(mods, 0.7, 0.9)
    for m, d, (th_o, buf_o) in zip(mods, dmods, want):
        n = m["n_elems"]
        if n == 0:
            continue
        assert rel_l2(host(d["theta"]), th_o) <= 1e-6
        assert rel_l2(host(d["momentum"]), buf_o) <= 2e-5
        if m["norm_scale"] == 1.0:        # the single-module entry point gives the same numbers
            th1, buf1 = dev(m["theta"]), dev(m["momentum"])
            dp.dipaco_module_outer_step(th1, buf1, [dev(x) for x in m["inputs"]], m["weights"], n, m["is_delta"], 0.7,
                                        0.9)
            assert np.abs(host(th1) - host(d["theta"])).max() <= 1e-6
    # a second step with the same table (momentum carried over) still follows the oracle
    dp.dipaco_outer_step_table(image, table, 0.7, 0.9)
    mods2 = [dict(m, theta=th, momentum=buf) for m, (th, buf) in zip(mods, want)]
    for m in mods2:                       # inputs that were local copies keep their values; deltas too
        pass
    want2 = orc.outer_step_modules(mods2, 0.7, 0.9)
    for m, d, (th_o, _b) in zip(mods, dmods, want2):
        if m["n_elems"]:
            assert rel_l2(host(d["theta"]), th_o) <= 2e-6


def test_synchronous_baseline_step_is_gradient_mean_plus_adamw():
    """The fully synchronous ablation of Section 4.5 exchanges and aggregates gradients module by module at every step: on one device its arithmetic is
    the mean of the gradients of the paths that share the parameters, followed by the inner optimiser.  Both pieces
    exist (the accumulation entry point with ready-made inputs, then AdamW); here they are chained at config-1 size
    and checked against the oracle's mean + AdamW over three steps."""
    a, ctx = make_arch(SMALL, dp.F32)
    n = orc.param_count(a)
    mask = orc.decay_mask(a)
    P = 4
    rng = np.random.default_rng(11)
    theta = rng.standard_normal(n).astype(np.float32)
    th_d = dev(theta)
    m_d = torch.zeros(n, dtype=torch.float32, device=DEV)
    v_d = torch.zeros(n, dtype=torch.float32, device=DEV)
    acc = torch.empty(n, dtype=torch.float32, device=DEV)
    th_o, m_o, v_o = theta.astype(np.float64), np.zeros(n), np.zeros(n)
    for step in (1, 2, 3):
        gs = [rng.standard_normal(n).astype(np.float32) for _ in range(P)]
        for i, g in enumerate(gs):
            dp.dipaco_module_delta_accumulate(acc, None, dev(g), 1.0 / P, n, True, i == 0)
        dp.dipaco_inner_adamw(ctx, th_d, acc, m_d, v_d, None, step, 1e-3, 0.9, 0.95, 1e-8, 0.1)
        g_mean = sum(g.astype(np.float64) for g in gs) / P
        assert rel_l2(host(acc), g_mean) <= 1e-6
        th_o, m_o, v_o = orc.adamw_step(th_o, g_mean, m_o, v_o, step, 1e-3, 0.9, 0.95, 1e-8, 0.1, mask)
        assert rel_l2(host(th_d), th_o) <= 1e-6 and rel_l2(host(m_d), m_o) <= 1e-6 and rel_l2(host(v_d), v_o) <= 2e-6
