"""GPU parity of the path step (loss, per-token NLL, every gradient tensor) and of the whole inner/outer round
against the oracle, through the five C-ABI calls.

Tolerances (fp32): loss rel <= 1e-5, gradients and parameters rel <= 1e-4 per tensor (L2).  bf16: loss rel <= 2e-2;
gradients are checked per tensor at rel <= 6e-2 as a supplementary bound (operands and activations are rounded to
8 significant bits, accumulation is fp32).
"""
import math

import numpy as np
import pytest
import torch

import dipaco_inputs as gen
import paper_2403_10616_amd as dp
from oracle import dipaco_oracle as orc
from gpu_util import DEV, PathState, dev, host, make_arch, per_tensor_maxabs, per_tensor_rel, rel_l2

pytestmark = pytest.mark.gpu

SHAPES = {
    # several GEMM tiles with ragged tails (tokens = 3*50 = 150, widths not multiples of 128), heads*d_head != d_model
    "ragged": dict(layers_per_level=(1, 2), d_model=72, n_heads=3, d_head=32, d_mlp=200, vocab=264, max_seq=56),
    "wide": dict(layers_per_level=(1, 1), d_model=256, n_heads=2, d_head=64, d_mlp=520, vocab=1000, max_seq=160),
    "one_level": dict(layers_per_level=(2,), d_model=64, n_heads=1, d_head=128, d_mlp=64, vocab=64, max_seq=16),
    # a vocabulary row too long for the register-resident cross-entropy kernel: the three-pass kernel runs
    "big_vocab": dict(layers_per_level=(1,), d_model=64, n_heads=2, d_head=32, d_mlp=64, vocab=40000, max_seq=8),
    # the widest models the library takes: the embedding gradient's 16 partial rows need 96 / 128 KB of LDS
    "d1536": dict(layers_per_level=(1,), d_model=1536, n_heads=2, d_head=64, d_mlp=264, vocab=512, max_seq=24),
    "d2048": dict(layers_per_level=(1, 1), d_model=2048, n_heads=1, d_head=128, d_mlp=136, vocab=264, max_seq=16),
}


def _batch(cfg, B, S, seed, mask_prefix=0, zipf=False):
    if zipf:
        seqs = gen.zipf_tokens((B, S + 1), cfg["vocab"], 1.1, seed)
    else:
        seqs = gen.uniform_tokens((B, S + 1), cfg["vocab"], seed)
    tok, tgt = gen.split_inputs_targets(seqs)
    tgt = tgt.copy()
    if mask_prefix:
        tgt[:, :mask_prefix] = -1
    return tok, tgt


@pytest.mark.parametrize("name,B,S,mask", [("ragged", 3, 50, 0), ("ragged", 2, 56, 5), ("wide", 2, 160, 32),
                                           ("one_level", 5, 16, 0), ("one_level", 1, 1, 0), ("big_vocab", 2, 8, 1),
                                           ("d1536", 3, 24, 0), ("d2048", 4, 16, 2)])
def test_fp32_loss_and_gradients_match_oracle(name, B, S, mask):
    print(f"fp32 path {name} B={B} S={S} mask={mask}", flush=True)
    cfg = SHAPES[name]
    a, ctx = make_arch(cfg, dp.F32)
    lay = orc.param_layout(a)
    # entries of N(0, 0.08), narrower for the widest models so that pre-activations stay O(1) (at width 2048 a scale
    # of 0.08 gives attention scores of +-13, a softmax so peaked that fp32 gradients lose three digits on both sides)
    theta = gen.random_params(orc.param_count(a), seed=5, scale=min(0.08, 1.5 / math.sqrt(cfg["d_model"])))
    # LayerNorm gains near 1 so that activations keep a realistic scale
    for n_, (off, shape, _) in lay.items():
        if n_.endswith("_g"):
            theta[off:off + shape[0]] += 1.0
    tok, tgt = _batch(cfg, B, S, seed=6, mask_prefix=mask)
    st = PathState(ctx, theta, B, S)
    loss = st.fwd_bwd(tok, tgt)
    o_loss, o_grad = orc.path_loss_and_grad(theta, a, tok, tgt)
    assert abs(loss - o_loss) <= 1e-5 * abs(o_loss)
    nll = host(st.nll).reshape(B, S)
    o_nll = orc.path_token_nll(theta, a, tok, tgt)
    assert np.abs(nll - o_nll).max() <= 2e-5 * max(1.0, np.abs(o_nll).max())
    assert np.all(nll[tgt < 0] == 0.0)
    worst, where = per_tensor_rel(lay, host(st.grads), o_grad)
    assert worst <= 1e-4, (where, worst)
    # bit-reproducible
    g0 = host(st.grads).copy()
    loss2 = st.fwd_bwd(tok, tgt)
    assert loss2 == loss and np.array_equal(g0, host(st.grads))


def test_config1_full_round_matches_oracle():
    """Tiny 2x2 grid, fp32: compose -> 2 inner AdamW steps on each of the 4 paths -> outer Nesterov step of the
    4 block modules (2 paths each) and of the stem and head (shared by all 4 paths)."""
    cfg = gen.CONFIGS[1]
    a, ctx = make_arch(cfg, dp.F32)
    K = cfg["K"]
    B, S, steps = cfg["batch"], cfg["seq"], cfg["inner_steps"]
    lay = orc.param_layout(a)
    bounds = orc.segment_bounds(a)
    n = orc.param_count(a)
    # global modules: stem, K[0] level-1 modules, K[1] level-2 modules, head -- distinct seeded inits
    def seg(level, e):
        full = gen.init_params(lay, a.n_layers, seed=1000 * level + e)
        lo, hi = bounds[level]
        return full[lo:hi].copy()
    glob = {(0, 0): seg(0, 0), (3, 0): seg(3, 0)}
    for l in (1, 2):
        for e in range(K[l - 1]):
            glob[(l, e)] = seg(l, e)
    seqs = gen.uniform_tokens((4, steps, B, S + 1), cfg["vocab"], cfg["seed"])
    mask = orc.decay_mask(a)

    gpu_local, orc_local, losses = {}, {}, []
    for j in range(4):
        mods = dp.dipaco_path_modules(j, K)
        assert mods == orc.modules_of_path(j, K)
        keys = [(0, 0), (1, mods[0]), (2, mods[1]), (3, 0)]
        segs = [glob[k] for k in keys]
        master = torch.empty(n, dtype=torch.float32, device=DEV)
        dp.dipaco_compose_path(ctx, [dev(s) for s in segs], master, None)
        th_o = orc.compose_path(segs)
        assert np.array_equal(host(master).astype(np.float64), th_o)
        st = PathState(ctx, host(master), B, S)
        m_o, v_o = np.zeros(n), np.zeros(n)
        for t in range(steps):
            tok, tgt = gen.split_inputs_targets(seqs[j, t])
            loss = st.fwd_bwd(tok, tgt)
            st.adamw(t + 1, cfg["lr"], cfg["beta1"], cfg["beta2"], cfg["eps"], cfg["wd"])
            o_loss, o_g = orc.path_loss_and_grad(th_o, a, tok, tgt)
            assert abs(loss - o_loss) <= 1e-5 * abs(o_loss), (j, t)
            th_o, m_o, v_o = orc.adamw_step(th_o, o_g, m_o, v_o, t + 1, cfg["lr"], cfg["beta1"], cfg["beta2"],
                                            cfg["eps"], cfg["wd"], mask)
            losses.append((loss, o_loss))
        # The key bias has an identically zero gradient (adding one vector to every key shifts all scores of a
        # query equally, which softmax ignores), so what either side feeds AdamW there is rounding noise, and
        # AdamW's g/(|g|+eps) turns noise of size ~eps into steps of size ~lr.  Those entries are compared
        # against AdamW's step bound instead of the oracle's value.
        got = host(st.master).astype(np.float64)
        A = a.d_attn
        for layer in range(a.n_layers):
            off = lay[f"blk{layer}.b_qkv"][0]
            ksl = slice(off + A, off + 2 * A)
            assert np.abs(o_g[ksl]).max() <= 1e-9 * np.abs(o_g[off:off + A]).max()
            assert np.abs(got[ksl]).max() <= steps * cfg["lr"] * 1.001
            got[ksl] = th_o[ksl]
        worst, where = per_tensor_rel(lay, got, th_o)
        assert worst <= 1e-4, (j, where, worst)
        gpu_local[j], orc_local[j] = st.master, th_o
    # outer step per module
    for (level, e), theta_prev in glob.items():
        lo, hi = bounds[level]
        if level in (0, 3):
            sharing = list(range(4))
        else:
            sharing = orc.paths_through_module(level - 1, e, K)
            assert len(sharing) == 2
        th_d = dev(theta_prev)
        buf_d = torch.zeros(hi - lo, dtype=torch.float32, device=DEV)
        ins = [gpu_local[j][lo:hi].clone() for j in sharing]     # 16-byte aligned copies of the paths' segments
        dp.dipaco_module_outer_step(th_d, buf_d, ins, None, hi - lo, False, cfg["outer_lr"], cfg["outer_momentum"])
        th_o, buf_o = orc.outer_step(theta_prev, np.zeros(hi - lo), [orc_local[j][lo:hi] for j in sharing], None, False,
                                     cfg["outer_lr"], cfg["outer_momentum"])
        assert rel_l2(host(th_d), th_o) <= 1e-4, (level, e)
        # the update itself (theta - theta_prev) is small against theta: check it on its own scale too
        assert rel_l2(host(th_d) - theta_prev, th_o - theta_prev) <= 2e-3, (level, e)


@pytest.mark.parametrize("name,B,S,mask", [("ragged", 3, 50, 4), ("wide", 2, 160, 0), ("d1536", 3, 24, 0),
                                           ("d2048", 4, 16, 2)])
def test_bf16_loss_and_gradients_close_to_oracle(name, B, S, mask):
    print(f"bf16 path {name} B={B} S={S}", flush=True)
    cfg = SHAPES[name]
    a, ctx = make_arch(cfg, dp.BF16)
    lay = orc.param_layout(a)
    theta = gen.init_params(lay, a.n_layers, seed=8)
    theta += gen.random_params(theta.size, seed=9, scale=0.02)          # non-zero biases, gains off 1
    theta = torch.from_numpy(theta).to(torch.bfloat16).float().numpy()  # masters exactly representable in bf16
    tok, tgt = _batch(cfg, B, S, seed=10, mask_prefix=mask, zipf=True)
    st = PathState(ctx, theta, B, S)
    loss = st.fwd_bwd(tok, tgt)
    o_loss, o_grad = orc.path_loss_and_grad(theta, a, tok, tgt)
    assert abs(loss - o_loss) <= 2e-2 * abs(o_loss)
    assert abs(loss - o_loss) <= 2e-3 * abs(o_loss)      # in practice an order of magnitude closer
    worst, where = per_tensor_rel(lay, host(st.grads), o_grad)
    assert worst <= 3e-2, (where, worst)                    # observed 4e-3 .. 1.2e-2
    worst_abs, where_abs = per_tensor_maxabs(lay, host(st.grads), o_grad)     # every element, on its tensor's scale
    print(f"  worst tensor rel-L2 {worst:.2e} ({where}), worst max-abs/max {worst_abs:.2e} ({where_abs})", flush=True)
    assert worst_abs <= 3e-2, (where_abs, worst_abs)        # observed 4e-3 .. 1.2e-2
    g0 = host(st.grads).copy()
    assert st.fwd_bwd(tok, tgt) == loss and np.array_equal(g0, host(st.grads))


# ---- router features: forward through the blocks, mean over the prefix ------------------------------------------
def _features_gpu(ctx, theta, tok):
    B, S = tok.shape
    n = dp.dipaco_path_param_count(ctx)
    master = dev(theta.astype(np.float32))
    lowp = master.to(torch.bfloat16) if ctx.compute == dp.BF16 else None
    out = torch.full((B, ctx_d(ctx)), 7.0, dtype=torch.float32, device=DEV)
    ws = torch.empty(dp.dipaco_features_workspace_bytes(ctx, B, S), dtype=torch.uint8, device=DEV)
    dp.dipaco_path_prefix_features(ctx, master, lowp, dev(tok.astype(np.int32)), B, S, out, ws)
    return host(out)


def ctx_d(ctx):
    return next(cols for name, _, rows, cols, _ in (dp.dipaco_tensor_info(ctx, i) for i in range(dp.dipaco_tensor_count(ctx)))
                if name == "tok_emb")


@pytest.mark.parametrize("name,B,S,compute,tol", [("ragged", 5, 32, dp.F32, 1e-5), ("wide", 130, 32, dp.F32, 1e-5),
                                                  ("one_level", 3, 1, dp.F32, 1e-5), ("wide", 130, 32, dp.BF16, 2e-2),
                                                  ("ragged", 7, 56, dp.BF16, 2e-2)])
def test_prefix_features_match_oracle(name, B, S, compute, tol):
    print(f"features {name} B={B} S={S} compute={compute}", flush=True)
    cfg = SHAPES[name]
    a, ctx = make_arch(cfg, compute)
    lay = orc.param_layout(a)
    theta = gen.random_params(orc.param_count(a), seed=31, scale=0.08)
    for n_, (off, shape, _) in lay.items():
        if n_.endswith("_g"):
            theta[off:off + shape[0]] += 1.0
    tok = gen.uniform_tokens((B, S), cfg["vocab"], 32)
    ref_theta = theta if compute == dp.F32 else torch.from_numpy(theta.astype(np.float32)).to(torch.bfloat16).float().numpy()
    want = orc.prefix_features(ref_theta, a, tok)
    got = _features_gpu(ctx, theta, tok)
    assert got.shape == want.shape
    assert rel_l2(got, want) <= tol
    assert np.abs(got - want).max() <= tol * 10 * np.abs(want).max()
    with pytest.raises(dp.DipacoError):      # workspace too small is refused on the host
        dp.dipaco_path_prefix_features(ctx, dev(theta.astype(np.float32)), None if compute == dp.F32 else dev(theta).to(torch.bfloat16),
                                       dev(tok.astype(np.int32)), B, S, torch.zeros((B, a.d_model), device=DEV),
                                       torch.empty(16, dtype=torch.uint8, device=DEV))


@pytest.mark.parametrize("name,B,S,compute,mask", [("ragged", 3, 50, dp.F32, 5), ("wide", 4, 160, dp.F32, 32),
                                                   ("wide", 4, 160, dp.BF16, 32), ("one_level", 2, 16, dp.F32, 0)])
def test_path_scores_match_oracle_and_training_loss(name, B, S, compute, mask):
    print(f"scores {name} B={B} S={S} compute={compute}", flush=True)
    cfg = SHAPES[name]
    a, ctx = make_arch(cfg, compute)
    lay = orc.param_layout(a)
    theta = gen.random_params(orc.param_count(a), seed=41, scale=0.08)
    for n_, (off, shape, _) in lay.items():
        if n_.endswith("_g"):
            theta[off:off + shape[0]] += 1.0
    tok, tgt = _batch(cfg, B, S, seed=42, mask_prefix=mask)
    master = dev(theta.astype(np.float32))
    lowp = master.to(torch.bfloat16) if compute == dp.BF16 else None
    score = torch.zeros(B, dtype=torch.float32, device=DEV)
    nll = torch.zeros(B * S, dtype=torch.float32, device=DEV)
    ws = torch.empty(dp.dipaco_score_workspace_bytes(ctx, B, S), dtype=torch.uint8, device=DEV)
    dp.dipaco_path_score(ctx, master, lowp, dev(tok.astype(np.int32)), dev(tgt.astype(np.int32)), B, S, score, nll, ws)
    ref_theta = theta if compute == dp.F32 else master.to(torch.bfloat16).float().cpu().numpy()
    want = orc.path_doc_scores(ref_theta, a, tok, tgt)
    tol = 1e-5 if compute == dp.F32 else 2e-2
    assert np.abs(host(score) - want).max() <= tol * np.abs(want).max()
    assert np.abs(host(nll).reshape(B, S).sum(1) + host(score)).max() <= 1e-3 * np.abs(want).max()
    # the forward pass of the training step gives the same per-token values
    st = PathState(ctx, theta, B, S)
    st.fwd_bwd(tok, tgt)
    assert np.abs(host(st.nll) - host(nll)).max() <= (1e-5 if compute == dp.F32 else 5e-2)
