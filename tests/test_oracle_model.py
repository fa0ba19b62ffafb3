"""Pins for the oracle's path forward / backward (CPU only).

What fixes the expected values here is not the oracle itself:
  * central finite differences of the oracle's own scalar loss (checks backward against forward),
  * an independent build of the same network from torch's library routines (layer_norm, scaled-dot-product
    attention with the causal flag, exact GELU, cross_entropy) differentiated by autograd (checks forward and
    backward against library definitions),
  * closed forms and structural facts: zero head => loss = ln V; causality; one position => attention is the
    identity on v; the mean loss does not depend on the order of the sequences.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import dipaco_inputs as gen
from oracle import dipaco_oracle as orc

TINY = orc.Arch(layers_per_level=(1, 1), d_model=8, n_heads=2, d_head=4, d_mlp=16, vocab=11, max_seq=6)
# heads * d_head != d_model on purpose (the paper's own 150M has 16 heads of 64 on width 896)
WIDE = orc.Arch(layers_per_level=(2, 1), d_model=12, n_heads=3, d_head=8, d_mlp=20, vocab=13, max_seq=8)


def _data(a, B, S, seed, mask_prefix=0):
    seqs = gen.uniform_tokens((B, S + 1), a.vocab, seed)
    tok, tgt = gen.split_inputs_targets(seqs)
    tgt = tgt.copy()
    if mask_prefix:
        tgt[:, :mask_prefix] = -1
    return tok, tgt


def _torch_hidden(p, a, tok):
    """residual stream after the last block, [B, S, d], built from torch's library routines"""
    B, S = tok.shape
    x = p["tok_emb"][tok] + p["pos_emb"][:S]
    A, H, dh = a.d_attn, a.n_heads, a.d_head
    for l in range(a.n_layers):
        w = lambda n: p[f"blk{l}.{n}"]
        h = F.layer_norm(x, (a.d_model,), w("ln1_g"), w("ln1_b"), a.ln_eps)
        qkv = h @ w("w_qkv") + w("b_qkv")
        q, k, v = [t.reshape(B, S, H, dh).transpose(1, 2) for t in qkv.split(A, dim=-1)]
        o = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(B, S, A)
        x = x + o @ w("w_o") + w("b_o")
        h = F.layer_norm(x, (a.d_model,), w("ln2_g"), w("ln2_b"), a.ln_eps)
        x = x + F.gelu(h @ w("w_up") + w("b_up")) @ w("w_down") + w("b_down")
    return x


def _torch_loss(flat, a, tok, tgt):
    lay = orc.param_layout(a)
    p = {n: flat[o:o + int(np.prod(s))].reshape(s) for n, (o, s, _) in lay.items()}
    B, S = tok.shape
    tok = torch.as_tensor(tok, dtype=torch.long)
    tgt = torch.as_tensor(tgt, dtype=torch.long)
    x = p["tok_emb"][tok] + p["pos_emb"][:S]
    A, H, dh = a.d_attn, a.n_heads, a.d_head
    for l in range(a.n_layers):
        w = lambda n: p[f"blk{l}.{n}"]
        h = F.layer_norm(x, (a.d_model,), w("ln1_g"), w("ln1_b"), a.ln_eps)
        qkv = h @ w("w_qkv") + w("b_qkv")
        q, k, v = [t.reshape(B, S, H, dh).transpose(1, 2) for t in qkv.split(A, dim=-1)]
        o = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(B, S, A)
        x = x + o @ w("w_o") + w("b_o")
        h = F.layer_norm(x, (a.d_model,), w("ln2_g"), w("ln2_b"), a.ln_eps)
        x = x + F.gelu(h @ w("w_up") + w("b_up")) @ w("w_down") + w("b_down")
    y = F.layer_norm(x, (a.d_model,), p["lnf_g"], p["lnf_b"], a.ln_eps)
    logits = y @ p["w_head"]
    n_t = int((tgt >= 0).sum())
    return F.cross_entropy(logits.reshape(B * S, -1), tgt.reshape(-1), ignore_index=-1, reduction="sum") / n_t


@pytest.mark.parametrize("a,B,S,mask", [(TINY, 2, 5, 0), (WIDE, 3, 7, 2), (TINY, 1, 6, 3)])
def test_loss_and_grad_match_autograd_build(a, B, S, mask):
    n = orc.param_count(a)
    theta = gen.random_params(n, seed=7, scale=0.3, dtype=np.float64)
    tok, tgt = _data(a, B, S, seed=11, mask_prefix=mask)
    loss, grad = orc.path_loss_and_grad(theta, a, tok, tgt)
    t = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
    tl = _torch_loss(t, a, tok, tgt)
    tl.backward()
    assert abs(loss - tl.item()) <= 1e-12 * abs(tl.item())
    tg = t.grad.numpy()
    lay = orc.param_layout(a)
    for name, (off, shape, _) in lay.items():
        sl = slice(off, off + int(np.prod(shape)))
        ref = tg[sl]
        if name == "pos_emb":      # rows beyond S get no gradient
            assert np.all(grad[sl].reshape(shape)[S:] == 0.0)
        denom = np.linalg.norm(ref)
        assert denom > 0, name
        assert np.linalg.norm(grad[sl] - ref) <= 1e-10 * denom, name


@pytest.mark.parametrize("a,B,S,mask", [(TINY, 2, 4, 0), (WIDE, 2, 5, 1)])
def test_grad_matches_central_finite_differences(a, B, S, mask):
    n = orc.param_count(a)
    theta = gen.random_params(n, seed=3, scale=0.3, dtype=np.float64)
    tok, tgt = _data(a, B, S, seed=5, mask_prefix=mask)
    _, grad = orc.path_loss_and_grad(theta, a, tok, tgt)
    lay = orc.param_layout(a)
    rng = np.random.default_rng(0)
    h = 1e-5
    for name, (off, shape, _) in lay.items():
        size = int(np.prod(shape))
        rows = S if name == "pos_emb" else None
        picks = rng.choice(size if rows is None else rows * shape[1], size=min(6, size), replace=False)
        fd = np.empty(len(picks))
        for i, k in enumerate(picks):
            tp = theta.copy(); tp[off + k] += h
            tm = theta.copy(); tm[off + k] -= h
            fd[i] = (orc.path_loss(tp, a, tok, tgt) - orc.path_loss(tm, a, tok, tgt)) / (2 * h)
        an = grad[off + picks]
        assert np.linalg.norm(fd - an) <= 1e-6 * max(np.linalg.norm(an), 1e-3), (name, fd, an)


def test_zero_head_gives_log_vocab():
    a = WIDE
    lay = orc.param_layout(a)
    theta = gen.random_params(orc.param_count(a), seed=1, scale=0.5, dtype=np.float64)
    orc.view(theta, lay, "w_head")[...] = 0.0
    tok, tgt = _data(a, 2, 6, seed=2)
    assert abs(orc.path_loss(theta, a, tok, tgt) - math.log(a.vocab)) < 1e-13
    nll = orc.path_token_nll(theta, a, tok, tgt)
    assert np.allclose(nll, math.log(a.vocab), atol=1e-13)


def test_causality_later_tokens_do_not_change_earlier_logits():
    a = WIDE
    theta = gen.random_params(orc.param_count(a), seed=4, scale=0.4, dtype=np.float64)
    tok, _ = _data(a, 1, 8, seed=9)
    base = orc.path_logits(theta, a, tok)
    tok2 = tok.copy()
    tok2[0, 5] = (tok2[0, 5] + 1) % a.vocab
    moved = orc.path_logits(theta, a, tok2)
    assert np.array_equal(base[0, :5], moved[0, :5])
    assert not np.allclose(base[0, 5:], moved[0, 5:])


def test_single_position_attention_is_identity_on_v():
    """With S = 1 the softmax has one entry, so o = v: block output is computable without any attention code."""
    a = orc.Arch(layers_per_level=(1,), d_model=8, n_heads=2, d_head=4, d_mlp=16, vocab=7, max_seq=1)
    lay = orc.param_layout(a)
    theta = gen.random_params(orc.param_count(a), seed=8, scale=0.4, dtype=np.float64)
    tok = np.array([[3]], dtype=np.int32)
    logits = orc.path_logits(theta, a, tok)[0, 0]
    v_ = lambda n: orc.view(theta, lay, n)

    def ln(x, g, b):
        mu = x.mean(); var = ((x - mu) ** 2).mean()
        return (x - mu) / math.sqrt(var + a.ln_eps) * g + b
    x = v_("tok_emb")[3] + v_("pos_emb")[0]
    qkv = ln(x, v_("blk0.ln1_g"), v_("blk0.ln1_b")) @ v_("blk0.w_qkv") + v_("blk0.b_qkv")
    x = x + qkv[2 * a.d_attn:] @ v_("blk0.w_o") + v_("blk0.b_o")
    u = ln(x, v_("blk0.ln2_g"), v_("blk0.ln2_b")) @ v_("blk0.w_up") + v_("blk0.b_up")
    act = np.array([0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in u])
    x = x + act @ v_("blk0.w_down") + v_("blk0.b_down")
    want = ln(x, v_("lnf_g"), v_("lnf_b")) @ v_("w_head")
    assert np.allclose(logits, want, rtol=1e-12, atol=1e-13)


def test_sequence_order_does_not_change_mean_loss():
    a = TINY
    theta = gen.random_params(orc.param_count(a), seed=6, scale=0.3, dtype=np.float64)
    tok, tgt = _data(a, 4, 6, seed=13)
    perm = np.array([2, 0, 3, 1])
    l0, g0 = orc.path_loss_and_grad(theta, a, tok, tgt)
    l1, g1 = orc.path_loss_and_grad(theta, a, tok[perm], tgt[perm])
    assert abs(l0 - l1) < 1e-13
    assert np.allclose(g0, g1, rtol=1e-11, atol=1e-15)


def test_param_counts_of_the_benchmark_architectures():
    c = gen.CONFIGS[2]
    a = orc.Arch(c["layers_per_level"], c["d_model"], c["n_heads"], c["d_head"], c["d_mlp"], c["vocab"], c["max_seq"])
    b = orc.segment_bounds(a)
    assert b[1][1] - b[1][0] == 57_872_640 == gen.CONFIGS[3]["n_elems"]
    assert orc.param_count(a) == 174_008_576
    c = gen.CONFIGS[1]
    a = orc.Arch(c["layers_per_level"], c["d_model"], c["n_heads"], c["d_head"], c["d_mlp"], c["vocab"], c["max_seq"])
    assert orc.param_count(a) == 136_960


# ---- router features --------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("a,B,S", [(TINY, 3, 5), (WIDE, 2, 8)])
def test_prefix_features_match_library_build(a, B, S):
    theta = gen.random_params(orc.param_count(a), seed=17, scale=0.3, dtype=np.float64)
    tok = gen.uniform_tokens((B, S), a.vocab, 18)
    lay = orc.param_layout(a)
    t = torch.tensor(theta, dtype=torch.float64)
    p = {n: t[o:o + int(np.prod(s))].reshape(s) for n, (o, s, _) in lay.items()}
    want = _torch_hidden(p, a, torch.as_tensor(tok, dtype=torch.long)).mean(dim=1).numpy()
    got = orc.prefix_features(theta, a, tok)
    assert got.shape == (B, a.d_model)
    assert np.abs(got - want).max() <= 1e-12


def test_prefix_features_closed_forms():
    # no blocks: the feature is the mean of token + position embeddings
    a0 = orc.Arch(layers_per_level=(0,), d_model=8, n_heads=2, d_head=4, d_mlp=16, vocab=11, max_seq=6)
    theta = gen.random_params(orc.param_count(a0), seed=19, scale=0.3, dtype=np.float64)
    lay = orc.param_layout(a0)
    tok = gen.uniform_tokens((2, 4), a0.vocab, 20)
    E, Ppos = orc.view(theta, lay, "tok_emb"), orc.view(theta, lay, "pos_emb")
    want = np.stack([(E[tok[b]] + Ppos[:4]).mean(axis=0) for b in range(2)])
    assert np.abs(orc.prefix_features(theta, a0, tok) - want).max() <= 1e-15
    # rows are independent and a one-token prefix is that token's own hidden state: the final LayerNorm of it,
    # times the head, gives the logits of path_logits
    theta = gen.random_params(orc.param_count(TINY), seed=21, scale=0.3, dtype=np.float64)
    tok = gen.uniform_tokens((3, 1), TINY.vocab, 22)
    f = orc.prefix_features(theta, TINY, tok)
    lay = orc.param_layout(TINY)
    y, _ = orc._layer_norm(f, orc.view(theta, lay, "lnf_g"), orc.view(theta, lay, "lnf_b"), TINY.ln_eps)
    logits = y @ orc.view(theta, lay, "w_head")
    assert np.abs(logits - orc.path_logits(theta, TINY, tok)[:, 0, :]).max() <= 1e-12
    assert np.array_equal(orc.prefix_features(theta, TINY, tok[[2, 0]]), f[[2, 0]])


# ---- path scores for discriminative routing ------------------------------------------------------------------------
def test_doc_scores_relation_to_loss_and_closed_form():
    a = WIDE
    theta = gen.random_params(orc.param_count(a), seed=23, scale=0.3, dtype=np.float64)
    tok, tgt = _data(a, 4, 7, seed=24, mask_prefix=2)
    sc = orc.path_doc_scores(theta, a, tok, tgt)
    n_t = int((tgt >= 0).sum())
    assert abs(-sc.sum() / n_t - orc.path_loss(theta, a, tok, tgt)) <= 1e-12       # the loss is their mean
    t = torch.tensor(theta, dtype=torch.float64)
    for b in range(4):                                                           # per document, from the torch build
        lb = _torch_loss(t, a, tok[b:b + 1], tgt[b:b + 1]).item() * int((tgt[b] >= 0).sum())
        assert abs(sc[b] + lb) <= 1e-10
    lay = orc.param_layout(a)
    off, shape, _ = lay["w_head"]
    flat = theta.copy()
    flat[off:off + int(np.prod(shape))] = 0.0                                    # zero head: uniform prediction
    sc0 = orc.path_doc_scores(flat, a, tok, tgt)
    assert np.allclose(sc0, -(tgt >= 0).sum(axis=1) * math.log(a.vocab), atol=1e-12)
    labels = orc.route_labels_from_scores(np.array([[1.0, 5.0, 2.0], [1.0, 4.0, 3.0]]))
    assert np.array_equal(labels, [0, 0, 1])                                     # ties to the first path
