"""CPU oracle for the DiPaCo path step, the per-module outer step and k-means prefix routing.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of what the GPU library has to
compute.  Only tests, the smoke check and the benchmark's `cpu_baseline` leg may import it; the product
path (the HIP library and its Python binding) never does, and shares no code with it.

Everything is numpy in float64.  Inputs may arrive as float32 and are widened on entry.  There is no
tiling, no online softmax, no expanded-square distance: each function is the definition written out, with
numpy's matmul / sum / argmin as library steps.

What each function follows (arXiv 2403.10616):
  * path_index / modules_of_path / paths_through_module ... Section 2.3 (Notation): a path is one module per
    level, the tuple (j_1..j_L) collapses to one number j in [0, prod K_l).
  * compose_path ............ Algorithm 1, worker start-of-round copy (theta_i^t = theta_i^{t-1}) and Section 2.6.
  * path_loss / path_loss_and_grad ... Algorithm 1 inner loop: L = f(x, theta_i) and its gradient, f being the
    usual next-token language-model loss of a decoder-only transformer (Section 4, hyper-parameter table).
  * adamw_step .............. Algorithm 1 inner loop, InnerOpt = AdamW (Sections 2.5, 2.6).
  * outer_step .............. Algorithm 1 outer loop (delta average, OuterOpt = Nesterov momentum), with the
    shard-size weights of Section 2.7 (loss re-weighing).
  * route_prefix ............ Section 2.4.1, eq. (1): r(z) = argmin_i ||z - c_i||^2.

Pins (tests/test_oracle_*.py, CPU only): central finite differences and an independent autograd build of
the same network for the gradient; loss = ln V with a zero head; causality; AdamW first-step closed form and
a hand-expanded two-step scalar case; outer step special cases (one path without momentum is SGD on the
delta, equal inputs, weight scaling, permutation, hand-expanded momentum recursion); brute-force argmin with
constructed ties.  The multi-step chain (inner steps followed by an outer step on a whole grid) has no
closed form: "parity unpinned" beyond its component pins.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple

import numpy as np
from scipy.special import erf

F64 = np.float64


# --------------------------------------------------------------------------------------------------
# Architecture and flat parameter layout
# --------------------------------------------------------------------------------------------------
@dataclass(frozen=True)
class Arch:
    """One path's architecture: pre-LN decoder-only transformer, learned positions, untied head.

    Sizes per Section 4 / hyper-parameter table of the paper; the choices the paper leaves open (biases on the
    linears, LayerNorm with gain and bias, exact-erf GELU, eps 1e-5) are fixed here.
    """
    layers_per_level: Tuple[int, ...]
    d_model: int
    n_heads: int
    d_head: int
    d_mlp: int
    vocab: int
    max_seq: int
    ln_eps: float = 1e-5

    @property
    def n_levels(self) -> int:
        return len(self.layers_per_level)

    @property
    def n_layers(self) -> int:
        return int(sum(self.layers_per_level))

    @property
    def d_attn(self) -> int:
        return self.n_heads * self.d_head


def block_tensors(a: Arch) -> List[Tuple[str, Tuple[int, ...], bool]]:
    """(name, shape, weight-decayed?) of one decoder block, in storage order."""
    d, A, F = a.d_model, a.d_attn, a.d_mlp
    return [
        ("ln1_g", (d,), False), ("ln1_b", (d,), False),
        ("w_qkv", (d, 3 * A), True), ("b_qkv", (3 * A,), False),
        ("w_o", (A, d), True), ("b_o", (d,), False),
        ("ln2_g", (d,), False), ("ln2_b", (d,), False),
        ("w_up", (d, F), True), ("b_up", (F,), False),
        ("w_down", (F, d), True), ("b_down", (d,), False),
    ]


def param_layout(a: Arch) -> Dict[str, Tuple[int, Tuple[int, ...], bool]]:
    """name -> (offset in elements, shape, decayed?) for the flat path buffer.

    Order: stem (token embedding, positions) | level-1 blocks | ... | level-L blocks | head (final LN, W_head).
    Matrices are row-major [in, out]: y = x @ W.
    """
    out: Dict[str, Tuple[int, Tuple[int, ...], bool]] = {}
    off = 0

    def put(name, shape, decay):
        nonlocal off
        out[name] = (off, tuple(shape), decay)
        off += int(np.prod(shape))

    put("tok_emb", (a.vocab, a.d_model), True)
    put("pos_emb", (a.max_seq, a.d_model), True)
    for layer in range(a.n_layers):
        for name, shape, decay in block_tensors(a):
            put(f"blk{layer}.{name}", shape, decay)
    put("lnf_g", (a.d_model,), False)
    put("lnf_b", (a.d_model,), False)
    put("w_head", (a.d_model, a.vocab), True)
    return out


def param_count(a: Arch) -> int:
    lay = param_layout(a)
    last = max(lay.values(), key=lambda v: v[0])
    return last[0] + int(np.prod(last[1]))


def segment_bounds(a: Arch) -> List[Tuple[int, int]]:
    """[start, end) element ranges of the L+2 segments: stem, level 1..L, head."""
    lay = param_layout(a)
    bounds = []
    stem_end = lay["blk0.ln1_g"][0] if a.n_layers else lay["lnf_g"][0]
    bounds.append((0, stem_end))
    per_block = sum(int(np.prod(s)) for _, s, _ in block_tensors(a))
    pos = stem_end
    for n in a.layers_per_level:
        bounds.append((pos, pos + n * per_block))
        pos += n * per_block
    bounds.append((pos, param_count(a)))
    return bounds


def decay_mask(a: Arch) -> np.ndarray:
    """1.0 where AdamW applies weight decay (matrices and embeddings), 0.0 on biases and LayerNorm."""
    mask = np.zeros(param_count(a), dtype=F64)
    for off, shape, decay in param_layout(a).values():
        if decay:
            mask[off:off + int(np.prod(shape))] = 1.0
    return mask


def view(flat: np.ndarray, lay, name: str) -> np.ndarray:
    off, shape, _ = lay[name]
    return flat[off:off + int(np.prod(shape))].reshape(shape)


# --------------------------------------------------------------------------------------------------
# Paths and modules (Section 2.3)
# --------------------------------------------------------------------------------------------------
def path_index(modules: Sequence[int], K: Sequence[int]) -> int:
    """Collapse (j_1..j_L) into j, 0-based, level 1 most significant (row-major)."""
    j = 0
    for jl, kl in zip(modules, K):
        assert 0 <= jl < kl
        j = j * kl + jl
    return j


def modules_of_path(j: int, K: Sequence[int]) -> Tuple[int, ...]:
    """Inverse of path_index."""
    digits = []
    for kl in reversed(K):
        digits.append(j % kl)
        j //= kl
    assert j == 0
    return tuple(reversed(digits))


def paths_through_module(level: int, e: int, K: Sequence[int]) -> List[int]:
    """All paths whose module at `level` (0-based) is e.  Their number is P_{l,e} = P / K_l (Algorithm 1)."""
    P = int(np.prod(K))
    return [j for j in range(P) if modules_of_path(j, K)[level] == e]


def compose_path(segments: Sequence[np.ndarray]) -> np.ndarray:
    """Local copy of a path's parameters: stem, the chosen module of each level, head, concatenated."""
    return np.concatenate([np.asarray(s, dtype=F64).ravel() for s in segments])


# --------------------------------------------------------------------------------------------------
# Transformer pieces
# --------------------------------------------------------------------------------------------------
def _layer_norm(x, g, b, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)        # biased variance, eps inside the root
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return xhat * g + b, (xhat, rstd)


def _layer_norm_bwd(dy, g, cache):
    xhat, rstd = cache
    dg = (dy * xhat).sum(axis=0)
    db = dy.sum(axis=0)
    dxhat = dy * g
    dx = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True)
                 - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return dx, dg, db


def _gelu(u):
    return 0.5 * u * (1.0 + erf(u / math.sqrt(2.0)))


def _gelu_grad(u):
    cdf = 0.5 * (1.0 + erf(u / math.sqrt(2.0)))
    pdf = np.exp(-0.5 * u * u) / math.sqrt(2.0 * math.pi)
    return cdf + u * pdf


def _attention(q, k, v, a: Arch):
    """Causal softmax attention for one sequence.  q,k,v: [S, H*dh].  Returns o [S, H*dh] and the probabilities."""
    S = q.shape[0]
    H, dh = a.n_heads, a.d_head
    o = np.empty_like(q)
    probs = np.empty((H, S, S), dtype=F64)
    allowed = np.tril(np.ones((S, S), dtype=bool))
    for h in range(H):
        sl = slice(h * dh, (h + 1) * dh)
        s = (q[:, sl] @ k[:, sl].T) / math.sqrt(dh)
        s = np.where(allowed, s, -np.inf)
        s = s - s.max(axis=-1, keepdims=True)
        e = np.exp(s)
        p = e / e.sum(axis=-1, keepdims=True)
        probs[h] = p
        o[:, sl] = p @ v[:, sl]
    return o, probs


def _attention_bwd(do, q, k, v, probs, a: Arch):
    H, dh = a.n_heads, a.d_head
    dq = np.empty_like(q)
    dk = np.empty_like(k)
    dv = np.empty_like(v)
    for h in range(H):
        sl = slice(h * dh, (h + 1) * dh)
        p = probs[h]
        dv[:, sl] = p.T @ do[:, sl]
        dp = do[:, sl] @ v[:, sl].T
        ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
        ds = ds / math.sqrt(dh)
        dq[:, sl] = ds @ k[:, sl]
        dk[:, sl] = ds.T @ q[:, sl]
    return dq, dk, dv


def _forward_sequence(P, lay, a: Arch, tok: np.ndarray):
    """Forward of one sequence up to the logits.  Returns logits [S, V] and what backward needs."""
    S = tok.shape[0]
    A = a.d_attn
    x = view(P, lay, "tok_emb")[tok] + view(P, lay, "pos_emb")[:S]
    caches = []
    for layer in range(a.n_layers):
        w = lambda n: view(P, lay, f"blk{layer}.{n}")
        x_in = x
        h1, ln1 = _layer_norm(x_in, w("ln1_g"), w("ln1_b"), a.ln_eps)
        qkv = h1 @ w("w_qkv") + w("b_qkv")
        q, k, v = qkv[:, :A], qkv[:, A:2 * A], qkv[:, 2 * A:]
        o, probs = _attention(q, k, v, a)
        x_mid = x_in + o @ w("w_o") + w("b_o")
        h2, ln2 = _layer_norm(x_mid, w("ln2_g"), w("ln2_b"), a.ln_eps)
        u = h2 @ w("w_up") + w("b_up")
        act = _gelu(u)
        x = x_mid + act @ w("w_down") + w("b_down")
        caches.append(dict(h1=h1, ln1=ln1, q=q, k=k, v=v, o=o, probs=probs, h2=h2, ln2=ln2, u=u, act=act))
    y, lnf = _layer_norm(x, view(P, lay, "lnf_g"), view(P, lay, "lnf_b"), a.ln_eps)
    logits = y @ view(P, lay, "w_head")
    return logits, dict(blocks=caches, y=y, lnf=lnf)


def _token_nll(logits: np.ndarray, targets: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Per-position negative log-likelihood (0 where target < 0) and the softmax, natural log."""
    z = logits - logits.max(axis=-1, keepdims=True)
    e = np.exp(z)
    denom = e.sum(axis=-1, keepdims=True)
    soft = e / denom
    lse = np.log(denom[:, 0])
    keep = targets >= 0
    safe = np.where(keep, targets, 0)
    nll = np.where(keep, lse - z[np.arange(z.shape[0]), safe], 0.0)
    return nll, soft


def path_logits(params, a: Arch, tokens) -> np.ndarray:
    """Logits [B, S, V] (small inputs only)."""
    P = np.asarray(params, dtype=F64)
    lay = param_layout(a)
    tokens = np.asarray(tokens)
    return np.stack([_forward_sequence(P, lay, a, tokens[b])[0] for b in range(tokens.shape[0])])


def path_token_nll(params, a: Arch, tokens, targets) -> np.ndarray:
    """Per-position NLL [B, S]; ignored positions (target < 0) hold 0."""
    P = np.asarray(params, dtype=F64)
    lay = param_layout(a)
    tokens = np.asarray(tokens)
    targets = np.asarray(targets)
    out = np.zeros(tokens.shape, dtype=F64)
    for b in range(tokens.shape[0]):
        logits, _ = _forward_sequence(P, lay, a, tokens[b])
        out[b], _ = _token_nll(logits, targets[b])
    return out


def path_loss(params, a: Arch, tokens, targets) -> float:
    """L = f(x, theta_i): mean next-token NLL over the positions whose target is >= 0."""
    n_t = int((np.asarray(targets) >= 0).sum())
    return float(path_token_nll(params, a, tokens, targets).sum() / n_t)


def path_loss_and_grad(params, a: Arch, tokens, targets) -> Tuple[float, np.ndarray]:
    """Loss and its gradient with respect to every parameter, flat, in the parameter layout."""
    P = np.asarray(params, dtype=F64)
    lay = param_layout(a)
    tokens = np.asarray(tokens)
    targets = np.asarray(targets)
    B, S = tokens.shape
    A = a.d_attn
    n_t = int((targets >= 0).sum())
    G = np.zeros_like(P)
    g = lambda name: view(G, lay, name)
    total = 0.0
    for b in range(B):
        tok, tgt = tokens[b], targets[b]
        logits, cache = _forward_sequence(P, lay, a, tok)
        nll, soft = _token_nll(logits, tgt)
        total += nll.sum()
        keep = tgt >= 0
        dlogits = soft.copy()
        dlogits[np.arange(S)[keep], tgt[keep]] -= 1.0
        dlogits[~keep] = 0.0
        dlogits /= n_t
        g("w_head")[...] += cache["y"].T @ dlogits
        dy = dlogits @ view(P, lay, "w_head").T
        dx, dg, db = _layer_norm_bwd(dy, view(P, lay, "lnf_g"), cache["lnf"])
        g("lnf_g")[...] += dg
        g("lnf_b")[...] += db
        for layer in reversed(range(a.n_layers)):
            w = lambda n: view(P, lay, f"blk{layer}.{n}")
            gw = lambda n: view(G, lay, f"blk{layer}.{n}")
            c = cache["blocks"][layer]
            # x = x_mid + gelu(u) @ w_down + b_down
            gw("w_down")[...] += c["act"].T @ dx
            gw("b_down")[...] += dx.sum(axis=0)
            du = (dx @ w("w_down").T) * _gelu_grad(c["u"])
            gw("w_up")[...] += c["h2"].T @ du
            gw("b_up")[...] += du.sum(axis=0)
            dmid, dg, db = _layer_norm_bwd(du @ w("w_up").T, w("ln2_g"), c["ln2"])
            gw("ln2_g")[...] += dg
            gw("ln2_b")[...] += db
            dmid = dmid + dx
            # x_mid = x_in + o @ w_o + b_o
            gw("w_o")[...] += c["o"].T @ dmid
            gw("b_o")[...] += dmid.sum(axis=0)
            do = dmid @ w("w_o").T
            dq, dk, dv = _attention_bwd(do, c["q"], c["k"], c["v"], c["probs"], a)
            dqkv = np.concatenate([dq, dk, dv], axis=1)
            gw("w_qkv")[...] += c["h1"].T @ dqkv
            gw("b_qkv")[...] += dqkv.sum(axis=0)
            din, dg, db = _layer_norm_bwd(dqkv @ w("w_qkv").T, w("ln1_g"), c["ln1"])
            gw("ln1_g")[...] += dg
            gw("ln1_b")[...] += db
            dx = din + dmid
        np.add.at(g("tok_emb"), tok, dx)
        g("pos_emb")[:S] += dx
    return float(total / n_t), G


# --------------------------------------------------------------------------------------------------
# Inner optimiser: AdamW
# --------------------------------------------------------------------------------------------------
def adamw_step(theta, grad, m, v, step: int, lr: float, beta1: float, beta2: float, eps: float,
               weight_decay: float, mask):
    """One AdamW update; `step` counts from 1.  Returns new (theta, m, v).

    m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;  mhat = m/(1-b1^t);  vhat = v/(1-b2^t);
    theta <- theta - lr * ( mhat / (sqrt(vhat) + eps) + wd * mask * theta ).
    """
    theta = np.asarray(theta, dtype=F64)
    grad = np.asarray(grad, dtype=F64)
    m = beta1 * np.asarray(m, dtype=F64) + (1.0 - beta1) * grad
    v = beta2 * np.asarray(v, dtype=F64) + (1.0 - beta2) * grad * grad
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    theta = theta - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * np.asarray(mask, dtype=F64) * theta)
    return theta, m, v


# --------------------------------------------------------------------------------------------------
# Outer optimiser: weighted delta average + Nesterov momentum
# --------------------------------------------------------------------------------------------------
def outer_step(theta_prev, momentum, inputs: Sequence[np.ndarray], weights, is_delta: bool,
               outer_lr: float, outer_momentum: float):
    """One module's outer update.  Returns new (theta, momentum).

    Delta = sum_i alpha_i (theta_prev - theta_i), alpha_i = w_i / sum w (uniform weights give the plain mean of
    Algorithm 1; unequal ones are the shard-size weights of Section 2.7, normalised over the paths that share
    the module).  `inputs` are the paths' local copies theta_i, or ready-made deltas when is_delta.
    Nesterov: buf <- mu*buf + Delta;  theta <- theta_prev - lr * (Delta + mu*buf).
    """
    theta_prev = np.asarray(theta_prev, dtype=F64)
    buf = np.asarray(momentum, dtype=F64)
    n = len(inputs)
    w = np.ones(n, dtype=F64) if weights is None else np.asarray(weights, dtype=F64)
    alpha = w / w.sum()
    delta = np.zeros_like(theta_prev)
    for i in range(n):
        x = np.asarray(inputs[i], dtype=F64)
        delta += alpha[i] * (x if is_delta else (theta_prev - x))
    buf = outer_momentum * buf + delta
    theta = theta_prev - outer_lr * (delta + outer_momentum * buf)
    return theta, buf


# --------------------------------------------------------------------------------------------------
# Routing: k-means assignment
# --------------------------------------------------------------------------------------------------
def route_prefix(z, centroids):
    """idx[n] = argmin_k ||z_n - c_k||^2 (lowest k on ties), hist[k] = #{n : idx[n] = k},
    margin[n] = second-smallest minus smallest squared distance (inf when K = 1)."""
    z = np.asarray(z, dtype=F64)
    c = np.asarray(centroids, dtype=F64)
    N, K = z.shape[0], c.shape[0]
    idx = np.empty(N, dtype=np.int32)
    margin = np.empty(N, dtype=F64)
    for n in range(N):
        diff = z[n][None, :] - c
        d = (diff * diff).sum(axis=1)
        k = int(np.argmin(d))                     # numpy returns the first minimiser
        idx[n] = k
        if K > 1:
            rest = np.delete(d, k)
            margin[n] = rest.min() - d[k]
        else:
            margin[n] = np.inf
    hist = np.bincount(idx, minlength=K).astype(np.int64)
    return idx, hist, margin


def route_prefix_top2(z, centroids):
    """The two closest centroids of every row (overlapping shards of Section 2.4.4, where a document joins the
    shards of its two best routing choices).

    idx2[n] = (closest, second closest) under the order (squared distance, index): exact ties go to the lower
    index; the second entry is -1 when there is only one centroid.  hist[k] = number of rows that have k as either
    choice (the sizes of the overlapping shards)."""
    z = np.asarray(z, dtype=F64)
    c = np.asarray(centroids, dtype=F64)
    N, K = z.shape[0], c.shape[0]
    idx2 = np.full((N, 2), -1, dtype=np.int32)
    for n in range(N):
        diff = z[n][None, :] - c
        d = (diff * diff).sum(axis=1)
        first = int(np.argmin(d))                 # the first minimiser
        idx2[n, 0] = first
        if K > 1:
            d2 = d.copy()
            d2[first] = np.inf
            idx2[n, 1] = int(np.argmin(d2))       # the first minimiser among the others
    hist = np.bincount(idx2[idx2 >= 0], minlength=K).astype(np.int64)
    return idx2, hist


def kmeans_update(z, idx, centroids_prev):
    """The update half of a k-means (Lloyd) iteration (Section 2.4.1 fits the prototypes c_1..c_k by k-means):
    every centroid becomes the mean of the rows assigned to it; one without rows keeps its value.
    Returns (centroids, counts)."""
    z = np.asarray(z, dtype=F64)
    idx = np.asarray(idx)
    c = np.array(centroids_prev, dtype=F64, copy=True)
    K = c.shape[0]
    counts = np.zeros(K, dtype=np.int64)
    for k in range(K):
        rows = z[idx == k]
        counts[k] = rows.shape[0]
        if rows.shape[0] > 0:
            c[k] = rows.sum(axis=0) / rows.shape[0]
    return c, counts


def kmeans_objective(z, idx, centroids):
    """sum_n ||z_n - c_idx[n]||^2: what both halves of a Lloyd iteration can only lower."""
    z = np.asarray(z, dtype=F64)
    c = np.asarray(centroids, dtype=F64)
    diff = z - c[np.asarray(idx)]
    return float((diff * diff).sum())


def outer_step_streaming(theta_prev, momentum, inputs: Sequence[np.ndarray], weights, is_delta: bool,
                         outer_lr: float, outer_momentum: float, norm_scale: float = 1.0):
    """The outer update with the paths' results added one at a time, in arrival order, to a running weighted sum
    (Section 3.3, online parameter gradient averaging), and the optional rescaling of the averaged outer gradient
    (Section 2.7, outer gradient norm rescaling):
    Delta = norm_scale * (sum_i w_i d_i) / (sum_i w_i), d_i = theta_prev - theta_i (or the ready-made delta);
    then Nesterov as in outer_step.  norm_scale = sqrt(P_le) is the paper's rescaling read as a multiplication."""
    theta_prev = np.asarray(theta_prev, dtype=F64)
    buf = np.asarray(momentum, dtype=F64)
    n = len(inputs)
    w = np.ones(n, dtype=F64) if weights is None else np.asarray(weights, dtype=F64)
    acc = np.zeros_like(theta_prev)
    wsum = 0.0
    for i in range(n):
        x = np.asarray(inputs[i], dtype=F64)
        acc = acc + w[i] * (x if is_delta else (theta_prev - x))
        wsum += w[i]
    delta = norm_scale * acc / wsum
    buf = outer_momentum * buf + delta
    theta = theta_prev - outer_lr * (delta + outer_momentum * buf)
    return theta, buf


def window_targets(token_scores, window: int) -> np.ndarray:
    """Labels for the token-level router (appendix, more frequent routing during evaluation):
    T[i, j] = argmax_p sum_{j' = j}^{min(len, j + L - 1)} S[i, j', p], lowest p on ties.
    token_scores: S as an array [P, n_docs, len] of per-token log-likelihoods."""
    S = np.asarray(token_scores, dtype=F64)
    P, n, length = S.shape
    T = np.empty((n, length), dtype=np.int32)
    for i in range(n):
        for j in range(length):
            hi = min(length, j + window)
            sums = [S[p, i, j:hi].sum() for p in range(P)]
            T[i, j] = int(np.argmax(sums))
    return T


def chunk_routed_scores(token_scores, chunk_path, chunk: int) -> np.ndarray:
    """Section 2.4.3: a document is cut into chunks of W consecutive tokens and chunk c is scored by the path
    chunk_path[i, c] (each path sees the whole preceding text).  Returns the documents' log-likelihoods."""
    S = np.asarray(token_scores, dtype=F64)
    _P, n, length = S.shape
    out = np.zeros(n, dtype=F64)
    for i in range(n):
        for c, lo in enumerate(range(0, length, chunk)):
            out[i] += S[chunk_path[i][c], i, lo:min(length, lo + chunk)].sum()
    return out


def route_linear(z, weights, bias):
    """The trained discriminative router used as r(z) (Section 2.4.2): idx[n] = argmax_k (w_k . z_n + b_k), lowest k
    on ties; hist[k] = #{n : idx[n] = k}; margin[n] = largest minus second-largest logit (inf when K = 1)."""
    z = np.asarray(z, dtype=F64)
    W = np.asarray(weights, dtype=F64)
    b = np.asarray(bias, dtype=F64)
    N, K = z.shape[0], W.shape[0]
    idx = np.empty(N, dtype=np.int32)
    margin = np.empty(N, dtype=F64)
    for n in range(N):
        logit = W @ z[n] + b
        k = int(np.argmax(logit))                   # numpy returns the first maximiser
        idx[n] = k
        margin[n] = logit[k] - np.delete(logit, k).max() if K > 1 else np.inf
    return idx, np.bincount(idx, minlength=K).astype(np.int64), margin


def logistic_loss_grad(z, labels, weights, bias):
    """K-class linear logistic classifier on router features (appendix on routing: target argmax_p sum_j S_ijp,
    feature g(document)): mean cross-entropy over the N documents and its gradients.
        p_n = softmax(W z_n + b);  loss = -(1/N) sum_n log p_n[y_n]
        dW = (1/N) sum_n (p_n - e_{y_n}) z_n^T;  db = (1/N) sum_n (p_n - e_{y_n})
    A label outside [0, K) drops its document (the mean stays over N).  Returns (loss, dW [K, D], db [K])."""
    z = np.asarray(z, dtype=F64)
    W = np.asarray(weights, dtype=F64)
    b = np.asarray(bias, dtype=F64)
    y = np.asarray(labels)
    N, K = z.shape[0], W.shape[0]
    loss = 0.0
    dW = np.zeros_like(W)
    db = np.zeros_like(b)
    for n in range(N):
        if y[n] < 0 or y[n] >= K:
            continue
        logit = W @ z[n] + b
        m = logit.max()
        lse = m + np.log(np.exp(logit - m).sum())
        p = np.exp(logit - lse)
        loss -= (logit[y[n]] - lse)
        p[y[n]] -= 1.0
        dW += np.outer(p, z[n])
        db += p
    return loss / N, dW / N, db / N


def outer_step_modules(modules, outer_lr: float, outer_momentum: float):
    """Outer update of every module of a grid (Algorithm 1: the loop over levels and experts; Section 2.6: a
    path-specific module has a single path and is updated by the same rule).  `modules` is a sequence of dicts with
    theta, momentum, inputs, weights (or None), is_delta and optionally norm_scale (Section 2.7, read as a
    multiplication of the averaged Delta).  Returns a list of (theta, momentum), one per module; modules do not
    interact."""
    out = []
    for m in modules:
        theta_prev = np.asarray(m["theta"], dtype=F64)
        buf = np.asarray(m["momentum"], dtype=F64)
        n = len(m["inputs"])
        w = np.ones(n, dtype=F64) if m.get("weights") is None else np.asarray(m["weights"], dtype=F64)
        delta = np.zeros_like(theta_prev)
        for i in range(n):
            x = np.asarray(m["inputs"][i], dtype=F64)
            delta += (w[i] / w.sum()) * (x if m["is_delta"] else (theta_prev - x))
        delta = float(m.get("norm_scale", 1.0)) * delta
        buf = outer_momentum * buf + delta
        out.append((theta_prev - outer_lr * (delta + outer_momentum * buf), buf))
    return out


def prefix_features(params, a: Arch, tokens) -> np.ndarray:
    """Router features (appendix on routing): for every row of tokens [B, S] (S = 32 in the paper), the mean over
    the S positions of the hidden state that leaves the last transformer block.  Read as the residual stream after
    the last block, before the final LayerNorm.  Returns [B, d_model]."""
    P = np.asarray(params, dtype=F64)
    lay = param_layout(a)
    tokens = np.asarray(tokens)
    A = a.d_attn
    out = np.empty((tokens.shape[0], a.d_model), dtype=F64)
    for b in range(tokens.shape[0]):
        tok = tokens[b]
        S = tok.shape[0]
        x = view(P, lay, "tok_emb")[tok] + view(P, lay, "pos_emb")[:S]
        for layer in range(a.n_layers):
            w = lambda n: view(P, lay, f"blk{layer}.{n}")
            h1, _ = _layer_norm(x, w("ln1_g"), w("ln1_b"), a.ln_eps)
            qkv = h1 @ w("w_qkv") + w("b_qkv")
            o, _ = _attention(qkv[:, :A], qkv[:, A:2 * A], qkv[:, 2 * A:], a)
            x = x + o @ w("w_o") + w("b_o")
            h2, _ = _layer_norm(x, w("ln2_g"), w("ln2_b"), a.ln_eps)
            x = x + _gelu(h2 @ w("w_up") + w("b_up")) @ w("w_down") + w("b_down")
        out[b] = x.sum(axis=0) / S
    return out


def path_doc_scores(params, a: Arch, tokens, targets) -> np.ndarray:
    """Scores for discriminative routing (appendix on routing): for every document (row), the summed
    auto-regressive log-likelihood sum_j log p(t_j | t_<j) under this path, over positions with target >= 0."""
    return -path_token_nll(params, a, tokens, targets).sum(axis=1)


def route_labels_from_scores(scores) -> np.ndarray:
    """Router training labels: argmax over paths of the documents' scores; scores [n_paths, n_docs]; the first
    path wins exact ties."""
    return np.argmax(np.asarray(scores, dtype=F64), axis=0).astype(np.int32)
