"""Writes the stored oracle results that the full-size GPU tests compare against (tests/golden/config*_oracle.npz).

Everything stored here is computed by `oracle/dipaco_oracle.py` alone on inputs drawn by `dipaco_inputs.py`; nothing
comes from the GPU library.  The oracle needs minutes (config 2, config 4) to about an hour (config 5) for these sizes,
which is why its results are kept instead of being recomputed inside the tests.  Each file carries a SHA-256 of the
inputs it was computed from, so that a test can tell when the input recipe has changed under it.

    python tests/golden/make_golden.py 2      # one path step at batch 32 x seq 1024 (Algorithm 1, inner loop)
    python tests/golden/make_golden.py 4      # eq. (1) on all 2^20 prefix embeddings
    python tests/golden/make_golden.py 5      # eight inner steps at batch 16 x seq 2048 (Algorithm 1, inner loop)

What is kept for a flat parameter-sized vector (a gradient, the parameters after AdamW): per tensor, its L2 norm and
the values at up to SAMPLES_PER_TENSOR seeded offsets (every element of the small tensors).
"""
from __future__ import annotations

import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import dipaco_inputs as gen                      # noqa: E402
from oracle import dipaco_oracle as orc          # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))
SAMPLES_PER_TENSOR = 1024
NEAR_TIE = 1e-3


def say(msg):
    print(time.strftime("%H:%M:%S"), msg, flush=True)


input_hash = gen.input_hash


def arch_of(cfg) -> orc.Arch:
    return orc.Arch(tuple(cfg["layers_per_level"]), cfg["d_model"], cfg["n_heads"], cfg["d_head"], cfg["d_mlp"],
                    cfg["vocab"], cfg["max_seq"])


def tensor_samples(lay, seed: int):
    """(names, start of each tensor's run in the sample arrays, flat offsets into the parameter vector)."""
    names = sorted(lay, key=lambda n: lay[n][0])
    starts, flat = [0], []
    for t, name in enumerate(names):
        off, shape, _ = lay[name]
        local = gen.sample_offsets(int(np.prod(shape)), SAMPLES_PER_TENSOR, seed, "golden:" + name)
        flat.append(off + local)
        starts.append(starts[-1] + len(local))
    return names, np.asarray(starts, dtype=np.int64), np.concatenate(flat)


def tensor_norms(lay, names, vec):
    return np.asarray([np.linalg.norm(vec[lay[n][0]:lay[n][0] + int(np.prod(lay[n][1]))]) for n in names])


def config2():
    cfg = gen.CONFIGS[2]
    a = arch_of(cfg)
    lay = orc.param_layout(a)
    B, S = cfg["batch"], cfg["seq"]
    theta = gen.round_to_bf16(gen.init_params(lay, a.n_layers, cfg["seed"]))
    tok, tgt = gen.split_inputs_targets(gen.zipf_tokens((B, S + 1), cfg["vocab"], cfg["zipf_s"], cfg["seed"]))
    names, starts, flat = tensor_samples(lay, cfg["seed"])
    say("config 2: per-token NLL of the 32 sequences")
    nll = orc.path_token_nll(theta, a, tok, tgt)
    say("config 2: loss and gradient of the batch")
    loss, grad = orc.path_loss_and_grad(theta, a, tok, tgt)
    say(f"config 2: loss {loss:.9f}; AdamW step 1")
    th1, m1, v1 = orc.adamw_step(theta, grad, 0.0, 0.0, 1, cfg["lr"], cfg["beta1"], cfg["beta2"], cfg["eps"],
                                 cfg["wd"], orc.decay_mask(a))
    np.savez_compressed(
        os.path.join(HERE, "config2_oracle.npz"),
        input_sha256=np.asarray(input_hash(theta, tok, tgt)), loss=np.float64(loss), token_nll=nll.astype(np.float32),
        tensor_names=np.asarray(names), sample_starts=starts, sample_offsets=flat,
        grad_samples=grad[flat], grad_norms=tensor_norms(lay, names, grad),
        theta1_samples=th1[flat], update1_norms=tensor_norms(lay, names, th1 - theta))
    say("config 2: written")


def config5():
    cfg = gen.CONFIGS[5]
    a = arch_of(cfg)
    lay = orc.param_layout(a)
    B, S, steps = cfg["batch"], cfg["seq"], cfg["inner_steps"]
    theta0 = gen.round_to_bf16(gen.init_params(lay, a.n_layers, cfg["seed"]))
    seqs = gen.zipf_tokens((steps, B, S + 1), cfg["vocab"], cfg["zipf_s"], cfg["seed"])
    names, starts, flat = tensor_samples(lay, cfg["seed"])
    mask = orc.decay_mask(a)
    theta = theta0.astype(np.float64)
    m = v = 0.0
    keep = dict(input_sha256=np.asarray(input_hash(theta0, seqs)), tensor_names=np.asarray(names), sample_starts=starts,
                sample_offsets=flat)
    losses = []
    for t in range(steps):
        tok, tgt = gen.split_inputs_targets(seqs[t])
        if t == 0:
            say("config 5: per-token NLL of the first batch")
            keep["token_nll_step1"] = orc.path_token_nll(theta, a, tok, tgt).astype(np.float32)
        say(f"config 5: inner step {t + 1}: loss and gradient")
        loss, grad = orc.path_loss_and_grad(theta, a, tok, tgt)
        losses.append(loss)
        if t == 0:
            keep["grad1_samples"] = grad[flat]
            keep["grad1_norms"] = tensor_norms(lay, names, grad)
        theta, m, v = orc.adamw_step(theta, grad, m, v, t + 1, cfg["lr"], cfg["beta1"], cfg["beta2"], cfg["eps"],
                                     cfg["wd"], mask)
        say(f"config 5: inner step {t + 1}: loss {loss:.9f}")
        keep["losses"] = np.asarray(losses)
        keep[f"theta_samples_after_step{t + 1}"] = theta[flat]
        keep[f"update_norms_after_step{t + 1}"] = tensor_norms(lay, names, theta - theta0)
        np.savez_compressed(os.path.join(HERE, "config5_oracle.npz"), steps_done=np.int64(t + 1), **keep)
    say("config 5: written")


def config4():
    cfg = gen.CONFIGS[4]
    N, D, K = cfg["N"], cfg["D"], cfg["K"]
    say("config 4: drawing the mixture")
    z, c, _ = gen.gaussian_mixture(N, D, K, cfg["noise_std"], cfg["seed"])
    say("config 4: eq. (1) on every point")
    idx, hist, margin = orc.route_prefix(z, c)
    near = np.nonzero(margin <= NEAR_TIE)[0]
    say(f"config 4: {len(near)} points with margin <= {NEAR_TIE}; their two closest centroids")
    top2, _ = orc.route_prefix_top2(z[near], c)
    assert np.array_equal(top2[:, 0], idx[near])
    np.savez_compressed(
        os.path.join(HERE, "config4_oracle.npz"),
        input_sha256=np.asarray(input_hash(z[:: 4096], c)), idx=idx.astype(np.uint8), hist=hist,
        near_tie_bound=np.float64(NEAR_TIE), near_n=near.astype(np.int64), near_margin=margin[near],
        near_top2=top2.astype(np.int32), margin_head=margin[:65536].astype(np.float32))
    say("config 4: written")


if __name__ == "__main__":
    which = sys.argv[1:] or ["2", "4", "5"]
    for w in which:
        {"2": config2, "4": config4, "5": config5}[w]()
