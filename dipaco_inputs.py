"""Seeded synthetic inputs for the DiPaCo path-step library: the only module both the CPU oracle's tests and
the GPU tests / benchmark draw from.  It holds no arithmetic of the method itself: only random draws of
parameters, token ids, perturbations, shard weights and prefix embeddings, with the shapes and value
distributions of the paper's workloads (32k vocabulary, 1024 / 2048-token sequences, 150M-class path, 16x16
grid) standing in for its text corpus and pretrained weights, which are not available here.

All draws use numpy's `default_rng(seed)` (or a (seed, stream) pair), generated once on the host.
"""
from __future__ import annotations

import hashlib
import zlib
from typing import Dict, Sequence, Tuple

import numpy as np

# The five benchmark configurations (sizes only; nothing here computes with them).
CONFIGS = {
    # tiny 2x2 grid, fp32
    1: dict(layers_per_level=(1, 1), K=(2, 2), d_model=64, n_heads=2, d_head=32, d_mlp=256, vocab=256, max_seq=64,
            batch=4, seq=64, inner_steps=2, lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, wd=0.1,
            outer_lr=0.7, outer_momentum=0.9, seed=0),
    # ~150M-class path step, bf16
    2: dict(layers_per_level=(6, 6), K=(16, 16), d_model=896, n_heads=14, d_head=64, d_mlp=3584, vocab=32000,
            max_seq=1024, batch=32, seq=1024, inner_steps=1, lr=4e-4, beta1=0.9, beta2=0.95, eps=1e-8, wd=0.1,
            zipf_s=1.1, seed=1),
    # outer step of one level-1 module
    3: dict(n_elems=57_872_640, n_paths=16, delta_std=1e-3, outer_lr=0.7, outer_momentum=0.9, seed=3),
    # prefix routing
    4: dict(N=1 << 20, D=768, K=256, noise_std=0.3, seed=4),
    # full round on one path, bf16
    5: dict(layers_per_level=(6, 6), K=(16, 16), d_model=896, n_heads=14, d_head=64, d_mlp=3584, vocab=32000,
            max_seq=2048, batch=16, seq=2048, inner_steps=8, lr=4e-4, beta1=0.9, beta2=0.95, eps=1e-8, wd=0.1,
            zipf_s=1.1, n_partners=15, delta_std=1e-3, outer_lr=0.7, outer_momentum=0.9, seed=2),
}


def _rng(seed: int, stream: str = "") -> np.random.Generator:
    return np.random.default_rng([int(seed), zlib.crc32(stream.encode())])


def init_params(layout: Dict[str, Tuple[int, Tuple[int, ...], bool]], n_layers: int, seed: int,
                dtype=np.float32) -> np.ndarray:
    """Flat parameter vector for a path.  `layout` maps tensor name -> (offset, shape, decayed?).

    Matrices and embeddings ~ N(0, 0.02); the two residual-writing matrices (w_o, w_down) are scaled by
    1/sqrt(2*n_layers); biases 0; LayerNorm gains 1.  (The paper starts from a pretrained model instead.)
    """
    total = max(off + int(np.prod(shape)) for off, shape, _ in layout.values())
    flat = np.zeros(total, dtype=dtype)
    rng = _rng(seed, "params")
    for name in sorted(layout, key=lambda n: layout[n][0]):
        off, shape, _ = layout[name]
        n = int(np.prod(shape))
        leaf = name.split(".")[-1]
        if len(shape) == 2:
            w = rng.standard_normal(n, dtype=np.float32) * np.float32(0.02)
            if leaf in ("w_o", "w_down"):
                w = w / np.float32(np.sqrt(2.0 * max(n_layers, 1)))
            flat[off:off + n] = w
        elif leaf.endswith("_g"):
            flat[off:off + n] = 1.0
    return flat


def random_params(total: int, seed: int, scale: float = 0.1, dtype=np.float32) -> np.ndarray:
    """Every entry ~ N(0, scale): no zeros and no ones, so that a mistake in any gain, bias or weight shows."""
    return (_rng(seed, "random_params").standard_normal(total) * scale).astype(dtype)


def uniform_tokens(shape: Sequence[int], vocab: int, seed: int, stream: str = "tokens") -> np.ndarray:
    return _rng(seed, stream).integers(0, vocab, size=tuple(shape)).astype(np.int32)


def zipf_tokens(shape: Sequence[int], vocab: int, s: float, seed: int, stream: str = "tokens") -> np.ndarray:
    """Token id r-1 with probability proportional to r^-s, r = 1..vocab (inverse CDF on uniform draws)."""
    p = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(p / p.sum())
    u = _rng(seed, stream).random(size=tuple(shape))
    return np.minimum(np.searchsorted(cdf, u, side="right"), vocab - 1).astype(np.int32)


def split_inputs_targets(seqs: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Sequences of S+1 ids -> (first S as inputs, last S as next-token targets)."""
    return np.ascontiguousarray(seqs[..., :-1]), np.ascontiguousarray(seqs[..., 1:])


def perturbation(n: int, std: float, seed: int, dtype=np.float32) -> np.ndarray:
    return (_rng(seed, "perturbation").standard_normal(n, dtype=np.float32) * np.float32(std)).astype(dtype)


def shard_weights(n_paths: int, seed: int) -> np.ndarray:
    """Un-normalised shard sizes, uniform in [0.5, 1.5]."""
    return _rng(seed, "shard_weights").uniform(0.5, 1.5, size=n_paths).astype(np.float32)


def gaussian_mixture(N: int, D: int, K: int, noise_std: float, seed: int, dtype=np.float32):
    """K unit-norm centres; N points = centre of a uniformly drawn component + isotropic noise.
    Returns (z [N,D], centres [K,D], component [N])."""
    rng = _rng(seed, "mixture")
    c = rng.standard_normal((K, D))
    c /= np.linalg.norm(c, axis=1, keepdims=True)
    comp = rng.integers(0, K, size=N)
    z = np.empty((N, D), dtype=dtype)
    step = 1 << 16
    for s in range(0, N, step):
        e = min(N, s + step)
        z[s:e] = (c[comp[s:e]] + noise_std * rng.standard_normal((e - s, D), dtype=np.float32)).astype(dtype)
    return z, c.astype(dtype), comp.astype(np.int32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 values rounded to the nearest bf16-representable value (ties to even), returned as fp32: the bf16
    configurations start from master weights that their 16-bit image represents exactly."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    u = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
    return u.view(np.float32)


def sample_offsets(n: int, count: int, seed: int, stream: str) -> np.ndarray:
    """`count` distinct sorted offsets in [0, n) (all of them when n <= count): which elements of a tensor the stored
    oracle results keep."""
    if n <= count:
        return np.arange(n, dtype=np.int64)
    return np.sort(_rng(seed, stream).choice(n, size=count, replace=False)).astype(np.int64)


def input_hash(*arrays) -> str:
    """SHA-256 over dtype, shape and bytes of the arrays: stored oracle results carry it, so that a test can tell
    whether the inputs it has just drawn are the ones those results were computed from."""
    h = hashlib.sha256()
    for x in arrays:
        x = np.ascontiguousarray(x)
        h.update(str(x.dtype).encode() + str(x.shape).encode())
        h.update(x.tobytes())
    return h.hexdigest()
