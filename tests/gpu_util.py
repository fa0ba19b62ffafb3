"""Helpers shared by the GPU parity tests: device buffers, tolerances, oracle/GPU architecture twins."""
import os

import numpy as np
import torch

import dipaco_inputs as gen
import paper_2403_10616_amd as dp
from oracle import dipaco_oracle as orc

DEV = "cuda"


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.detach().float().cpu().numpy() if t.dtype == torch.bfloat16 else t.detach().cpu().numpy()


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    nb = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / nb) if nb > 0 else float(np.linalg.norm(a))


def make_arch(cfg, compute):
    a = orc.Arch(tuple(cfg["layers_per_level"]), cfg["d_model"], cfg["n_heads"], cfg["d_head"], cfg["d_mlp"],
                 cfg["vocab"], cfg["max_seq"])
    ctx = dp.Context(list(cfg["layers_per_level"]), cfg["d_model"], cfg["n_heads"], cfg["d_head"], cfg["d_mlp"],
                     cfg["vocab"], cfg["max_seq"], a.ln_eps, compute)
    return a, ctx


class PathState:
    """Device buffers of one path: master, optional bf16 image, grads, AdamW moments, workspace."""

    def __init__(self, ctx, theta_host, batch, seq):
        self.ctx = ctx
        n = dp.dipaco_path_param_count(ctx)
        assert theta_host.shape == (n,)
        self.n = n
        self.master = dev(theta_host.astype(np.float32))
        self.lowp = self.master.to(torch.bfloat16) if ctx.compute == dp.BF16 else None
        self.grads = torch.empty(n, dtype=torch.float32, device=DEV)
        self.m = torch.zeros(n, dtype=torch.float32, device=DEV)
        self.v = torch.zeros(n, dtype=torch.float32, device=DEV)
        self.ws = torch.empty(dp.dipaco_workspace_bytes(ctx, batch, seq), dtype=torch.uint8, device=DEV)
        self.loss = torch.zeros(1, dtype=torch.float32, device=DEV)
        self.nll = torch.zeros(batch * seq, dtype=torch.float32, device=DEV)
        self.batch, self.seq = batch, seq

    def fwd_bwd(self, tok, tgt, want_nll=True):
        t = dev(tok.astype(np.int32))
        g = dev(tgt.astype(np.int32))
        dp.dipaco_path_fwd_bwd(self.ctx, self.master, self.lowp, t, g, tok.shape[0], tok.shape[1], self.loss,
                               self.nll if want_nll else None, self.grads, self.ws)
        torch.cuda.synchronize()
        return float(self.loss.item())

    def adamw(self, step, lr, b1, b2, eps, wd):
        dp.dipaco_inner_adamw(self.ctx, self.master, self.grads, self.m, self.v, self.lowp, step, lr, b1, b2, eps, wd)


def per_tensor_rel(layout, got, want, skip_zero=True):
    """max over tensors of ||got-want||/||want||, and the tensor where it occurs."""
    worst, where = 0.0, None
    for name, (off, shape, _) in layout.items():
        n = int(np.prod(shape))
        w = want[off:off + n]
        g = got[off:off + n]
        if skip_zero and not np.any(w):
            assert not np.any(g), f"{name}: expected all zeros"
            continue
        r = rel_l2(g, w)
        if r > worst:
            worst, where = r, name
    return worst, where


GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def load_golden(name):
    """Stored oracle results (written by tests/golden/make_golden.py from the oracle alone)."""
    path = os.path.join(GOLDEN, name)
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path}: run `python tests/golden/make_golden.py`")
    return np.load(path, allow_pickle=False)


def sampled_tensor_errors(gold, got_flat, samples_key, norms_key=None, got_norm=None):
    """Per tensor, on the stored sample of its elements: L2 error relative to the sample's L2 norm, largest absolute
    error relative to the sample's largest magnitude and, when the stored full norms are given, the ratio of the whole
    tensor's norm to the oracle's.  Returns a list of (name, rel_l2, rel_max, norm_ratio); tensors whose oracle values
    are all zero are checked to be zero."""
    names = [str(n) for n in gold["tensor_names"]]
    starts, flat = gold["sample_starts"], gold["sample_offsets"]
    want_all = gold[samples_key]
    out = []
    for t, name in enumerate(names):
        sl = slice(int(starts[t]), int(starts[t + 1]))
        want = want_all[sl]
        got = np.asarray(got_flat[flat[sl]], dtype=np.float64)
        if not np.any(want):
            assert not np.any(got), f"{name}: expected zeros"
            continue
        rel = float(np.linalg.norm(got - want) / np.linalg.norm(want))
        mx = float(np.abs(got - want).max() / np.abs(want).max())
        ratio = float(got_norm(name) / gold[norms_key][t]) if norms_key is not None else 1.0
        out.append((name, rel, mx, ratio))
    return out


def per_tensor_maxabs(layout, got, want):
    """max over tensors of max|got - want| / max|want|, and the tensor where it occurs (all-zero tensors skipped)."""
    worst, where = 0.0, None
    for name, (off, shape, _) in layout.items():
        n = int(np.prod(shape))
        w = np.asarray(want[off:off + n], dtype=np.float64)
        if not np.any(w):
            continue
        r = float(np.abs(np.asarray(got[off:off + n], dtype=np.float64) - w).max() / np.abs(w).max())
        if r > worst:
            worst, where = r, name
    return worst, where
