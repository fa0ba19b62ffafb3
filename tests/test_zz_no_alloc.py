"""The router-feature entry point that allocates nothing (static device scratch) against the workspace entry point it
is a variant of: identical bits, on two calls in a row of which the second is smaller, plus the oracle's features and
the size limit.  Collected last: a failure here must not hide the other GPU tests."""
import numpy as np
import pytest
import torch

import dipaco_inputs as gen
import paper_2403_10616_amd as dp
from oracle import dipaco_oracle as orc
from gpu_util import DEV, dev, host, make_arch, rel_l2

pytestmark = pytest.mark.gpu

ARCHS = {
    "bf16_d128": (dict(layers_per_level=(2, 1), d_model=128, n_heads=2, d_head=64, d_mlp=512, vocab=1000, max_seq=64),
                  dp.BF16, 2e-2),
    "fp32_ragged": (dict(layers_per_level=(1, 2), d_model=72, n_heads=3, d_head=32, d_mlp=200, vocab=264, max_seq=56),
                    dp.F32, 1e-5),
}


def _params(a, seed):
    lay = orc.param_layout(a)
    theta = gen.random_params(orc.param_count(a), seed=seed, scale=0.08)
    for name, (off, shape, _) in lay.items():
        if name.endswith("_g"):
            theta[off:off + shape[0]] += 1.0
    return theta


@pytest.mark.parametrize("name", sorted(ARCHS))
def test_static_scratch_features_equal_workspace_features_on_two_calls(name):
    cfg, compute, tol = ARCHS[name]
    a, ctx = make_arch(cfg, compute)
    theta = _params(a, 51)
    master = dev(theta.astype(np.float32))
    lowp = master.to(torch.bfloat16) if compute == dp.BF16 else None
    ref_theta = theta if compute == dp.F32 else gen.round_to_bf16(theta)
    assert dp.dipaco_static_scratch_bytes() == 64 << 20
    for call, (B, S) in enumerate([(40, 32), (5, 17)]):          # the second call is smaller and reuses the array
        print(f"no-alloc features {name} call {call} B={B} S={S}", flush=True)
        tok = gen.uniform_tokens((B, S), cfg["vocab"], 52 + call)
        tok_d = dev(tok.astype(np.int32))
        assert dp.dipaco_features_workspace_bytes(ctx, B, S) <= dp.dipaco_static_scratch_bytes()
        want = torch.full((B, a.d_model), 7.0, dtype=torch.float32, device=DEV)
        ws = torch.empty(dp.dipaco_features_workspace_bytes(ctx, B, S), dtype=torch.uint8, device=DEV)
        dp.dipaco_path_prefix_features(ctx, master, lowp, tok_d, B, S, want, ws)
        got = torch.full((B, a.d_model), -7.0, dtype=torch.float32, device=DEV)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        dp.dipaco_path_prefix_features_static(ctx, master, lowp, tok_d, B, S, got)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(got, want)                           # same kernels, same order: identical bits
        o = orc.prefix_features(ref_theta, a, tok)
        assert rel_l2(host(got), o) <= tol


def test_static_scratch_refuses_what_does_not_fit():
    cfg, compute, _ = ARCHS["bf16_d128"]
    cfg = dict(cfg, max_seq=4096)
    a, ctx = make_arch(cfg, compute)
    B, S = 64, 4096
    assert dp.dipaco_features_workspace_bytes(ctx, B, S) > dp.dipaco_static_scratch_bytes()
    n = dp.dipaco_path_param_count(ctx)
    master = torch.zeros(n, dtype=torch.float32, device=DEV)
    out = torch.zeros((B, a.d_model), dtype=torch.float32, device=DEV)
    tok = torch.zeros((B, S), dtype=torch.int32, device=DEV)
    with pytest.raises(dp.DipacoError, match="static scratch"):
        dp.dipaco_path_prefix_features_static(ctx, master, master.to(torch.bfloat16), tok, B, S, out)
