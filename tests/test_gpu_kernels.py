"""GPU parity of single kernels (through the C ABI) against their plain definitions in fp64."""
import math

import numpy as np
import pytest
import torch
from scipy.special import erf

import paper_2403_10616_amd as dp
from oracle import dipaco_oracle as orc
from gpu_util import DEV, dev, host, rel_l2

pytestmark = pytest.mark.gpu

TDT = {dp.F32: torch.float32, dp.BF16: torch.bfloat16}


def _rand(shape, seed, dtype):
    """fp32 draws, rounded to the kernel's operand type so that the fp64 reference sees the same values."""
    x = np.random.default_rng(seed).standard_normal(shape).astype(np.float32)
    t = torch.from_numpy(x).to(TDT[dtype])
    return t.to(DEV), t.to(torch.float64).numpy()


@pytest.fixture(params=[0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13], ids=lambda t: f"tile{t}")
def gemm_tile(request):
    """Every workgroup tile shape must reach the same parity; 0 is the library's own choice."""
    dp.dipaco_k_set_gemm_tile(request.param)
    yield request.param
    dp.dipaco_k_set_gemm_tile(0)


# (M, N, K): several tiles with ragged tails in every direction; K not a multiple of the K tile
GEMM_SHAPES = [(128, 128, 64), (200, 136, 72), (1, 8, 8), (300, 264, 520), (64, 512, 1000), (520, 776, 160),
               (257, 8, 32),
               # widths that are multiples of 224: the tile shape with columns every 224 takes them (tile 10)
               (300, 448, 544), (520, 224, 160), (257, 896, 64),
               # short contractions around the depth of the LDS rings (K tiles of 64 in a ring of two, of 32 in a ring of
               # four): one to five K tiles of either size, so that every prologue / steady / tail split runs
               (130, 72, 128), (300, 264, 192), (264, 520, 320), (200, 136, 96), (72, 264, 384)]


@pytest.mark.parametrize("dtype", [dp.F32, dp.BF16])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_forward_layout_with_epilogues(dtype, M, N, K, gemm_tile):
    print(f"gemm fwd tile={gemm_tile} dtype={dtype} M={M} N={N} K={K}", flush=True)
    A, Ar = _rand((M, K), 1, dtype)
    B, Br = _rand((K, N), 2, dtype)
    bias, br = _rand((N,), 3, dtype)
    resid, rr = _rand((M, N), 4, dtype)
    tol = 1e-5 if dtype == dp.F32 else 6e-3
    scale = math.sqrt(K)
    # plain
    C = torch.empty((M, N), dtype=TDT[dtype], device=DEV)
    dp.dipaco_k_gemm(dtype, False, False, False, M, N, K, A, B, C)
    ref = Ar @ Br
    assert np.abs(host(C) - ref).max() <= tol * scale * 4
    assert rel_l2(host(C), ref) <= tol
    # bias + residual
    dp.dipaco_k_gemm(dtype, False, False, False, M, N, K, A, B, C, bias=bias, resid=resid)
    assert rel_l2(host(C), ref + br + rr) <= tol
    # bias + GELU, pre-activation saved
    U = torch.empty_like(C)
    dp.dipaco_k_gemm(dtype, False, False, False, M, N, K, A, B, C, bias=bias, aux_out=U, act=1)
    u_ref = ref + br
    assert rel_l2(host(U), u_ref) <= tol
    u_seen = host(U).astype(np.float64)
    g_ref = 0.5 * u_seen * (1 + erf(u_seen / math.sqrt(2)))
    assert rel_l2(host(C), g_ref) <= tol
    # bias + GELU, derivative saved (what the path step uses): both from the unrounded pre-activation
    dp.dipaco_k_gemm(dtype, False, False, False, M, N, K, A, B, C, bias=bias, aux_out=U, act=3)
    assert rel_l2(host(C), 0.5 * u_ref * (1 + erf(u_ref / math.sqrt(2)))) <= tol
    d_ref = 0.5 * (1 + erf(u_ref / math.sqrt(2))) + u_ref * np.exp(-0.5 * u_ref * u_ref) / math.sqrt(2 * math.pi)
    assert rel_l2(host(U), d_ref) <= tol
    with pytest.raises(dp.DipacoError):
        dp.dipaco_k_gemm(dtype, False, False, False, M, N, K, A, B, C, act=1)   # no aux_out: refused on the host


@pytest.mark.parametrize("dtype", [dp.F32, dp.BF16])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_input_gradient_layout(dtype, M, N, K, gemm_tile):
    print(f"gemm dX tile={gemm_tile} dtype={dtype} M={M} N={N} K={K}", flush=True)
    A, Ar = _rand((M, K), 5, dtype)
    Bt, Btr = _rand((N, K), 6, dtype)          # B stored [N, K]
    U, Ur = _rand((M, N), 7, dtype)
    tol = 1e-5 if dtype == dp.F32 else 6e-3
    C = torch.empty((M, N), dtype=TDT[dtype], device=DEV)
    dp.dipaco_k_gemm(dtype, False, True, False, M, N, K, A, Bt, C)
    ref = Ar @ Btr.T
    assert rel_l2(host(C), ref) <= tol
    dp.dipaco_k_gemm(dtype, False, True, False, M, N, K, A, Bt, C, aux_in=U, act=2)
    gp = 0.5 * (1 + erf(Ur / math.sqrt(2))) + Ur * np.exp(-0.5 * Ur * Ur) / math.sqrt(2 * math.pi)
    assert rel_l2(host(C), ref * gp) <= tol
    dp.dipaco_k_gemm(dtype, False, True, False, M, N, K, A, Bt, C, aux_in=U, act=4)   # plain multiplication
    assert rel_l2(host(C), ref * Ur) <= tol


@pytest.mark.parametrize("dtype", [dp.F32, dp.BF16])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES + [(1000, 264, 64)])
def test_gemm_column_sums_of_the_output(dtype, M, N, K, gemm_tile):
    """The bias gradient taken in the epilogue: column sums of what the product writes (here the input-gradient
    layout with the saved-operand multiplication, as in the step)."""
    print(f"gemm colsum tile={gemm_tile} dtype={dtype} M={M} N={N} K={K}", flush=True)
    A, Ar = _rand((M, K), 11, dtype)
    Bt, Btr = _rand((N, K), 12, dtype)
    U, Ur = _rand((M, N), 13, dtype)
    C = torch.empty((M, N), dtype=TDT[dtype], device=DEV)
    cs = torch.full((N,), 77.0, dtype=torch.float32, device=DEV)
    scratch = torch.full((((M + 31) // 32) * N,), float("nan"), dtype=torch.float32, device=DEV)
    dp.dipaco_k_gemm_colsum(dtype, False, True, M, N, K, A, Bt, C, None, None, None, U, 4, cs, scratch)
    ref = (Ar @ Btr.T) * Ur
    tol = 1e-5 if dtype == dp.F32 else 6e-3
    assert rel_l2(host(C), ref) <= tol
    want = ref.sum(0)
    scale = np.abs(ref).sum(0).max()
    assert np.abs(host(cs) - want).max() <= (2e-6 if dtype == dp.F32 else 2e-3) * scale
    # forward layout with bias: same sums
    B2, B2r = _rand((K, N), 14, dtype)
    bias, biasr = _rand((N,), 15, dtype)
    dp.dipaco_k_gemm_colsum(dtype, False, False, M, N, K, A, B2, C, bias, None, None, None, 0, cs, scratch)
    ref2 = Ar @ B2r + biasr
    assert np.abs(host(cs) - ref2.sum(0)).max() <= (2e-6 if dtype == dp.F32 else 2e-3) * np.abs(ref2).sum(0).max()


@pytest.mark.parametrize("dtype", [dp.F32, dp.BF16])
@pytest.mark.parametrize("M,N,K,splits", [(128, 128, 64, 1), (200, 136, 77, 1), (72, 264, 1000, 4), (8, 8, 5, 1),
                                          (136, 64, 4099, 16), (264, 520, 1024, 5), (8, 776, 96, 1),
                                          (896, 1024, 2048, 8), (384, 1160, 512, 3)])
def test_gemm_weight_gradient_layout_and_split_k(dtype, M, N, K, splits, gemm_tile):
    print(f"gemm dW tile={gemm_tile} dtype={dtype} M={M} N={N} K={K} splits={splits}", flush=True)
    At, Atr = _rand((K, M), 8, dtype)          # A stored [K, M]: contraction over rows (tokens)
    B, Br = _rand((K, N), 9, dtype)
    C = torch.empty((M, N), dtype=torch.float32, device=DEV)
    partial = torch.empty((splits, M, N), dtype=torch.float32, device=DEV) if splits > 1 else None
    dp.dipaco_k_gemm(dtype, True, False, True, M, N, K, At, B, C, splits=splits, partial=partial)
    ref = Atr.T @ Br
    assert rel_l2(host(C), ref) <= 2e-6
    first = host(C).copy()
    dp.dipaco_k_gemm(dtype, True, False, True, M, N, K, At, B, C, splits=splits, partial=partial)
    assert np.array_equal(first, host(C))       # fixed summation order: bit-identical from call to call


def _attn_ref(qkv, B, S, H, dh):
    a = orc.Arch((1,), H * dh, H, dh, 8, 8, S)
    A = H * dh
    o = np.empty((B * S, A))
    lse = np.empty((B, H, S))
    probs = []
    for b in range(B):
        x = qkv[b * S:(b + 1) * S]
        ob, pb = orc._attention(x[:, :A], x[:, A:2 * A], x[:, 2 * A:], a)
        o[b * S:(b + 1) * S] = ob
        probs.append(pb)
        for h in range(H):
            s = (x[:, h * dh:(h + 1) * dh] @ x[:, A + h * dh:A + (h + 1) * dh].T) / math.sqrt(dh)
            s = np.where(np.tril(np.ones((S, S), bool)), s, -np.inf)
            mx = s.max(-1)
            lse[b, h] = mx + np.log(np.exp(s - mx[:, None]).sum(-1))
    return a, o, lse, probs


@pytest.fixture(params=[1, 0], ids=["single_block", "paired_blocks"])
def attn_blocks(request):
    """Both ways of dealing the causal triangle's blocks to workgroups; 1 is the default."""
    dp.dipaco_k_set_attention_blocks(request.param)
    yield request.param
    dp.dipaco_k_set_attention_blocks(1)


@pytest.mark.parametrize("dtype", [dp.F32, dp.BF16])
@pytest.mark.parametrize("B,S,H,dh", [(2, 64, 2, 32), (1, 200, 3, 64), (2, 77, 1, 128), (1, 1, 2, 64), (1, 333, 2, 64),
                                      (2, 1024, 2, 64), (1, 130, 1, 64), (1, 900, 1, 64), (1, 2048, 2, 64),
                                      (1, 1100, 1, 64)])
def test_attention_forward_backward(dtype, B, S, H, dh, attn_blocks):
    print(f"attention dtype={dtype} B={B} S={S} H={H} dh={dh} blocks={attn_blocks}", flush=True)
    A = H * dh
    qkv, qr = _rand((B * S, 3 * A), 10, dtype)
    d_o, gr = _rand((B * S, A), 11, dtype)
    o = torch.empty((B * S, A), dtype=TDT[dtype], device=DEV)
    lse = torch.empty((B, H, S), dtype=torch.float32, device=DEV)
    dp.dipaco_k_attention_fwd(dtype, qkv, o, lse, B, S, H, dh)
    a, o_ref, lse_ref, probs = _attn_ref(qr, B, S, H, dh)
    tol = 2e-5 if dtype == dp.F32 else 1e-2
    assert rel_l2(host(o), o_ref) <= tol
    # every element: the probabilities enter the second product rounded to bf16 (relative 2^-9 each, averaging out
    # over a row) and the result is rounded once more
    o_err = np.abs(host(o) - o_ref).max() / np.abs(o_ref).max()
    assert o_err <= (1e-5 if dtype == dp.F32 else 8e-3), o_err
    assert np.abs(host(lse) - lse_ref).max() <= (1e-5 if dtype == dp.F32 else 2e-2)
    dqkv = torch.empty_like(qkv)
    dsum = torch.empty(2 * B * H * ((S + 127) // 128 * 128), dtype=torch.float32, device=DEV)
    cs = torch.full((3 * A,), 55.0, dtype=torch.float32, device=DEV)
    cs_scratch = torch.full((max((B * S + 255) // 256, B * ((S + 127) // 128)) * 3 * A,), float("nan"),
                            dtype=torch.float32, device=DEV)
    dp.dipaco_k_attention_bwd(dtype, qkv, o, d_o, lse, dqkv, dsum, B, S, H, dh, colsum_out=cs, colsum_scratch=cs_scratch)
    ref = np.empty((B * S, 3 * A))
    for b in range(B):
        x = qr[b * S:(b + 1) * S]
        dq, dk, dv = orc._attention_bwd(gr[b * S:(b + 1) * S], x[:, :A], x[:, A:2 * A], x[:, 2 * A:], probs[b], a)
        ref[b * S:(b + 1) * S] = np.concatenate([dq, dk, dv], axis=1)
    got = host(dqkv)
    for name, sl in (("dq", slice(0, A)), ("dk", slice(A, 2 * A)), ("dv", slice(2 * A, 3 * A))):
        assert rel_l2(got[:, sl], ref[:, sl]) <= (2e-5 if dtype == dp.F32 else 2e-2), name
        top = np.abs(ref[:, sl]).max()
        worst = np.abs(got[:, sl] - ref[:, sl]).max() / (top if top > 0 else 1.0)      # S = 1: dq and dk are zero
        print(f"  {name}: max-abs error / max |{name}| = {worst:.2e}, o: {o_err:.2e}", flush=True)
        assert worst <= (2e-5 if dtype == dp.F32 else 2e-2), (name, worst)
    # column sums of dqkv (the QKV bias gradient), taken in the kernels' epilogues where the matrix-core path runs
    scale = np.abs(ref).sum(0).max()
    assert np.abs(host(cs) - ref.sum(0)).max() <= (1e-5 if dtype == dp.F32 else 1e-2) * scale
    dqkv2 = torch.empty_like(qkv)
    dp.dipaco_k_attention_bwd(dtype, qkv, o, d_o, lse, dqkv2, dsum, B, S, H, dh)            # without the sums
    assert torch.equal(dqkv2, dqkv)


# ---- the benchmarked kernels at the step's own shapes, element by element ---------------------------------------
def _bf16_ulp(x):
    """Spacing of bf16 numbers at |x| (8 significant bits)."""
    mag = np.maximum(np.abs(x), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(mag)) - 7)


def _assert_within_one_bf16_ulp(got, ref, what):
    """The kernels accumulate exactly representable bf16 products in fp32 and round once: the stored value is the
    fp64 result rounded to bf16, give or take the fp32 accumulation error (which can tip a rounding, and is all that
    is left of elements near zero: 2e-5 of the result's typical magnitude covers it)."""
    got = got.astype(np.float64)
    slack = 2e-5 * math.sqrt(float(np.mean(ref * ref)))
    excess = np.abs(got - ref) - (_bf16_ulp(np.maximum(np.abs(ref), np.abs(got))) + slack)
    worst = int(np.argmax(excess))
    assert excess.flat[worst] <= 0, (what, np.unravel_index(worst, ref.shape), got.flat[worst], ref.flat[worst])


STEP_M = 32768
# (name, M, N, K): the forward products of one block at config 2 and a 4096-row slice of the vocabulary head
STEP_FORWARD = [("qkv", STEP_M, 2688, 896), ("out_proj", STEP_M, 896, 896), ("mlp_up", STEP_M, 3584, 896),
                ("mlp_down", STEP_M, 896, 3584), ("head_rows", 4096, 32000, 896)]


@pytest.mark.parametrize("name,M,N,K", STEP_FORWARD, ids=[s[0] for s in STEP_FORWARD])
def test_bf16_forward_products_of_the_step_element_by_element(name, M, N, K):
    print(f"step-shape forward product {name} M={M} N={N} K={K}", flush=True)
    A, Ar = _rand((M, K), 21, dp.BF16)
    B, Br = _rand((K, N), 22, dp.BF16)
    Br *= 0.05                                   # weight-sized entries keep GELU in its curved range
    B = torch.from_numpy(Br).to(torch.bfloat16)
    Br = B.to(torch.float64).numpy()
    B = B.to(DEV)
    bias, br = _rand((N,), 23, dp.BF16)
    resid, rr = _rand((M, N), 24, dp.BF16)
    ref = Ar @ Br
    C = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    if name == "head_rows":                      # plain product
        dp.dipaco_k_gemm(dp.BF16, False, False, False, M, N, K, A, B, C)
        _assert_within_one_bf16_ulp(host(C), ref, name)
        return
    if name == "mlp_up":                         # + bias, GELU out, GELU' saved
        U = torch.empty_like(C)
        dp.dipaco_k_gemm(dp.BF16, False, False, False, M, N, K, A, B, C, bias=bias, aux_out=U, act=3)
        u = ref + br
        cdf = 0.5 * (1 + erf(u / math.sqrt(2)))
        _assert_within_one_bf16_ulp(host(C), u * cdf, name + " GELU")
        _assert_within_one_bf16_ulp(host(U), cdf + u * np.exp(-0.5 * u * u) / math.sqrt(2 * math.pi), name + " GELU'")
        return
    if name == "qkv":                            # + bias
        dp.dipaco_k_gemm(dp.BF16, False, False, False, M, N, K, A, B, C, bias=bias)
        _assert_within_one_bf16_ulp(host(C), ref + br, name)
        return
    dp.dipaco_k_gemm(dp.BF16, False, False, False, M, N, K, A, B, C, bias=bias, resid=resid)   # + bias + residual
    _assert_within_one_bf16_ulp(host(C), ref + br + rr, name)


# input-gradient products dX = dY W^T (W stored [N_out = rows here, K]) of one block, and a slice of the head's
STEP_INPUT_GRAD = [("d_qkv_in", STEP_M, 896, 2688), ("d_out_proj_in", STEP_M, 896, 896), ("d_mlp_up_in", STEP_M, 896, 3584),
                   ("d_mlp_down_in", STEP_M, 3584, 896), ("d_head_in_rows", 4096, 896, 32000)]


@pytest.mark.parametrize("name,M,N,K", STEP_INPUT_GRAD, ids=[s[0] for s in STEP_INPUT_GRAD])
def test_bf16_input_gradient_products_of_the_step_element_by_element(name, M, N, K):
    print(f"step-shape input-gradient product {name} M={M} N={N} K={K}", flush=True)
    A, Ar = _rand((M, K), 25, dp.BF16)
    Bt, Btr = _rand((N, K), 26, dp.BF16)
    ref = Ar @ Btr.T
    C = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    if name != "d_mlp_down_in":
        dp.dipaco_k_gemm(dp.BF16, False, True, False, M, N, K, A, Bt, C)
        _assert_within_one_bf16_ulp(host(C), ref, name)
        return
    # the product that writes dU: multiplied by the saved GELU', with the column sums (the gradient of b_up)
    U, Ur = _rand((M, N), 27, dp.BF16)
    cs = torch.full((N,), 77.0, dtype=torch.float32, device=DEV)
    scratch = torch.full((((M + 31) // 32) * N,), float("nan"), dtype=torch.float32, device=DEV)
    dp.dipaco_k_gemm_colsum(dp.BF16, False, True, M, N, K, A, Bt, C, None, None, None, U, 4, cs, scratch)
    ref = ref * Ur
    _assert_within_one_bf16_ulp(host(C), ref, name)
    assert np.abs(host(cs) - ref.sum(0)).max() <= 1e-5 * np.abs(ref).sum(0).max()   # fp32 sums of unrounded values


STEP_WEIGHT_GRAD = [("d_w_qkv", 896, 2688), ("d_w_o", 896, 896), ("d_w_up", 896, 3584), ("d_w_down", 3584, 896)]


@pytest.mark.parametrize("name,M,N", STEP_WEIGHT_GRAD, ids=[s[0] for s in STEP_WEIGHT_GRAD])
def test_bf16_weight_gradient_products_of_the_step_element_by_element(name, M, N):
    """dW = X^T dY over the 32768 tokens, fp32 out, with the split-K plan the step launches them with."""
    K = STEP_M
    print(f"step-shape weight-gradient product {name} M={M} N={N} K={K}", flush=True)
    At, Atr = _rand((K, M), 28, dp.BF16)
    B, Br = _rand((K, N), 29, dp.BF16)
    plan = dp.dipaco_k_gemm_split_plan(M, N, K, 32)
    splits = max(plan["slices"]) if plan["tile"][0] else 8
    C = torch.empty((M, N), dtype=torch.float32, device=DEV)
    partial = torch.empty((splits, M, N), dtype=torch.float32, device=DEV)
    dp.dipaco_k_gemm(dp.BF16, True, False, True, M, N, K, At, B, C, splits=splits, partial=partial)
    ref = Atr.T @ Br
    rms = math.sqrt(float(np.mean(ref * ref)))
    err = np.abs(host(C).astype(np.float64) - ref)
    assert err.max() <= 1e-4 * rms, (name, np.unravel_index(int(np.argmax(err)), ref.shape), err.max() / rms)
