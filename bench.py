#!/usr/bin/env python3
"""Benchmark of the DiPaCo path step on one MI355X.

Default workload ("path_step"): one inner step of a 174M-parameter path -- forward, backward and AdamW over a
[32, 1024] batch of Zipf(1.1) tokens, bf16 compute with fp32 master weights and optimiser state -- through the
C-ABI calls dipaco_path_fwd_bwd + dipaco_inner_adamw.  Prints ONE JSON line.

Other workloads (for profiling single kernels; same JSON shape):
  --workload outer_step   16 deltas x 57,872,640 parameters, weighted mean + Nesterov
  --workload route        2^20 x 768 prefix embeddings against 256 centroids
  --workload outer_stream the same module, the 16 deltas accumulated one at a time, then the Nesterov update
  --workload outer_table  two shared modules (16 deltas each) and 32 path-specific blocks updated by one launch
  --workload features     router features of 8192 documents (32-token prefixes) through the config-2 path's blocks
  --workload score        forward-only log-likelihood of 16 documents x 2048 tokens under the config-5 path
  --workload router       discriminative router on the config-4 data: logistic loss + gradients, and linear routing
  --workload reroute      evaluation at seq 2048 under 4 paths with the path re-chosen every 128 tokens
  --workload kmeans       one Lloyd iteration on the config-4 data: top-1 (or --n-best 2) assignment + centroid update
  --workload gemm         one bf16 GEMM of the step: --mnk M,N,K --layout nn|nt|tn --epilogue none|bias|gelu|dgelu|resid
  --workload attention    causal attention of one layer of the step (batch 32 x 14 heads x 1024 x 64): --pass fwd|bwd
  --workload issue_probe  register-only loops: do matrix-core and vector-ALU instructions of a SIMD overlap?
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3     # MI355X fp32 MFMA
PEAK_HBM_GBS = 8000.0
TRAFFIC_PROFILE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "path_step_config2_traffic.txt")


def fwd_gemm_traffic_bytes():
    """Bytes that crossed the L2 / memory-fabric boundary per launch of the forward-layout GEMM, averaged over its
    launches in the config-2 step: the last line of the committed counter summary (read requests x 128 B + write
    requests x 64 B, from two `rocprofv3 --pmc` runs; that file derives the request sizes from kernels of known
    traffic and states the algorithmic figure, 366.2 MB, beside it).  None when the summary is not there."""
    try:
        with open(TRAFFIC_PROFILE) as f:
            for line in f:
                if line.startswith("TRAFFIC_BYTES_PER_LAUNCH_FWD_GEMM"):
                    return float(line.split()[1])
    except OSError:
        pass
    return None


def _events(torch):
    return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)


def _arch_kwargs(cfg, compute):
    return dict(layers_per_level=list(cfg["layers_per_level"]), d_model=cfg["d_model"], n_heads=cfg["n_heads"],
                d_head=cfg["d_head"], d_mlp=cfg["d_mlp"], vocab=cfg["vocab"], max_seq=cfg["max_seq"], compute=compute)


def step_gemm_shapes(cfg, B, S):
    """(M, N, K) of every GEMM launch of one step, by kernel instantiation (operand layout)."""
    T, d, A, F, V = B * S, cfg["d_model"], cfg["n_heads"] * cfg["d_head"], cfg["d_mlp"], cfg["vocab"]
    NL = sum(cfg["layers_per_level"])
    fwd = [(T, 3 * A, d), (T, d, A), (T, F, d), (T, d, F)] * NL + [(T, V, d)]
    dx = [(T, F, d), (T, d, F), (T, A, d), (T, d, 3 * A)] * NL + [(T, d, V)]
    dw = [(F, d, T), (d, F, T), (A, d, T), (d, 3 * A, T)] * NL + [(d, V, T)]
    return fwd, dx, dw


def attention_flops(cfg, B, S):
    H, dh = cfg["n_heads"], cfg["d_head"]
    NL = sum(cfg["layers_per_level"])
    fwd = NL * B * H * (2 * 2 * S * S * dh) / 2          # QK^T and PV over the causal half
    # backward: the four products the definition has (dV, dP, dQ, dK), twice the forward pass; the scores that the
    # kernels recompute are not model work and are not counted
    return fwd, 2.0 * fwd


def bench_path_step(args):
    import torch
    import dipaco_inputs as gen
    import paper_2403_10616_amd as dp

    cfg = gen.CONFIGS[2]
    B, S = cfg["batch"], cfg["seq"]
    ctx = dp.Context(**_arch_kwargs(cfg, dp.BF16))
    if args.gemm_tile:
        dp.dipaco_k_set_gemm_tile(args.gemm_tile)
    n = dp.dipaco_path_param_count(ctx)
    layout = {}
    for i in range(dp.dipaco_tensor_count(ctx)):
        name, off, rows, cols, dec = dp.dipaco_tensor_info(ctx, i)
        layout[name] = (off, (rows, cols) if cols > 1 else (rows,), dec)
    n_layers = sum(cfg["layers_per_level"])
    theta = gen.init_params(layout, n_layers, cfg["seed"])
    dev = "cuda"
    # the path is composed from its four global segments, as at the start of a round
    segs = []
    for s_ in range(dp.dipaco_segment_count(ctx)):
        lo = dp.dipaco_segment_offset(ctx, s_)
        segs.append(torch.from_numpy(theta[lo:lo + dp.dipaco_segment_size(ctx, s_)]).to(dev))
    master = torch.empty(n, dtype=torch.float32, device=dev)
    lowp = torch.empty(n, dtype=torch.bfloat16, device=dev)
    dp.dipaco_compose_path(ctx, segs, master, lowp)
    del segs
    grads = torch.empty(n, dtype=torch.float32, device=dev)
    m = torch.zeros(n, dtype=torch.float32, device=dev)
    v = torch.zeros(n, dtype=torch.float32, device=dev)
    ws = torch.empty(dp.dipaco_workspace_bytes(ctx, B, S), dtype=torch.uint8, device=dev)
    loss = torch.zeros(1, dtype=torch.float32, device=dev)
    n_batches = min(4, args.steps + args.warmup)
    seqs = gen.zipf_tokens((n_batches, B, S + 1), cfg["vocab"], cfg["zipf_s"], cfg["seed"])
    toks = [torch.from_numpy(np.ascontiguousarray(seqs[i, :, :-1])).to(dev) for i in range(n_batches)]
    tgts = [torch.from_numpy(np.ascontiguousarray(seqs[i, :, 1:])).to(dev) for i in range(n_batches)]

    def step(i):
        dp.dipaco_path_fwd_bwd(ctx, master, lowp, toks[i % n_batches], tgts[i % n_batches], B, S, loss, None, grads, ws)
        dp.dipaco_inner_adamw(ctx, master, grads, m, v, lowp, i + 1, cfg["lr"], cfg["beta1"], cfg["beta2"], cfg["eps"],
                              cfg["wd"])

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = _events(torch)
    t0 = time.perf_counter()
    e0.record()
    for i in range(args.steps):
        step(args.warmup + i)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    final_loss = float(loss.item())

    # ---- roofline of the dominant kernel: the forward-layout bf16 GEMM (projections, MLP, vocabulary head) ----
    # Its 49 launches of one step are replayed with the step's own epilogues (bias, GELU + saved GELU',
    # residual) on scratch operands and timed with events on the stream they are launched on.
    fwd, dx, dw = step_gemm_shapes(cfg, B, S)
    T = B * S
    big = max(max(M * N for M, N, K in fwd), max(M * K for M, N, K in fwd))
    a_buf = torch.empty(big, dtype=torch.bfloat16, device=dev).normal_()
    b_buf = torch.empty(max(K * N for M, N, K in fwd), dtype=torch.bfloat16, device=dev).normal_(std=0.02)
    c_buf = torch.empty(big, dtype=torch.bfloat16, device=dev)
    r_buf = torch.empty(T * cfg["d_mlp"], dtype=torch.bfloat16, device=dev).normal_()
    u_buf = torch.empty(T * cfg["d_mlp"], dtype=torch.bfloat16, device=dev)
    bias = torch.zeros(max(N for M, N, K in fwd), dtype=torch.bfloat16, device=dev)
    epilogues = [dict(bias=bias), dict(bias=bias, resid=r_buf), dict(bias=bias, aux_out=u_buf, act=3),
                 dict(bias=bias, resid=r_buf)] * n_layers + [dict()]

    def replay():
        for (M, N, K), ep in zip(fwd, epilogues):
            dp.dipaco_k_gemm(dp.BF16, False, False, False, M, N, K, a_buf, b_buf, c_buf, **ep)
    replay()
    torch.cuda.synchronize()
    reps = max(1, min(args.steps, 5))
    e0.record()
    for _ in range(reps):
        replay()
    e1.record()
    torch.cuda.synchronize()
    gemm_ms = e0.elapsed_time(e1) / reps
    fwd_flops = sum(2.0 * M * N * K for M, N, K in fwd)
    achieved = fwd_flops / (gemm_ms * 1e-3) / 1e12
    att_f, att_b = attention_flops(cfg, B, S)
    step_flops = 3.0 * fwd_flops + att_f + att_b
    out = {
        "metric": "path-step tokens/sec on 1 MI355X (~150M path fwd+bwd+AdamW)", "value": B * S / (ms_per_step * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config 2: 174.0M-parameter path (12 blocks, d 896, 14x64 heads, MLP 3584, vocab 32000), "
                               "batch 32 x seq 1024 Zipf(1.1) tokens, one fwd+bwd+AdamW step",
                   "params": n, "tokens_per_step": B * S, "final_loss": final_loss,
                   "model_tflops_per_step": step_flops / 1e12,
                   "model_flops_utilisation": step_flops / (ms_per_step * 1e-3) / (PEAK_BF16_TFLOPS * 1e12)},
        "roofline": {"bound": "mfma", "kernel": "gemm_dlds_kernel<bf16 out, A [M,K], B [K,N]> (forward layout)",
                     "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                     "traffic": fwd_gemm_traffic_bytes(), "traffic_unit": "bytes per launch (fetch + write)",
                     "launches_per_step": len(fwd), "flops_per_launch": fwd_flops / len(fwd),
                     "avg_launch_us": gemm_ms * 1e3 / len(fwd)},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_path_step(cfg, theta, seqs[0, :3], layout)
    return out


def cpu_baseline_path_step(cfg, theta, seqs, layout):
    """The oracle (numpy fp64, as it stands) on one sequence of the same batch: forward, backward, AdamW."""
    from oracle import dipaco_oracle as orc
    a = orc.Arch(tuple(cfg["layers_per_level"]), cfg["d_model"], cfg["n_heads"], cfg["d_head"], cfg["d_mlp"],
                 cfg["vocab"], cfg["max_seq"])
    tok, tgt = seqs[:, :-1], seqs[:, 1:]
    mask = orc.decay_mask(a)
    t0 = time.perf_counter()
    loss, g = orc.path_loss_and_grad(theta, a, tok, tgt)
    orc.adamw_step(theta, g, np.zeros_like(g), np.zeros_like(g), 1, cfg["lr"], cfg["beta1"], cfg["beta2"], cfg["eps"],
                   cfg["wd"], mask)
    dt = time.perf_counter() - t0
    return {"value": tok.size / dt, "unit": "tokens/s", "cores": _oracle_threads(), "kind": "oracle",
            "sample": f"{tok.shape[0]} of the 32 sequences ({tok.size} tokens) of the same batch, fwd+bwd+AdamW in fp64 numpy, "
                      f"{dt:.1f} s",
            "loss": loss}


def _oracle_threads():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] or [1]))
    except Exception:
        return int(os.cpu_count() or 1)


def cpu_baseline_outer_step(cfg):
    """The oracle's outer step (numpy fp64, as it stands) on the whole config-3 module: 16 weighted deltas of
    57,872,640 parameters, Nesterov update."""
    import dipaco_inputs as gen
    from oracle import dipaco_oracle as orc
    n, P = cfg["n_elems"], cfg["n_paths"]
    theta = gen.perturbation(n, 0.02, cfg["seed"])
    deltas = [gen.perturbation(n, cfg["delta_std"], 300 + i) for i in range(P)]
    w = gen.shard_weights(P, cfg["seed"])
    t0 = time.perf_counter()
    orc.outer_step(theta, np.zeros(n), deltas, w, True, cfg["outer_lr"], cfg["outer_momentum"])
    dt = time.perf_counter() - t0
    # elementwise numpy: one host thread
    return {"value": n / dt, "unit": "params/s", "cores": 1, "kind": "oracle",
            "sample": f"the whole module: {P} deltas x {n} parameters, weighted mean + Nesterov in fp64 numpy, {dt:.1f} s"}


def cpu_baseline_route(cfg, z, c, rows=16384):
    """The oracle's eq. (1) (numpy fp64 distances, as it stands) on the first `rows` points of the same set."""
    from oracle import dipaco_oracle as orc
    t0 = time.perf_counter()
    orc.route_prefix(z[:rows], c)
    dt = time.perf_counter() - t0
    # a python loop over the rows with elementwise numpy inside: one host thread
    return {"value": rows / dt, "unit": "documents/s", "cores": 1, "kind": "oracle",
            "sample": f"the first {rows} of the {len(z)} embeddings against the same {len(c)} centroids, {dt:.1f} s"}


def bench_outer_step(args):
    import torch
    import dipaco_inputs as gen
    import paper_2403_10616_amd as dp
    cfg = gen.CONFIGS[3]
    n, P = cfg["n_elems"], cfg["n_paths"]
    dev = "cuda"
    theta = torch.randn(n, device=dev) * 0.02
    buf = torch.zeros(n, device=dev)
    deltas = [torch.randn(n, device=dev) * cfg["delta_std"] for _ in range(P)]
    w = gen.shard_weights(P, cfg["seed"])

    def step():
        dp.dipaco_module_outer_step(theta, buf, deltas, w, n, True, cfg["outer_lr"], cfg["outer_momentum"])
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = _events(torch)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = e0.elapsed_time(e1) / args.steps
    bytes_ = (P + 4) * n * 4.0
    ach = bytes_ / (ms * 1e-3) / 1e9
    out = {"metric": "module outer-step parameters/sec on 1 MI355X", "value": n / (wall / args.steps), "unit": "params/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": "config 3: 57,872,640-parameter module, 16 weighted deltas, Nesterov"},
           "roofline": {"bound": "hbm", "kernel": "outer_kernel<16>", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": ach / PEAK_HBM_GBS, "traffic": None, "bytes_per_launch": bytes_}}
    if not args.no_cpu_baseline:
        del deltas, theta, buf
        out["cpu_baseline"] = cpu_baseline_outer_step(cfg)
    return out


def bench_round(args):
    """Config 5: one full round of one path = compose from the global segments, 8 inner steps (fwd + bwd + AdamW) at
    batch 16 x seq 2048, then the outer Nesterov step of the path's two block modules, each averaged with the copies of
    15 synthetic partner paths, and the new modules written back to the global segments.  A 'step' is one round."""
    import torch
    import dipaco_inputs as gen
    import paper_2403_10616_amd as dp

    cfg = gen.CONFIGS[5]
    B, S, inner, P = cfg["batch"], cfg["seq"], cfg["inner_steps"], cfg["n_partners"]
    ctx = dp.Context(**_arch_kwargs(cfg, dp.BF16))
    n = dp.dipaco_path_param_count(ctx)
    layout = {}
    for i in range(dp.dipaco_tensor_count(ctx)):
        name, off, rows, cols, dec = dp.dipaco_tensor_info(ctx, i)
        layout[name] = (off, (rows, cols) if cols > 1 else (rows,), dec)
    theta = gen.init_params(layout, sum(cfg["layers_per_level"]), cfg["seed"])
    dev = "cuda"
    nseg = dp.dipaco_segment_count(ctx)
    bounds = [(dp.dipaco_segment_offset(ctx, s_), dp.dipaco_segment_offset(ctx, s_) + dp.dipaco_segment_size(ctx, s_))
              for s_ in range(nseg)]
    segs = [torch.from_numpy(theta[lo:hi]).to(dev) for lo, hi in bounds]          # the global modules
    momentum = {l: torch.zeros(bounds[l][1] - bounds[l][0], dtype=torch.float32, device=dev) for l in (1, 2)}
    # the partners' local copies of the two block modules at the end of the round: global module + N(0, 1e-3)
    partners = {}
    for l in (1, 2):
        lo, hi = bounds[l]
        partners[l] = [torch.from_numpy((theta[lo:hi] + gen.perturbation(hi - lo, cfg["delta_std"], 500 + 16 * l + i))
                                        .astype(np.float32)).to(dev) for i in range(P)]
    master = torch.empty(n, dtype=torch.float32, device=dev)
    lowp = torch.empty(n, dtype=torch.bfloat16, device=dev)
    grads = torch.empty(n, dtype=torch.float32, device=dev)
    m = torch.zeros(n, dtype=torch.float32, device=dev)
    v = torch.zeros(n, dtype=torch.float32, device=dev)
    ws = torch.empty(dp.dipaco_workspace_bytes(ctx, B, S), dtype=torch.uint8, device=dev)
    loss = torch.zeros(1, dtype=torch.float32, device=dev)
    seqs = gen.zipf_tokens((inner, B, S + 1), cfg["vocab"], cfg["zipf_s"], cfg["seed"])
    toks = [torch.from_numpy(np.ascontiguousarray(seqs[i, :, :-1])).to(dev) for i in range(inner)]
    tgts = [torch.from_numpy(np.ascontiguousarray(seqs[i, :, 1:])).to(dev) for i in range(inner)]
    t_adam = [0]

    def one_round():
        dp.dipaco_compose_path(ctx, segs, master, lowp)
        for i in range(inner):
            dp.dipaco_path_fwd_bwd(ctx, master, lowp, toks[i], tgts[i], B, S, loss, None, grads, ws)
            t_adam[0] += 1
            dp.dipaco_inner_adamw(ctx, master, grads, m, v, lowp, t_adam[0], cfg["lr"], cfg["beta1"], cfg["beta2"],
                                  cfg["eps"], cfg["wd"])
        for l in (1, 2):
            lo, hi = bounds[l]
            dp.dipaco_module_outer_step(segs[l], momentum[l], [master[lo:hi]] + partners[l], None, hi - lo, False,
                                        cfg["outer_lr"], cfg["outer_momentum"])
        # stem and head are this path's own in this workload: carried over as they are
        segs[0].copy_(master[bounds[0][0]:bounds[0][1]])
        segs[nseg - 1].copy_(master[bounds[nseg - 1][0]:bounds[nseg - 1][1]])

    for _ in range(args.warmup):
        one_round()
    torch.cuda.synchronize()
    e0, e1 = _events(torch)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_round()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    # the outer step alone, on the stream's events
    lo, hi = bounds[1]
    e0.record()
    dp.dipaco_module_outer_step(segs[1], momentum[1], [master[lo:hi]] + partners[1], None, hi - lo, False,
                                cfg["outer_lr"], cfg["outer_momentum"])
    e1.record()
    torch.cuda.synchronize()
    outer_ms = e0.elapsed_time(e1)
    outer_bytes = (P + 1 + 4) * (hi - lo) * 4.0
    ach = outer_bytes / (outer_ms * 1e-3) / 1e9
    ms = wall * 1e3 / args.steps
    fwd, dx, dw = step_gemm_shapes(cfg, B, S)
    att_f, att_b = attention_flops(cfg, B, S)
    step_flops = 3.0 * sum(2.0 * M * N * K for M, N, K in fwd) + att_f + att_b
    return {"metric": "full-round tokens/sec on 1 MI355X (8 inner steps + outer step of two modules)",
            "value": inner * B * S / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "config 5: one round of one path: compose, 8 x (fwd+bwd+AdamW) at batch 16 x seq 2048, "
                                   "outer Nesterov step of both 57.9M-parameter modules over 16 copies each",
                       "tokens_per_round": inner * B * S, "final_loss": float(loss.item()),
                       "model_tflops_per_round": inner * step_flops / 1e12,
                       "model_flops_utilisation": inner * step_flops / (ms * 1e-3) / (PEAK_BF16_TFLOPS * 1e12),
                       "outer_step_ms_per_module": outer_ms},
            "roofline": {"bound": "hbm", "kernel": "outer_kernel<16> (copies form)", "achieved": ach, "peak": PEAK_HBM_GBS,
                         "unit": "GB/s", "frac": ach / PEAK_HBM_GBS, "traffic": None, "bytes_per_launch": outer_bytes}}


def bench_outer_stream(args):
    import torch
    import dipaco_inputs as gen
    import paper_2403_10616_amd as dp
    cfg = gen.CONFIGS[3]
    n, P = cfg["n_elems"], cfg["n_paths"]
    dev = "cuda"
    theta = torch.randn(n, device=dev) * 0.02
    buf = torch.zeros(n, device=dev)
    acc = torch.empty(n, device=dev)
    deltas = [torch.randn(n, device=dev) * cfg["delta_std"] for _ in range(P)]
    w = gen.shard_weights(P, cfg["seed"])

    def step():
        for i in range(P):
            dp.dipaco_module_delta_accumulate(acc, None, deltas[i], float(w[i]), n, True, i == 0)
        dp.dipaco_module_outer_apply(theta, buf, acc, float(w.sum()), float(P) ** 0.5, n, cfg["outer_lr"],
                                     cfg["outer_momentum"])
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = _events(torch)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    bytes_ = (8.0 + (P - 1) * 12.0 + 20.0) * n     # first delta: read + write; others: 2 reads + write; apply: 3 reads + 2 writes
    ach = bytes_ / (ms * 1e-3) / 1e9
    return {"metric": "streaming module outer-step parameters/sec on 1 MI355X", "value": n / (ms * 1e-3),
            "unit": "params/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": "config 3 module, 16 weighted deltas accumulated one by one, sqrt(16) rescaling, Nesterov"},
            "roofline": {"bound": "hbm", "kernel": "delta_accumulate_kernel x16 + outer_apply_kernel", "achieved": ach,
                         "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS, "traffic": None,
                         "bytes_per_launch": bytes_ / (P + 1)}}


def bench_outer_table(args):
    """Outer step of a phase's modules in one launch: two shared level modules (config-3 size, 16 weighted deltas
    each, sqrt(16) rescaling) and 32 path-specific blocks (one path each, no averaging)."""
    import torch
    import dipaco_inputs as gen
    import paper_2403_10616_amd as dp
    cfg = gen.CONFIGS[3]
    n_shared, P = cfg["n_elems"], cfg["n_paths"]
    n_own = 9_645_440          # one transformer block at d_model 896 (4 d^2 + 2 d d_mlp + biases and gains)
    dev = "cuda"
    mods = []
    for m in range(2):
        mods.append(dict(theta=torch.randn(n_shared, device=dev) * 0.02, momentum=torch.zeros(n_shared, device=dev),
                         inputs=[torch.randn(n_shared, device=dev) * cfg["delta_std"] for _ in range(P)],
                         weights=gen.shard_weights(P, cfg["seed"] + m), n_elems=n_shared, is_delta=True,
                         norm_scale=float(P) ** 0.5))
    for m in range(32):
        th = torch.randn(n_own, device=dev) * 0.02
        mods.append(dict(theta=th, momentum=torch.zeros(n_own, device=dev), inputs=[th + 1e-3 * torch.randn(n_own, device=dev)],
                         weights=None, n_elems=n_own, is_delta=False, norm_scale=1.0))
    image = dp.dipaco_outer_table_pack(mods)
    table = torch.frombuffer(bytearray(image), dtype=torch.uint8).to(dev)

    def step():
        dp.dipaco_outer_step_table(image, table, cfg["outer_lr"], cfg["outer_momentum"])
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = _events(torch)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    n_total = 2 * n_shared + 32 * n_own
    bytes_ = 2 * n_shared * 4.0 * (P + 4) + 32 * n_own * 4.0 * (1 + 4)   # inputs + theta, momentum read and written
    ach = bytes_ / (ms * 1e-3) / 1e9
    return {"metric": "table-driven outer-step parameters/sec on 1 MI355X", "value": n_total / (ms * 1e-3),
            "unit": "params/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": "2 shared modules (58M, 16 weighted deltas, sqrt(16) rescaling) + 32 path-specific blocks "
                                   "(9.6M, one path) in one launch"},
            "roofline": {"bound": "hbm", "kernel": "outer_table_kernel", "achieved": ach, "peak": PEAK_HBM_GBS,
                         "unit": "GB/s", "frac": ach / PEAK_HBM_GBS, "traffic": None, "bytes_per_launch": bytes_}}


def bench_route(args):
    import torch
    import dipaco_inputs as gen
    import paper_2403_10616_amd as dp
    cfg = gen.CONFIGS[4]
    N, D, K = cfg["N"], cfg["D"], cfg["K"]
    dev = "cuda"
    z, c, _ = gen.gaussian_mixture(N, D, K, cfg["noise_std"], cfg["seed"])
    zd, cd = torch.from_numpy(z).to(dev), torch.from_numpy(c).to(dev)
    idx = torch.empty(N, dtype=torch.int32, device=dev)
    hist = torch.empty(K, dtype=torch.int64, device=dev)
    margin = torch.empty(N, dtype=torch.float32, device=dev)

    def step():
        dp.dipaco_route_prefix(zd, cd, N, D, K, idx, hist, margin)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = _events(torch)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = e0.elapsed_time(e1) / args.steps
    flops = 2.0 * N * D * K
    ach = flops / (ms * 1e-3) / 1e12
    out = {"metric": "prefix-routing documents/sec on 1 MI355X", "value": N / (wall / args.steps), "unit": "documents/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": "config 4: 1,048,576 x 768 embeddings from a 256-Gaussian mixture vs 256 centroids"},
           "roofline": {"bound": "mfma", "kernel": "route_kernel", "achieved": ach, "peak": PEAK_F32_TFLOPS,
                        "unit": "TFLOP/s", "frac": ach / PEAK_F32_TFLOPS, "traffic": None, "flops_per_launch": flops,
                        "hbm_gbs": (N * D * 4.0 + N * 8.0) / (ms * 1e-3) / 1e9}}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_route(cfg, z, c)
    return out


def bench_features(args):
    import torch
    import dipaco_inputs as gen
    import paper_2403_10616_amd as dp
    cfg = gen.CONFIGS[2]
    B, S = 8192, 32
    ctx = dp.Context(**_arch_kwargs(cfg, dp.BF16))
    n = dp.dipaco_path_param_count(ctx)
    dev = "cuda"
    lowp = (torch.randn(n, device=dev) * 0.02).to(torch.bfloat16)
    tok = torch.from_numpy(gen.zipf_tokens((B, S), cfg["vocab"], cfg["zipf_s"], 9).astype(np.int32)).to(dev)
    out = torch.empty((B, cfg["d_model"]), dtype=torch.float32, device=dev)
    ws = torch.empty(dp.dipaco_features_workspace_bytes(ctx, B, S), dtype=torch.uint8, device=dev)

    def step():
        dp.dipaco_path_prefix_features(ctx, None, lowp, tok, B, S, out, ws)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = _events(torch)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    d, A, F = cfg["d_model"], cfg["n_heads"] * cfg["d_head"], cfg["d_mlp"]
    NL = sum(cfg["layers_per_level"])
    flops = NL * (2.0 * B * S * (d * 3 * A + A * d + 2 * d * F) + B * cfg["n_heads"] * 2 * 2 * S * S * cfg["d_head"] / 2)
    ach = flops / (ms * 1e-3) / 1e12
    return {"metric": "router-feature documents/sec on 1 MI355X", "value": B / (ms * 1e-3), "unit": "documents/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "8192 prefixes of 32 Zipf(1.1) tokens through the 12 blocks of the config-2 path, mean pooled"},
            "roofline": {"bound": "mfma", "kernel": "gemm_dlds_kernel (forward layout) + attn_fwd_mfma", "achieved": ach,
                         "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "traffic": None,
                         "flops_per_launch": flops}}


def bench_score(args):
    import torch
    import dipaco_inputs as gen
    import paper_2403_10616_amd as dp
    cfg = gen.CONFIGS[5]
    B, S = cfg["batch"], cfg["seq"]
    ctx = dp.Context(**_arch_kwargs(cfg, dp.BF16))
    n = dp.dipaco_path_param_count(ctx)
    dev = "cuda"
    lowp = (torch.randn(n, device=dev) * 0.02).to(torch.bfloat16)
    seqs = gen.zipf_tokens((B, S + 1), cfg["vocab"], cfg["zipf_s"], cfg["seed"])
    tok = torch.from_numpy(np.ascontiguousarray(seqs[:, :-1]).astype(np.int32)).to(dev)
    tgt = torch.from_numpy(np.ascontiguousarray(seqs[:, 1:]).astype(np.int32)).to(dev)
    out = torch.empty(B, dtype=torch.float32, device=dev)
    ws = torch.empty(dp.dipaco_score_workspace_bytes(ctx, B, S), dtype=torch.uint8, device=dev)

    def step():
        dp.dipaco_path_score(ctx, None, lowp, tok, tgt, B, S, out, None, ws)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = _events(torch)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    fwd, _, _ = step_gemm_shapes(cfg, B, S)
    flops = sum(2.0 * M * N * K for M, N, K in fwd) + attention_flops(cfg, B, S)[0]
    ach = flops / (ms * 1e-3) / 1e12
    return {"metric": "path-scoring tokens/sec on 1 MI355X (forward only)", "value": B * S / (ms * 1e-3), "unit": "tokens/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "config-5 path (174.9M parameters), 16 documents x 2048 Zipf(1.1) tokens, forward + per-document log-likelihood"},
            "roofline": {"bound": "mfma", "kernel": "gemm_dlds_kernel (forward layout) + attn_fwd_mfma", "achieved": ach,
                         "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "traffic": None,
                         "flops_per_launch": flops}}


def bench_reroute(args):
    """Forward-only evaluation at seq 2048 with the path re-chosen every 128 tokens (Section 2.4.3): every document
    is scored under each of 4 paths, the window labels of the token-level router are formed, and the chunk-routed
    log-likelihood is read off with the labels standing in for the trained router's decisions."""
    import torch
    import dipaco_inputs as gen
    import paper_2403_10616_amd as dp
    cfg = gen.CONFIGS[5]
    B, S, P, W = cfg["batch"], cfg["seq"], 4, 128
    ctx = dp.Context(**_arch_kwargs(cfg, dp.BF16))
    n = dp.dipaco_path_param_count(ctx)
    dev = "cuda"
    paths = [(torch.randn(n, device=dev) * 0.02).to(torch.bfloat16) for _ in range(P)]
    seqs = gen.zipf_tokens((B, S + 1), cfg["vocab"], cfg["zipf_s"], cfg["seed"])
    tok = torch.from_numpy(np.ascontiguousarray(seqs[:, :-1]).astype(np.int32)).to(dev)
    tgt = torch.from_numpy(np.ascontiguousarray(seqs[:, 1:]).astype(np.int32)).to(dev)
    doc = torch.empty(B, dtype=torch.float32, device=dev)
    nll = torch.empty((P, B, S), dtype=torch.float32, device=dev)
    labels = torch.empty((B, S), dtype=torch.int32, device=dev)
    n_chunks = (S + W - 1) // W
    routed = torch.empty(B, dtype=torch.float32, device=dev)
    ws = torch.empty(dp.dipaco_score_workspace_bytes(ctx, B, S), dtype=torch.uint8, device=dev)
    rbytes = dp.dipaco_reroute_workspace_bytes(P, B, S)
    rws = torch.empty(rbytes, dtype=torch.uint8, device=dev)

    def step():
        for p in range(P):
            dp.dipaco_path_score(ctx, None, paths[p], tok, tgt, B, S, doc, nll[p], ws)
        dp.dipaco_window_targets(nll, P, B, S, S, labels, rws, rbytes)
        # chunk c + 1 takes the path decided at the last token of chunk c; the first chunk takes the document's label
        choice = torch.cat([labels[:, :1], labels[:, W - 1:S - 1:W]], dim=1).contiguous()
        dp.dipaco_chunk_routed_score(nll, choice, P, B, S, W, routed, rws, rbytes)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = _events(torch)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    fwd, _, _ = step_gemm_shapes(cfg, B, S)
    flops = P * (sum(2.0 * M * N * K for M, N, K in fwd) + attention_flops(cfg, B, S)[0])
    ach = flops / (ms * 1e-3) / 1e12
    single = max(float(-nll[p].sum().item()) for p in range(P))
    return {"metric": "re-routed evaluation tokens/sec on 1 MI355X (forward only, 4 paths)", "value": B * S / (ms * 1e-3),
            "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "config-5 architecture, 4 random-init paths, 16 documents x 2048 tokens, path re-chosen "
                                   "every 128 tokens from the window labels (L = rest of the document)",
                       "n_chunks": n_chunks, "routed_loglik": float(routed.sum().item()), "best_single_path_loglik": single},
            "roofline": {"bound": "mfma", "kernel": "gemm_dlds_kernel (forward layout) + attn_fwd_mfma", "achieved": ach,
                         "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "traffic": None,
                         "flops_per_launch": flops}}


def bench_kmeans(args):
    import torch
    import dipaco_inputs as gen
    import paper_2403_10616_amd as dp
    cfg = gen.CONFIGS[4]
    N, D, K = cfg["N"], cfg["D"], cfg["K"]
    dev = "cuda"
    z, c, _ = gen.gaussian_mixture(N, D, K, cfg["noise_std"], cfg["seed"])
    zd, cd = torch.from_numpy(z).to(dev), torch.from_numpy(c).to(dev)
    nb = args.n_best
    idx = torch.empty(N * nb, dtype=torch.int32, device=dev)
    hist = torch.empty(K, dtype=torch.int64, device=dev)
    counts = torch.empty(K, dtype=torch.int64, device=dev)
    ws = torch.empty(dp.dipaco_kmeans_workspace_bytes(N, D, K), dtype=torch.uint8, device=dev)
    idx1 = torch.empty(N, dtype=torch.int32, device=dev)
    dp.dipaco_route_prefix(zd, cd, N, D, K, idx1, hist, None)

    def assign():
        dp.dipaco_route_prefix_top(zd, D, cd, N, D, K, nb, idx, hist, None)

    def update():
        dp.dipaco_kmeans_update(zd, D, idx1, N, D, K, cd, counts, ws)
    times = {}
    for name, fn in (("assign", assign), ("update", update)):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = _events(torch)
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        times[name] = e0.elapsed_time(e1) / args.steps
    ms = times["assign"] + times["update"]
    upd_bytes = N * D * 4.0 + N * 4.0 * 4 + K * D * 4.0   # the points once; cluster ids read three times, order written
    ach = upd_bytes / (times["update"] * 1e-3) / 1e9
    return {"metric": "k-means iteration documents/sec on 1 MI355X", "value": N / (ms * 1e-3), "unit": "documents/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": f"config 4 data: 1,048,576 x 768 embeddings, 256 centroids; top-{nb} assignment "
                                   "+ centroid update", "assign_ms": times["assign"], "update_ms": times["update"],
                       "assign_tflops": 2.0 * N * D * K / (times["assign"] * 1e-3) / 1e12},
            "roofline": {"bound": "hbm", "kernel": "kmeans_partial_kernel (+ stable sort, finish)", "achieved": ach,
                         "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS, "traffic": None,
                         "bytes_per_launch": upd_bytes}}


def bench_router(args):
    """Discriminative router on the config-4 data: one evaluation of the K-class logistic loss with its gradients
    (what one optimiser step costs), and the trained router used for routing."""
    import torch
    import dipaco_inputs as gen
    import paper_2403_10616_amd as dp
    cfg = gen.CONFIGS[4]
    N, D, K = cfg["N"], cfg["D"], cfg["K"]
    dev = "cuda"
    z, c, comp = gen.gaussian_mixture(N, D, K, cfg["noise_std"], cfg["seed"])
    zd = torch.from_numpy(z).to(dev)
    W = torch.from_numpy(c).to(dev).contiguous()             # a router near the generating centres
    b = torch.zeros(K, dtype=torch.float32, device=dev)
    labels = torch.from_numpy(comp.astype("int32")).to(dev)
    nbytes = dp.dipaco_router_workspace_bytes(N, D, K)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    loss = torch.zeros(4, dtype=torch.float32, device=dev)
    dW = torch.empty((K, D), dtype=torch.float32, device=dev)
    db = torch.empty(K, dtype=torch.float32, device=dev)
    idx = torch.empty(N, dtype=torch.int32, device=dev)
    hist = torch.empty(K, dtype=torch.int64, device=dev)

    def grad():
        dp.dipaco_router_logistic_grad(zd, labels, W, b, N, D, K, loss, dW, db, ws, nbytes)

    def route():
        dp.dipaco_route_linear(zd, D, W, b, N, D, K, idx, hist, None)
    times = {}
    for name, fn in (("grad", grad), ("route", route)):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = _events(torch)
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        times[name] = e0.elapsed_time(e1) / args.steps
    ms = times["grad"]
    flops = 4.0 * N * D * K                                  # logits and weight gradient
    ach = flops / (ms * 1e-3) / 1e12
    return {"metric": "router logistic loss+gradient documents/sec on 1 MI355X", "value": N / (ms * 1e-3),
            "unit": "documents/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": "config 4 data: 1,048,576 x 768 features, 256 paths; logistic loss + dW + db",
                       "route_linear_ms": times["route"],
                       "route_linear_tflops": 2.0 * N * D * K / (times["route"] * 1e-3) / 1e12,
                       "loss": float(loss[0].item())},
            "roofline": {"bound": "mfma", "kernel": "gemm_kernel<float> (logits, weight gradient) + logistic_rows_kernel",
                         "achieved": ach, "peak": PEAK_F32_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_F32_TFLOPS,
                         "traffic": None}}


def bench_gemm(args):
    import torch
    import paper_2403_10616_amd as dp
    M, N, K = (int(x) for x in args.mnk.split(","))
    dev = "cuda"
    ta, tb = args.layout[0] == "t", args.layout[1] == "t"
    out_f32 = args.layout == "tn"
    a = torch.empty(M * K, dtype=torch.bfloat16, device=dev).normal_()
    b = torch.empty(K * N, dtype=torch.bfloat16, device=dev).normal_(std=0.02)
    if args.operands == "zeros":   # no bit toggles in the matrix cores: the clock the chip holds is higher
        a.zero_()
        b.zero_()
    c = torch.empty(M * N, dtype=torch.float32 if out_f32 else torch.bfloat16, device=dev)
    ep = args.epilogue
    bias = torch.zeros(N, dtype=torch.bfloat16, device=dev) if ep in ("bias", "gelu", "resid") else None
    resid = torch.empty(M * N, dtype=torch.bfloat16, device=dev).normal_() if ep == "resid" else None
    aux_out = torch.empty(M * N, dtype=torch.bfloat16, device=dev) if ep == "gelu" else None
    aux_in = torch.empty(M * N, dtype=torch.bfloat16, device=dev).normal_() if ep == "dgelu" else None
    act = {"gelu": 3, "dgelu": 4}.get(ep, 0)   # the pair the path step uses: GELU' saved in forward, multiplied in backward
    splits, partial = 1, None
    if out_f32 and args.splits > 1:
        splits = args.splits
        partial = torch.empty(splits * M * N, dtype=torch.float32, device=dev)

    if args.gemm_tile:
        dp.dipaco_k_set_gemm_tile(args.gemm_tile)

    def step():
        dp.dipaco_k_gemm(dp.BF16, ta, tb, out_f32, M, N, K, a, b, c, bias, resid, aux_out, aux_in, act, splits, partial)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = _events(torch)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    flops = 2.0 * M * N * K
    ach = flops / (ms * 1e-3) / 1e12
    library = None
    if args.library_reference and not out_f32 and ep == "none":
        # context, not a target: the vendor library's product of the same operands on the same box (no epilogue)
        a2 = a.view(K, M).t() if ta else a.view(M, K)
        b2 = b.view(N, K).t() if tb else b.view(K, N)
        for _ in range(args.warmup):
            torch.matmul(a2, b2)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            torch.matmul(a2, b2)
        e1.record()
        torch.cuda.synchronize()
        lib_ms = e0.elapsed_time(e1) / args.steps
        library = {"ms": lib_ms, "tflops": flops / (lib_ms * 1e-3) / 1e12, "what": "torch.matmul (vendor GEMM library)"}
    return {"metric": "GEMM TFLOP/s on 1 MI355X", "value": ach, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16", "data": "synthetic",
            "config": {"workload": f"gemm {args.layout} M={M} N={N} K={K} epilogue={ep} splits={splits} operands={args.operands}",
                       "library_reference": library},
            "roofline": {"bound": "mfma", "kernel": "gemm_kernel", "achieved": ach, "peak": PEAK_BF16_TFLOPS,
                         "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "traffic": None, "flops_per_launch": flops}}


def bench_issue_probe(args):
    """How matrix-core and vector-ALU instructions share a SIMD: register-only loops (dipaco_k_issue_probe) at one to
    four waves per SIMD.  'value' is the time of mode 2 (16 MFMA then 256 FMA) over the sum of modes 0 and 1 at four waves
    per SIMD: 1 = the two kinds of work do not overlap at all, 0.5 = they overlap completely."""
    import torch
    import paper_2403_10616_amd as dp
    dev = "cuda"
    out = torch.empty(256 * 1024, dtype=torch.float32, device=dev)
    iters = 20000
    names = ["16 MFMA", "256 FMA", "16 MFMA then 256 FMA", "16 x (1 MFMA, 16 FMA)", "256 x (exp2, mul, add)"]
    table = {}
    e0, e1 = _events(torch)
    for waves in (1, 2, 3, 4):
        for mode in range(5):
            dp.dipaco_k_issue_probe(mode, waves, 100, out)
            torch.cuda.synchronize()
            e0.record()
            dp.dipaco_k_issue_probe(mode, waves, iters, out)
            e1.record()
            torch.cuda.synchronize()
            table[f"{waves} waves/SIMD: {names[mode]}"] = round(e0.elapsed_time(e1) * 1e6 / iters, 1)
    # the two bf16 matrix-core shapes at the chip's power limit (two waves per SIMD, 60000 iterations = some 30 ms each)
    shapes = {}
    for mode, name in ((5, "32x32x16 zeros"), (7, "16x16x32 zeros"), (6, "32x32x16 random"), (8, "16x16x32 random")):
        dp.dipaco_k_issue_probe(mode, 2, 2000, out)
        torch.cuda.synchronize()
        e0.record()
        dp.dipaco_k_issue_probe(mode, 2, 60000, out)
        e1.record()
        torch.cuda.synchronize()
        shapes[name] = round(256 * 8 * 60000 * 524288.0 / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    ratio = table["4 waves/SIMD: 16 MFMA then 256 FMA"] / (table["4 waves/SIMD: 16 MFMA"] + table["4 waves/SIMD: 256 FMA"])
    return {"metric": "time of (16 MFMA then 256 FMA) over the sum of the two alone, 4 waves per SIMD", "value": ratio,
            "unit": "ratio", "n_gpus": 1, "steps": iters, "warmup": 100, "ms_per_step": None, "higher_is_better": False,
            "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "instruction-issue probe: one workgroup per compute unit, no memory traffic",
                       "ns_per_iteration": table, "mfma_shape_tflops": shapes}}


def bench_attention(args):
    import torch
    import dipaco_inputs as gen
    import paper_2403_10616_amd as dp
    cfg = gen.CONFIGS[2]
    B, S, H, dh = cfg["batch"], args.seq or cfg["seq"], cfg["n_heads"], cfg["d_head"]
    if args.seq:
        B = max(1, B * cfg["seq"] // S)
    if args.batch:
        B = args.batch
    dev = "cuda"
    A = H * dh
    qkv = torch.empty(B * S * 3 * A, dtype=torch.bfloat16, device=dev).normal_()
    o = torch.empty(B * S * A, dtype=torch.bfloat16, device=dev)
    d_o = torch.empty(B * S * A, dtype=torch.bfloat16, device=dev).normal_()
    if args.operands == "zeros":          # the same launches on all-zero inputs: what the chip's power limit costs
        qkv.zero_()
        d_o.zero_()
    dqkv = torch.empty(B * S * 3 * A, dtype=torch.bfloat16, device=dev)
    lse = torch.empty(B * H * S, dtype=torch.float32, device=dev)
    dsum = torch.empty(2 * B * H * ((S + 127) // 128 * 128), dtype=torch.float32, device=dev)
    dp.dipaco_k_attention_fwd(dp.BF16, qkv, o, lse, B, S, H, dh)
    bwd = getattr(args, "pass") == "bwd"

    def step():
        if bwd:
            dp.dipaco_k_attention_bwd(dp.BF16, qkv, o, d_o, lse, dqkv, dsum, B, S, H, dh)
        else:
            dp.dipaco_k_attention_fwd(dp.BF16, qkv, o, lse, B, S, H, dh)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = _events(torch)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    flops = B * H * (2 * 2 * S * S * dh) / 2 * (2.5 if bwd else 1.0)   # causal half; backward = five matmuls
    ach = flops / (ms * 1e-3) / 1e12
    return {"metric": "causal attention TFLOP/s on 1 MI355X", "value": ach, "unit": "TFLOP/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": f"attention {'backward' if bwd else 'forward'} B={B} H={H} S={S} d_head={dh}"},
            "roofline": {"bound": "mfma", "kernel": "attn_bwd_*_mfma" if bwd else "attn_fwd_mfma", "achieved": ach,
                         "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "traffic": None,
                         "flops_per_launch": flops}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="path_step", choices=["path_step", "round", "outer_step", "outer_stream", "outer_table", "route", "router", "reroute", "kmeans", "features", "score", "gemm", "attention", "issue_probe"])
    ap.add_argument("--n-best", type=int, default=1, choices=[1, 2])
    ap.add_argument("--mnk", default="32768,3584,896")
    ap.add_argument("--layout", default="nn", choices=["nn", "nt", "tn"])
    ap.add_argument("--epilogue", default="none", choices=["none", "bias", "gelu", "dgelu", "resid"])
    ap.add_argument("--operands", default="normal", choices=["normal", "zeros"])
    ap.add_argument("--library-reference", action="store_true",
                    help="gemm workload, no epilogue, bf16 output: also time torch.matmul on the same operands (context)")
    ap.add_argument("--splits", type=int, default=1)
    ap.add_argument("--gemm-tile", type=int, default=0, help="gemm / path_step workloads: force a tile shape (dipaco_k_set_gemm_tile)")
    ap.add_argument("--pass", default="fwd", choices=["fwd", "bwd"])
    ap.add_argument("--attn-blocks", type=int, default=None, choices=[0, 1],
                    help="attention workload: 0 = a long and a short causal block per workgroup, 1 = one block, longest first")
    ap.add_argument("--seq", type=int, default=0)
    ap.add_argument("--batch", type=int, default=0, help="attention workload: sequences (default: the config's token count / seq)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs one path on ONE GPU (no collectives, no sharding); use --gpus 1")
    import paper_2403_10616_amd as dp
    dp.load()   # fails loudly if libdipaco.so is not built
    if args.attn_blocks is not None:
        dp.dipaco_k_set_attention_blocks(args.attn_blocks)
    fn = {"path_step": bench_path_step, "round": bench_round, "outer_step": bench_outer_step, "route": bench_route, "gemm": bench_gemm, "kmeans": bench_kmeans, "features": bench_features, "score": bench_score, "outer_stream": bench_outer_stream,
          "outer_table": bench_outer_table, "router": bench_router, "reroute": bench_reroute,
          "attention": bench_attention, "issue_probe": bench_issue_probe}[args.workload]
    print(json.dumps(fn(args)))


if __name__ == "__main__":
    main()
