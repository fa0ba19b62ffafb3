"""Python binding of libdipaco.so (ctypes): argument marshalling only.

Every function has the name and argument order of its C entry point in include/dipaco.h /
include/dipaco_kernels.h.  Tensors are torch CUDA(HIP) tensors used purely as device memory; the stream is
torch's current stream unless one is given.  Nothing here computes: if the shared library is missing or a
call fails, a DipacoError is raised — there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdipaco.so")
F32, BF16 = 0, 1
MAX_PATHS_PER_MODULE = 256

_lib = None


class DipacoError(RuntimeError):
    pass


class _Arch(C.Structure):
    _fields_ = [("n_levels", C.c_int32), ("layers_per_level", C.POINTER(C.c_int32)),
                ("d_model", C.c_int32), ("n_heads", C.c_int32), ("d_head", C.c_int32), ("d_mlp", C.c_int32),
                ("vocab", C.c_int32), ("max_seq", C.c_int32), ("ln_eps", C.c_float), ("compute", C.c_int32)]


class _ModuleDesc(C.Structure):
    _fields_ = [("theta", C.c_void_p), ("momentum", C.c_void_p), ("inputs", C.POINTER(C.c_void_p)),
                ("weights", C.POINTER(C.c_float)), ("n_elems", C.c_uint64), ("n_paths", C.c_int32),
                ("is_delta", C.c_int32), ("norm_scale", C.c_float)]


_SIGS = {
    "dipaco_create": (C.c_int, [C.POINTER(C.c_void_p), C.POINTER(_Arch)]),
    "dipaco_destroy": (None, [C.c_void_p]),
    "dipaco_last_error": (C.c_char_p, []),
    "dipaco_path_param_count": (C.c_size_t, [C.c_void_p]),
    "dipaco_segment_count": (C.c_int32, [C.c_void_p]),
    "dipaco_segment_offset": (C.c_size_t, [C.c_void_p, C.c_int32]),
    "dipaco_segment_size": (C.c_size_t, [C.c_void_p, C.c_int32]),
    "dipaco_tensor_count": (C.c_int32, [C.c_void_p]),
    "dipaco_tensor_info": (C.c_int, [C.c_void_p, C.c_int32, C.c_char_p, C.c_size_t, C.POINTER(C.c_size_t),
                                     C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int32)]),
    "dipaco_path_index": (C.c_int64, [C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int32]),
    "dipaco_path_modules": (C.c_int, [C.c_int64, C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_int32)]),
    "dipaco_workspace_bytes": (C.c_size_t, [C.c_void_p, C.c_int32, C.c_int32]),
    "dipaco_compose_path": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p), C.c_void_p, C.c_void_p, C.c_void_p]),
    "dipaco_path_fwd_bwd": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "dipaco_features_workspace_bytes": (C.c_size_t, [C.c_void_p, C.c_int32, C.c_int32]),
    "dipaco_path_prefix_features": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                              C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "dipaco_static_scratch_bytes": (C.c_size_t, []),
    "dipaco_path_prefix_features_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                                     C.c_int32, C.c_void_p, C.c_void_p]),
    "dipaco_score_workspace_bytes": (C.c_size_t, [C.c_void_p, C.c_int32, C.c_int32]),
    "dipaco_path_score": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "dipaco_inner_adamw": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                     C.c_float, C.c_float, C.c_float, C.c_float, C.c_float, C.c_void_p]),
    "dipaco_module_outer_step": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_float),
                                           C.c_int32, C.c_size_t, C.c_int32, C.c_float, C.c_float, C.c_void_p]),
    "dipaco_module_delta_accumulate": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_size_t, C.c_int32,
                                                 C.c_int32, C.c_void_p]),
    "dipaco_module_outer_apply": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_double, C.c_float, C.c_size_t,
                                            C.c_float, C.c_float, C.c_void_p]),
    "dipaco_outer_table_bytes": (C.c_size_t, [C.POINTER(_ModuleDesc), C.c_int32]),
    "dipaco_outer_table_pack": (C.c_int, [C.POINTER(_ModuleDesc), C.c_int32, C.c_void_p, C.c_size_t]),
    "dipaco_outer_step_table": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_float, C.c_float, C.c_void_p]),
    "dipaco_route_prefix": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p]),
    "dipaco_route_prefix_top": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                          C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "dipaco_reroute_workspace_bytes": (C.c_size_t, [C.c_int32, C.c_int32, C.c_int32]),
    "dipaco_window_targets": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                        C.c_size_t, C.c_void_p]),
    "dipaco_chunk_routed_score": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                            C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "dipaco_route_linear": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "dipaco_router_workspace_bytes": (C.c_size_t, [C.c_int64, C.c_int32, C.c_int32]),
    "dipaco_router_logistic_grad": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
                                              C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                              C.c_void_p]),
    "dipaco_kmeans_workspace_bytes": (C.c_size_t, [C.c_int64, C.c_int32, C.c_int32]),
    "dipaco_kmeans_update": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "dipaco_k_gemm": (C.c_int, [C.c_int32] * 7 + [C.c_void_p] * 7 + [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]),
    "dipaco_k_gemm_colsum": (C.c_int, [C.c_int32] * 6 + [C.c_void_p] * 7 + [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "dipaco_k_set_gemm_tile": (C.c_int, [C.c_int32]),
    "dipaco_k_gemm_split_plan": (C.c_int, [C.c_int32] * 4 + [C.POINTER(C.c_int32)]),
    "dipaco_k_set_attention_blocks": (C.c_int, [C.c_int32]),
    "dipaco_k_issue_probe": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]),
    "dipaco_k_attention_fwd": (C.c_int, [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                         C.c_int32, C.c_void_p]),
    "dipaco_k_attention_bwd": (C.c_int, [C.c_int32] + [C.c_void_p] * 8 + [C.c_int32] * 4 + [C.c_void_p]),
}

EXPORTS = tuple(_SIGS)


def load():
    """Load libdipaco.so (built by `python -m paper_2403_10616_amd.build`); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise DipacoError(f"{LIB_PATH} is not built: run `python -m paper_2403_10616_amd.build`")
        # torch ships its own HIP runtime; load it first so that libdipaco binds to the same libamdhip64 (one
        # runtime per process: streams and device pointers are only valid inside the runtime that made them)
        import torch  # noqa: F401
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(lib, name)      # AttributeError if the library lacks a declared symbol
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _check(status: int):
    if status != 0:
        raise DipacoError(f"libdipaco status {status}: {load().dipaco_last_error().decode()}")


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):   # a raw device address
        return t
    if not t.is_cuda or not t.is_contiguous():
        raise DipacoError("expected a contiguous device tensor")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def last_error() -> str:
    return load().dipaco_last_error().decode()


class Context:
    """Owns a dipaco_ctx*."""

    def __init__(self, layers_per_level: Sequence[int], d_model: int, n_heads: int, d_head: int, d_mlp: int,
                 vocab: int, max_seq: int, ln_eps: float = 1e-5, compute: int = F32):
        lib = load()
        self._levels = (C.c_int32 * len(layers_per_level))(*layers_per_level)
        arch = _Arch(len(layers_per_level), self._levels, d_model, n_heads, d_head, d_mlp, vocab, max_seq, ln_eps,
                     compute)
        self.handle = C.c_void_p()
        _check(lib.dipaco_create(C.byref(self.handle), C.byref(arch)))
        self.compute = compute

    def close(self):
        if getattr(self, "handle", None):
            load().dipaco_destroy(self.handle)
            self.handle = None

    __del__ = close


def dipaco_create(**kw) -> Context:
    return Context(**kw)


def dipaco_path_param_count(ctx: Context) -> int:
    return load().dipaco_path_param_count(ctx.handle)


def dipaco_segment_count(ctx: Context) -> int:
    return load().dipaco_segment_count(ctx.handle)


def dipaco_segment_offset(ctx: Context, segment: int) -> int:
    return load().dipaco_segment_offset(ctx.handle, segment)


def dipaco_segment_size(ctx: Context, segment: int) -> int:
    return load().dipaco_segment_size(ctx.handle, segment)


def dipaco_tensor_count(ctx: Context) -> int:
    return load().dipaco_tensor_count(ctx.handle)


def dipaco_tensor_info(ctx: Context, i: int):
    """(name, offset, rows, cols, decayed)"""
    name = C.create_string_buffer(64)
    off, rows, cols, dec = C.c_size_t(), C.c_int64(), C.c_int64(), C.c_int32()
    _check(load().dipaco_tensor_info(ctx.handle, i, name, 64, C.byref(off), C.byref(rows), C.byref(cols), C.byref(dec)))
    return name.value.decode(), off.value, rows.value, cols.value, bool(dec.value)


def dipaco_path_index(modules: Sequence[int], K: Sequence[int]) -> int:
    L = len(K)
    return load().dipaco_path_index((C.c_int32 * L)(*modules), (C.c_int32 * L)(*K), L)


def dipaco_path_modules(j: int, K: Sequence[int]):
    L = len(K)
    out = (C.c_int32 * L)()
    _check(load().dipaco_path_modules(j, (C.c_int32 * L)(*K), L, out))
    return tuple(out)


def dipaco_workspace_bytes(ctx: Context, batch: int, seq: int) -> int:
    return load().dipaco_workspace_bytes(ctx.handle, batch, seq)


def dipaco_compose_path(ctx: Context, segments, path_master, path_lowp=None, stream=None):
    n = len(segments)
    ptrs = (C.c_void_p * n)(*[_ptr(s) for s in segments])
    _check(load().dipaco_compose_path(ctx.handle, ptrs, _ptr(path_master), _ptr(path_lowp), _stream(stream)))


def dipaco_path_fwd_bwd(ctx: Context, path_master, path_lowp, tokens, targets, batch: int, seq: int, loss_out,
                        token_nll_out, grads, workspace, stream=None):
    _check(load().dipaco_path_fwd_bwd(ctx.handle, _ptr(path_master), _ptr(path_lowp), _ptr(tokens), _ptr(targets), batch,
                                      seq, _ptr(loss_out), _ptr(token_nll_out), _ptr(grads), _ptr(workspace),
                                      workspace.numel() * workspace.element_size(), _stream(stream)))


def dipaco_features_workspace_bytes(ctx: Context, batch: int, seq: int) -> int:
    return load().dipaco_features_workspace_bytes(ctx.handle, batch, seq)


def dipaco_path_prefix_features(ctx: Context, path_master, path_lowp, tokens, batch: int, seq: int, features_out,
                                workspace, stream=None):
    _check(load().dipaco_path_prefix_features(ctx.handle, _ptr(path_master), _ptr(path_lowp), _ptr(tokens), batch, seq,
                                              _ptr(features_out), _ptr(workspace),
                                              workspace.numel() * workspace.element_size(), _stream(stream)))


def dipaco_static_scratch_bytes() -> int:
    return load().dipaco_static_scratch_bytes()


def dipaco_path_prefix_features_static(ctx: Context, path_master, path_lowp, tokens, batch: int, seq: int, features_out,
                                       stream=None):
    _check(load().dipaco_path_prefix_features_static(ctx.handle, _ptr(path_master), _ptr(path_lowp), _ptr(tokens), batch,
                                                     seq, _ptr(features_out), _stream(stream)))


def dipaco_score_workspace_bytes(ctx: Context, batch: int, seq: int) -> int:
    return load().dipaco_score_workspace_bytes(ctx.handle, batch, seq)


def dipaco_path_score(ctx: Context, path_master, path_lowp, tokens, targets, batch: int, seq: int, doc_loglik_out,
                      token_nll_out, workspace, stream=None):
    _check(load().dipaco_path_score(ctx.handle, _ptr(path_master), _ptr(path_lowp), _ptr(tokens), _ptr(targets), batch,
                                    seq, _ptr(doc_loglik_out), _ptr(token_nll_out), _ptr(workspace),
                                    workspace.numel() * workspace.element_size(), _stream(stream)))


def dipaco_inner_adamw(ctx: Context, path_master, grads, m, v, path_lowp, step: int, lr: float, beta1: float,
                       beta2: float, eps: float, weight_decay: float, stream=None):
    _check(load().dipaco_inner_adamw(ctx.handle, _ptr(path_master), _ptr(grads), _ptr(m), _ptr(v), _ptr(path_lowp), step,
                                     lr, beta1, beta2, eps, weight_decay, _stream(stream)))


def dipaco_module_outer_step(theta, momentum, inputs, weights, n_elems: int, is_delta: bool, outer_lr: float,
                             outer_momentum: float, stream=None):
    n = len(inputs)
    ptrs = (C.c_void_p * n)(*[_ptr(t) for t in inputs])
    w = None if weights is None else (C.c_float * n)(*[float(x) for x in weights])
    _check(load().dipaco_module_outer_step(_ptr(theta), _ptr(momentum), ptrs, w, n, n_elems, int(bool(is_delta)),
                                           outer_lr, outer_momentum, _stream(stream)))


def dipaco_module_delta_accumulate(delta_sum, theta_prev, inp, weight: float, n_elems: int, is_delta: bool, first: bool,
                                   stream=None):
    _check(load().dipaco_module_delta_accumulate(_ptr(delta_sum), _ptr(theta_prev), _ptr(inp), weight, n_elems,
                                                 int(bool(is_delta)), int(bool(first)), _stream(stream)))


def dipaco_module_outer_apply(theta, momentum, delta_sum, weight_sum: float, norm_scale: float, n_elems: int,
                              outer_lr: float, outer_momentum: float, stream=None):
    _check(load().dipaco_module_outer_apply(_ptr(theta), _ptr(momentum), _ptr(delta_sum), weight_sum, norm_scale, n_elems,
                                            outer_lr, outer_momentum, _stream(stream)))


def dipaco_reroute_workspace_bytes(n_paths: int, batch: int, seq: int) -> int:
    return int(load().dipaco_reroute_workspace_bytes(n_paths, batch, seq))


def dipaco_window_targets(token_nll, n_paths: int, batch: int, seq: int, window: int, targets_out, workspace,
                          workspace_bytes: int, stream=None):
    _check(load().dipaco_window_targets(_ptr(token_nll), n_paths, batch, seq, window, _ptr(targets_out), _ptr(workspace),
                                        workspace_bytes, _stream(stream)))


def dipaco_chunk_routed_score(token_nll, chunk_path, n_paths: int, batch: int, seq: int, chunk: int, doc_loglik_out,
                              workspace, workspace_bytes: int, stream=None):
    _check(load().dipaco_chunk_routed_score(_ptr(token_nll), _ptr(chunk_path), n_paths, batch, seq, chunk,
                                            _ptr(doc_loglik_out), _ptr(workspace), workspace_bytes, _stream(stream)))


def dipaco_route_linear(z, ldz: int, weights, bias, N: int, D: int, K: int, idx_out, hist_out, margin_out=None,
                        stream=None, z_offset: int = 0):
    _check(load().dipaco_route_linear(_ptr_at(z, z_offset), ldz, _ptr(weights), _ptr(bias), N, D, K, _ptr(idx_out),
                                      _ptr(hist_out), _ptr(margin_out), _stream(stream)))


def dipaco_router_workspace_bytes(N: int, D: int, K: int) -> int:
    return int(load().dipaco_router_workspace_bytes(N, D, K))


def dipaco_router_logistic_grad(z, labels, weights, bias, N: int, D: int, K: int, loss_out, dweights_out, dbias_out,
                                workspace, workspace_bytes: int, stream=None):
    _check(load().dipaco_router_logistic_grad(_ptr(z), _ptr(labels), _ptr(weights), _ptr(bias), N, D, K, _ptr(loss_out),
                                              _ptr(dweights_out), _ptr(dbias_out), _ptr(workspace), workspace_bytes,
                                              _stream(stream)))


def _module_descs(modules):
    """ctypes array of dipaco_module_desc from dicts with keys theta, momentum, inputs (device tensors or integer
    addresses), weights (floats or None), n_elems, is_delta, norm_scale; also returns the objects it points into"""
    descs = (_ModuleDesc * len(modules))()
    keep = []
    for d, m in zip(descs, modules):
        n = len(m["inputs"])
        ptrs = (C.c_void_p * n)(*[_ptr(t) for t in m["inputs"]])
        w = None if m.get("weights") is None else (C.c_float * len(m["weights"]))(*[float(x) for x in m["weights"]])
        keep += [ptrs, w]
        d.theta, d.momentum = _ptr(m["theta"]), _ptr(m["momentum"])
        d.inputs = C.cast(ptrs, C.POINTER(C.c_void_p))
        d.weights = C.cast(w, C.POINTER(C.c_float)) if w is not None else None
        d.n_elems, d.n_paths = int(m["n_elems"]), n
        d.is_delta, d.norm_scale = int(bool(m["is_delta"])), float(m.get("norm_scale", 1.0))
    return descs, keep


def dipaco_outer_table_bytes(modules) -> int:
    descs, _keep = _module_descs(modules)
    return int(load().dipaco_outer_table_bytes(descs, len(modules)))


def dipaco_outer_table_pack(modules) -> bytes:
    """the table image, in host memory; copy it to the device and pass both to dipaco_outer_step_table"""
    descs, _keep = _module_descs(modules)
    need = int(load().dipaco_outer_table_bytes(descs, len(modules)))
    image = C.create_string_buffer(max(need, 1))
    _check(load().dipaco_outer_table_pack(descs, len(modules), image, need))
    return image.raw[:need]


def dipaco_outer_step_table(table_host: bytes, table_device, outer_lr: float, outer_momentum: float, stream=None):
    _check(load().dipaco_outer_step_table(table_host, _ptr(table_device), len(table_host), outer_lr, outer_momentum,
                                          _stream(stream)))


def dipaco_route_prefix(z, centroids, N: int, D: int, K: int, idx_out, hist_out, margin_out=None, stream=None):
    _check(load().dipaco_route_prefix(_ptr(z), _ptr(centroids), N, D, K, _ptr(idx_out), _ptr(hist_out),
                                      _ptr(margin_out), _stream(stream)))


def _ptr_at(t, offset_elems: int = 0) -> Optional[int]:
    """data pointer of a device tensor plus an element offset (a view's storage need not be contiguous)"""
    if t is None:
        return None
    if not t.is_cuda:
        raise DipacoError("expected a device tensor")
    return t.data_ptr() + offset_elems * t.element_size()


def dipaco_route_prefix_top(z, ldz: int, centroids, N: int, D: int, K: int, n_best: int, idx_out, hist_out,
                            margin_out=None, stream=None, z_offset: int = 0):
    """z: device tensor holding the feature matrix; row n starts z_offset + n * ldz elements into it"""
    _check(load().dipaco_route_prefix_top(_ptr_at(z, z_offset), ldz, _ptr(centroids), N, D, K, n_best, _ptr(idx_out),
                                          _ptr(hist_out), _ptr(margin_out), _stream(stream)))


def dipaco_kmeans_workspace_bytes(N: int, D: int, K: int) -> int:
    return load().dipaco_kmeans_workspace_bytes(N, D, K)


def dipaco_kmeans_update(z, ldz: int, idx, N: int, D: int, K: int, centroids, counts_out, workspace, stream=None,
                         z_offset: int = 0):
    _check(load().dipaco_kmeans_update(_ptr_at(z, z_offset), ldz, _ptr(idx), N, D, K, _ptr(centroids), _ptr(counts_out),
                                       _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


# ---- kernel-level entry points ---------------------------------------------------------------------------
def dipaco_k_gemm(dtype: int, trans_a: bool, trans_b: bool, out_f32: bool, M: int, N: int, K: int, A, B, Cout,
                  bias=None, resid=None, aux_out=None, aux_in=None, act: int = 0, splits: int = 1, partial=None,
                  stream=None):
    _check(load().dipaco_k_gemm(dtype, int(trans_a), int(trans_b), int(out_f32), M, N, K, _ptr(A), _ptr(B), _ptr(Cout),
                                _ptr(bias), _ptr(resid), _ptr(aux_out), _ptr(aux_in), act, splits, _ptr(partial),
                                _stream(stream)))


def dipaco_k_gemm_colsum(dtype: int, trans_a: bool, trans_b: bool, M: int, N: int, K: int, A, B, Cout, bias, resid,
                         aux_out, aux_in, act: int, colsum_out, colsum_scratch, stream=None):
    _check(load().dipaco_k_gemm_colsum(dtype, int(trans_a), int(trans_b), M, N, K, _ptr(A), _ptr(B), _ptr(Cout),
                                       _ptr(bias), _ptr(resid), _ptr(aux_out), _ptr(aux_in), act, _ptr(colsum_out),
                                       _ptr(colsum_scratch), _stream(stream)))


def dipaco_k_set_gemm_tile(tile: int):
    _check(load().dipaco_k_set_gemm_tile(tile))


def dipaco_k_gemm_split_plan(M: int, N: int, K: int, max_slices: int) -> dict:
    out = (C.c_int32 * 12)()
    _check(load().dipaco_k_gemm_split_plan(M, N, K, max_slices, out))
    v = list(out)
    return {"tile": (v[0], v[1]), "inside": (v[2], v[3]), "tiles": v[4:8], "slices": v[8:12]}


def dipaco_k_issue_probe(mode: int, waves_per_simd: int, iters: int, out, stream=None):
    _check(load().dipaco_k_issue_probe(mode, waves_per_simd, iters, _ptr(out), _stream(stream)))


def dipaco_k_set_attention_blocks(single_block: int):
    _check(load().dipaco_k_set_attention_blocks(int(single_block)))


def dipaco_k_attention_fwd(dtype: int, qkv, o, lse, B: int, S: int, H: int, dh: int, stream=None):
    _check(load().dipaco_k_attention_fwd(dtype, _ptr(qkv), _ptr(o), _ptr(lse), B, S, H, dh, _stream(stream)))


def dipaco_k_attention_bwd(dtype: int, qkv, o, d_o, lse, dqkv, dsum, B: int, S: int, H: int, dh: int, stream=None,
                           colsum_out=None, colsum_scratch=None):
    _check(load().dipaco_k_attention_bwd(dtype, _ptr(qkv), _ptr(o), _ptr(d_o), _ptr(lse), _ptr(dqkv), _ptr(dsum),
                                         _ptr(colsum_out), _ptr(colsum_scratch), B, S, H, dh, _stream(stream)))
