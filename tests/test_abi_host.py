"""CPU-only checks of the C-ABI library: it loads, exports every symbol the headers declare, and its host-side
logic (layout, path indexing, argument validation) agrees with the oracle's independent statement of the same."""
import ctypes
import os
import re

import numpy as np
import pytest

import dipaco_inputs as gen
import paper_2403_10616_amd as dp
from oracle import dipaco_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    for h in ("dipaco.h", "dipaco_kernels.h"):
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(dipaco_[a-z0-9_]+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(dp.LIB_PATH)
    declared = _declared_symbols()
    assert len(declared) >= 20
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(dp.EXPORTS)      # the binding covers exactly the declared entry points


@pytest.mark.parametrize("cfg_id", [1, 2, 5])
def test_layout_matches_oracle_layout(cfg_id):
    cfg = gen.CONFIGS[cfg_id]
    a = orc.Arch(tuple(cfg["layers_per_level"]), cfg["d_model"], cfg["n_heads"], cfg["d_head"], cfg["d_mlp"],
                 cfg["vocab"], cfg["max_seq"])
    ctx = dp.Context(list(cfg["layers_per_level"]), cfg["d_model"], cfg["n_heads"], cfg["d_head"], cfg["d_mlp"],
                     cfg["vocab"], cfg["max_seq"])
    lay = orc.param_layout(a)
    assert dp.dipaco_path_param_count(ctx) == orc.param_count(a)
    assert dp.dipaco_tensor_count(ctx) == len(lay)
    for i in range(dp.dipaco_tensor_count(ctx)):
        name, off, rows, cols, dec = dp.dipaco_tensor_info(ctx, i)
        o_off, o_shape, o_dec = lay[name]
        assert off == o_off and dec == o_dec, name
        assert (rows, cols) == (o_shape if len(o_shape) == 2 else (o_shape[0], 1)), name
    bounds = orc.segment_bounds(a)
    assert dp.dipaco_segment_count(ctx) == len(bounds)
    for s, (lo, hi) in enumerate(bounds):
        assert dp.dipaco_segment_offset(ctx, s) == lo and dp.dipaco_segment_size(ctx, s) == hi - lo
    assert dp.dipaco_workspace_bytes(ctx, cfg["batch"], cfg["seq"]) > 0


def test_path_index_matches_oracle():
    for K in [(2, 2), (16, 16), (3, 1, 4)]:
        P = int(np.prod(K))
        for j in range(P):
            mods = dp.dipaco_path_modules(j, K)
            assert mods == orc.modules_of_path(j, K)
            assert dp.dipaco_path_index(mods, K) == j == orc.path_index(mods, K)
    assert dp.dipaco_path_index([2, 0], [2, 2]) == -1
    with pytest.raises(dp.DipacoError):
        dp.dipaco_path_modules(4, [2, 2])


@pytest.mark.parametrize("kw", [dict(d_model=60), dict(d_head=48), dict(vocab=250), dict(d_mlp=0), dict(d_model=4096),
                                dict(layers_per_level=[])])
def test_create_rejects_unsupported_shapes(kw):
    base = dict(layers_per_level=[1, 1], d_model=64, n_heads=2, d_head=32, d_mlp=256, vocab=256, max_seq=64)
    base.update(kw)
    with pytest.raises(dp.DipacoError):
        dp.Context(**base)
    assert dp.last_error() != ""


def test_stateless_calls_validate_before_touching_the_gpu():
    lib = dp.load()
    null = ctypes.c_void_p()
    ptrs = (ctypes.c_void_p * 1)(null)
    st = lib.dipaco_module_outer_step(null, null, ptrs, None, 1, 16, 0, 0.7, 0.9, None)
    assert st == -1 and b"theta" in lib.dipaco_last_error()
    st = lib.dipaco_module_outer_step(ctypes.c_void_p(16), ctypes.c_void_p(16), ptrs, None, 0, 16, 0, 0.7, 0.9, None)
    assert st == -2
    st = lib.dipaco_module_outer_step(ctypes.c_void_p(20), ctypes.c_void_p(16), ptrs, None, 1, 16, 0, 0.7, 0.9, None)
    assert st == -3
    st = lib.dipaco_route_prefix(ctypes.c_void_p(16), ctypes.c_void_p(16), 8, 6, 4, ctypes.c_void_p(16),
                                 ctypes.c_void_p(16), None, None)
    assert st == -2 and b"multiple of 4" in lib.dipaco_last_error()
    st = lib.dipaco_route_prefix(ctypes.c_void_p(16), ctypes.c_void_p(16), 8, 8, 5000, ctypes.c_void_p(16),
                                 ctypes.c_void_p(16), None, None)
    assert st == -2
