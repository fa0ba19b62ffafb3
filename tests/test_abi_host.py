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


def test_outer_table_pack_is_host_only_and_validates():
    """The table image of the table-driven outer step is built on the host: sizes, chunk offsets and normalised
    weights can be checked without a GPU (the addresses are never dereferenced by the packer)."""
    import struct
    mods = [dict(theta=0x1000, momentum=0x2000, inputs=[0x3000, 0x4000, 0x5000], weights=[1.0, 2.0, 1.0],
                 n_elems=4096 * 2 + 5, is_delta=False),
            dict(theta=0x6000, momentum=0x7000, inputs=[0x8000], weights=None, n_elems=0, is_delta=True),
            dict(theta=0x9000, momentum=0xa000, inputs=[0xb000], weights=None, n_elems=10, is_delta=True,
                 norm_scale=4.0)]
    need = dp.dipaco_outer_table_bytes(mods)
    image = dp.dipaco_outer_table_pack(mods)
    assert len(image) == need and need % 16 == 0
    magic, n_modules, total_chunks, total_paths = struct.unpack_from("<4Q", image, 0)
    assert (n_modules, total_chunks, total_paths) == (3, 3 + 0 + 1, 5)
    entry = struct.Struct("<QQQQQii")                       # theta, momentum, n_elems, first_chunk, path_begin, ...
    ents = [entry.unpack_from(image, 32 + i * entry.size) for i in range(3)]
    assert [e[3] for e in ents] == [0, 3, 3] and [e[4] for e in ents] == [0, 3, 4]
    assert [e[0] for e in ents] == [0x1000, 0x6000, 0x9000] and [e[6] for e in ents] == [0, 1, 1]
    off_inputs = 32 + 3 * entry.size
    assert struct.unpack_from("<5Q", image, off_inputs) == (0x3000, 0x4000, 0x5000, 0x8000, 0xb000)
    alpha = struct.unpack_from("<5f", image, off_inputs + 5 * 8)
    assert np.allclose(alpha, [0.25, 0.5, 0.25, 1.0, 4.0], rtol=1e-7)
    for bad in (dict(mods[0], theta=0x1004), dict(mods[0], weights=[1.0, -1.0, 1.0]), dict(mods[0], inputs=[]),
                dict(mods[0], norm_scale=0.0), dict(mods[0], inputs=[0x3000, 0, 0x5000])):
        with pytest.raises(dp.DipacoError):
            dp.dipaco_outer_table_pack([bad])
    with pytest.raises(dp.DipacoError):                     # an image that the packer did not write
        dp.dipaco_outer_step_table(bytes(len(image)), 0x1000, 0.7, 0.9, stream=_NoStream())


class _NoStream:
    cuda_stream = 0


@pytest.mark.parametrize("M,N", [(896, 3584), (3584, 896), (896, 2688), (896, 896), (256, 256), (300, 200), (8, 776),
                                 (1024, 4096), (136, 64), (896, 32000)])
def test_uneven_split_plan_is_consistent(M, N):
    """Host logic of the weight-gradient launch: the plan's classes cover every tile of C once, no class gets more
    slices than allowed or than the class inside C, and one workgroup per (tile, slice) fits the 256 compute units."""
    K, cap = 32768, 32
    p = dp.dipaco_k_gemm_split_plan(M, N, K, cap)
    bm, bn = p["tile"]
    if bm == 0:                                   # no plan: too many tiles for one round (the head's gradient)
        assert ((M + 255) // 256) * ((N + 255) // 256) > 128
        return
    tiles_m, tiles_n = -(-M // bm), -(-N // bn)
    fm, fn = p["inside"]
    assert 0 <= tiles_m - fm <= 1 and 0 <= tiles_n - fn <= 1
    want = [fm * fn, (tiles_m - fm) * fn, fm * (tiles_n - fn), (tiles_m - fm) * (tiles_n - fn)]
    assert p["tiles"] == want and sum(want) == tiles_m * tiles_n
    s = p["slices"]
    live = [c for c in range(4) if want[c] > 0]
    assert all(1 <= s[c] <= min(cap, K // 32) for c in live)
    assert all(s[c] <= s[0] or want[0] == 0 for c in live)
    assert sum(want[c] * s[c] for c in range(4)) <= 256
    assert max(s[c] for c in live) >= 2
    # a tile with idle waves still loads whole operand panels: it never gets fewer than half the slices
    assert all(2 * s[c] >= s[0] for c in live)


def test_uneven_split_plan_of_the_step_shapes():
    """The shapes of the config-2 step: 896 = 3.5 x 256 rows take oblong tiles where that frees a K slice."""
    assert dp.dipaco_k_gemm_split_plan(896, 3584, 32768, 32)["tile"] == (128, 512)
    assert dp.dipaco_k_gemm_split_plan(3584, 896, 32768, 32)["tile"] == (512, 128)
    assert dp.dipaco_k_gemm_split_plan(896, 2688, 32768, 32)["tile"] == (256, 256)
    p = dp.dipaco_k_gemm_split_plan(896, 3584, 32768, 32)
    assert p["tiles"] == [49, 0, 0, 0] and p["slices"][0] == 5
    with pytest.raises(dp.DipacoError):
        dp.dipaco_k_gemm_split_plan(896, 3584, 1000, 32)
