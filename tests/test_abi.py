"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the header
declares, and validates configurations and arguments before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2603_20661_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
B = pytest.importorskip("paper_2603_20661_amd.binding", reason="libwww.so is not built")


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "www.h")).read()
    declared = set(re.findall(r"\b(www_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(B.lib, name), name


def test_config_struct_matches_header_layout():
    assert ctypes.sizeof(B.WwwConfig) == 18 * 4
    assert B.WwwConfig.num_kv_blocks.offset == 64


def test_query_sizes_and_config_validation():
    cfg = B.make_config(synth.M8B, 64, 272, 81920, 6000)
    wbytes, kvbytes, wsbytes = B.www_query_sizes(cfg)
    assert wbytes == synth.blob_layout(synth.M8B)[1]
    assert kvbytes == 6000 * 32 * 2 * 8 * 16 * (128 * 2 + 4)    # 2 MiB of 16-bit codes + 32 KiB of scales per block for the 8B shape
    # the blob of every source format, with and without the gains of the head normalisation, is as long as the generator's
    import dataclasses
    for base in (synth.M8B, synth.M1B, synth.TINY):
        for wd in ((base.weight_dtype,) if base is synth.TINY else (1, 2, 3, 4)):
            for qkn in (0, 1):
                shape = dataclasses.replace(base, weight_dtype=wd, qk_norm=qkn)
                assert B.www_query_sizes(B.make_config(shape, 4, 16, 512, 64))[0] == synth.blob_layout(shape)[1], shape
    assert wsbytes > synth.M8B.n_params() * 2 - synth.M8B.vocab * synth.M8B.d_model * 2
    for field, value, code in (("abi_version", 99, B.E_ABI_MISMATCH), ("head_dim", 96, B.E_BAD_CONFIG),
                               ("kv_block_size", 32, B.E_BAD_CONFIG), ("n_kv_heads", 3, B.E_BAD_CONFIG),
                               ("vocab", 1001, B.E_BAD_CONFIG), ("max_batch", 0, B.E_BAD_CONFIG), ("flags", 2, B.E_BAD_CONFIG)):
        bad = B.make_config(synth.TINY, 4, 16, 512, 64)
        setattr(bad, field, value)
        with pytest.raises(B.WwwError) as e:
            B.www_query_sizes(bad)
        assert e.value.code == code and str(e.value)


def test_null_arguments_are_rejected_before_any_launch():
    assert B.lib.www_query_sizes(None, None, None, None) == B.E_INVALID_ARG
    cfg = B.make_config(synth.TINY, 4, 16, 512, 64)
    h = ctypes.c_void_p()
    assert B.lib.www_model_load(ctypes.byref(cfg), None, None, None, None, ctypes.byref(h)) == B.E_INVALID_ARG
    assert B.lib.www_model_load(ctypes.byref(cfg), 256, 512, 100, None, ctypes.byref(h)) == B.E_INVALID_ARG   # misaligned workspace
    assert B.lib.www_prefill(None, None, None, None, None, 1, 1, None, None, None) == B.E_INVALID_ARG
    assert B.lib.www_decode_step(None, None, None, None, 1, None, None, None) == B.E_INVALID_ARG
    assert B.lib.www_debug_slots(None, None, 1, None, None) == B.E_INVALID_ARG
    assert b"NULL" in B.lib.www_last_error() or b"bad" in B.lib.www_last_error()
    B.lib.www_model_free(None)


def test_prefill_gemm_tile_order_visits_every_tile_once():
    """the workgroup -> tile map of the prefill projections (laid out for the GPU's eight L2 caches) is a bijection, for
    tile counts that fill whole super-groups of 32 token tiles, for remainders, and for single rows and columns"""
    shapes = [(314, 112), (314, 16), (314, 24), (1, 1), (1, 7), (9, 1), (2, 3), (32, 16), (33, 7), (5, 112), (64, 16),
              (63, 24), (31, 5), (32, 1), (40, 12), (157, 8), (4, 64)]
    for n_tt, n_rt in shapes:
        seen = {B.www_debug_prefill_tile(w, n_tt, n_rt) for w in range(n_tt * n_rt)}
        assert seen == {(t, r) for t in range(n_tt) for r in range(n_rt)}, (n_tt, n_rt)
    # in a full super-group the 32 workgroups an XCD gets per round of 256 are 4 token tiles x 8 row tiles,
    # and the eight XCDs work on the same 8 row tiles
    n_tt, n_rt = 64, 16
    for rnd in range(4):
        per_xcd = {}
        for w in range(256 * rnd, 256 * (rnd + 1)):
            per_xcd.setdefault(w % 8, []).append(B.www_debug_prefill_tile(w, n_tt, n_rt))
        rows = None
        for x, tiles in per_xcd.items():
            assert len({t for t, _ in tiles}) == 4 and len({r for _, r in tiles}) == 8, (rnd, x)
            rows = rows or {r for _, r in tiles}
            assert {r for _, r in tiles} == rows
    for bad in ((-1, 4, 4), (16, 4, 4), (0, 0, 4), (0, 4, 0)):
        with pytest.raises(Exception):
            B.www_debug_prefill_tile(*bad)
