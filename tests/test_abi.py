"""The C-ABI library loads and exports every entry point declared in include/specpipe.h,
and the pure-host entry points behave (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

import paper_2504_04104_amd as sp
from paper_2504_04104_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "specpipe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sp_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = sp.load_library()
    names = declared_functions()
    assert {"sp_stage_forward", "sp_tree_insert", "sp_tree_prune", "sp_kv_compact"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_version_and_strerror():
    lib = sp.load_library()
    assert lib.sp_version() == 1
    assert lib.sp_strerror(0) == b"ok"
    assert b"capacity" in lib.sp_strerror(-2)


def test_query_sizes_is_host_arithmetic():
    lib = sp.load_library()
    cfg = binding.sp_config(4, 4096, 32, 8, 128, 14336, 1e-5, 500000.0, binding.SP_BF16, 1, 256, 64, 2048 + 512, 0)
    sz = binding.sp_sizes()
    assert lib.sp_stage_query_sizes(C.byref(cfg), C.byref(sz)) == 0
    assert sz.kv_row_bytes == 256
    # one token of one layer: K and V rows over 8 heads = 4096 bytes (Sec. 4.5, Table 1)
    assert 2 * 8 * sz.kv_row_bytes == 4096
    assert sz.kv_bytes == 4 * 2 * 8 * (2048 + 512) * 256
    assert sz.tables_bytes > 0 and sz.workspace_bytes > 0
    bad = binding.sp_config(4, 4096, 32, 7, 128, 14336, 1e-5, 500000.0, binding.SP_BF16, 1, 256, 64, 2560, 0)
    assert lib.sp_stage_query_sizes(C.byref(bad), C.byref(sz)) == -1
    odd = binding.sp_config(4, 4096, 32, 8, 96, 14336, 1e-5, 500000.0, binding.SP_BF16, 1, 256, 64, 2560, 0)
    assert lib.sp_stage_query_sizes(C.byref(odd), C.byref(sz)) == -9


def test_struct_layouts_match_the_header():
    # counters, five 4-byte columns, the bitmask rows, the root's prediction + padding to 8
    assert C.sizeof(binding.sp_tree_view) == 8 + 5 * 4 * 256 + 8 * 4 * 256 + 8
    assert binding.sp_tree_view.pred.offset == 8 + 4 * 4 * 256 + 8 * 4 * 256
    assert C.sizeof(binding.sp_head_weights) == 24
    assert C.sizeof(binding.sp_config) == 64
