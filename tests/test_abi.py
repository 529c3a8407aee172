"""The C-ABI library loads and exports every entry point the header declares;
argument errors that need no GPU are reported as statuses, not crashes."""
import ctypes as C
import os
import re

import pytest

import paper_2601_12347_amd as rp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ripple.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ripple_[a-z_]+)\s*\(", text)))


def test_library_is_built_and_loads():
    assert os.path.exists(rp.LIB_PATH), "build with python -m paper_2601_12347_amd.build"
    rp.load_library()


def test_every_declared_symbol_is_exported():
    lib = rp.load_library()
    names = declared_functions()
    assert set(names) == set(rp.EXPORTS)
    for name in names:
        assert hasattr(lib, name), name


def test_struct_layouts_match_the_header():
    assert C.sizeof(rp.binding.LayerDesc) == 72
    assert C.sizeof(rp.BatchResult) == 4 * 6 + 8 + 4 * 9 + 4 + 8 * 9 + 4 + 3 * 4 * 9 + 4 * 9 + 4   # the last two: hop_mode, n_ops_done
    assert C.sizeof(rp.Stats) == 8 + 8 * 8 * 9 * 2 + 8 * 9 * 3
    assert C.sizeof(rp.binding.Peaks) == 6 * 8 + 2 * 4


def test_null_and_bad_arguments_return_statuses():
    lib = rp.load_library()
    assert lib.ripple_init_graph(None, 1, 1, 0, 0, None, None, None, 1, 0, None) == rp.binding.RIPPLE_EINVAL
    ctx = C.c_void_p()
    # capacity smaller than the vertex count; zero feature width; unknown storage type
    assert lib.ripple_init_graph(C.byref(ctx), 5, 4, 0, 0, None, None, None, 4, 0, None) == rp.binding.RIPPLE_EINVAL
    assert lib.ripple_init_graph(C.byref(ctx), 0, 4, 0, 0, None, None, None, 0, 0, None) == rp.binding.RIPPLE_EINVAL
    assert lib.ripple_init_graph(C.byref(ctx), 0, 4, 0, 0, None, None, None, 4, 7, None) == rp.binding.RIPPLE_EINVAL
    assert not ctx.value
    for fn in (lib.ripple_full_infer, lib.ripple_compact):
        assert fn(None) == rp.binding.RIPPLE_EINVAL
    assert lib.ripple_load_model(None, 1, None) == rp.binding.RIPPLE_EINVAL
    assert lib.ripple_apply_updates(None, None, 0, None, 0, None) == rp.binding.RIPPLE_EINVAL
    assert lib.ripple_get_embeddings(None, 0, None, 0, None) == rp.binding.RIPPLE_EINVAL
    assert lib.ripple_measure_peaks(None, None) == rp.binding.RIPPLE_EINVAL
    assert lib.ripple_last_error(None) == b""
    lib.ripple_destroy(None)
