"""CPU-only checks of the C-ABI library: it loads, exports every function include/hdt.h declares, and
its host-side argument checks answer without a GPU (no compute call is made here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2407_08330_amd import binding
    if not os.path.exists(binding.library_path()):
        from paper_2407_08330_amd import build
        build.build()
    return binding.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "hdt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hdt_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_three_calls_of_the_path():
    names = declared_functions()
    for must in ("hdt_build_layout", "hdt_attn_fwd", "hdt_attn_bwd"):
        assert must in names


def test_library_exports_every_declared_function(lib):
    from paper_2407_08330_amd import binding
    names = declared_functions()
    assert len(names) >= 13
    for name in names:
        assert hasattr(lib, name), f"{name} declared in hdt.h but not exported"
    assert sorted(binding.EXPORTED_SYMBOLS) == names


def test_status_strings(lib):
    expect = ["HDT_OK", "HDT_ERR_INVALID_ARG", "HDT_ERR_SHAPE", "HDT_ERR_HIERARCHY", "HDT_ERR_UNSUPPORTED",
              "HDT_ERR_OOM", "HDT_ERR_HIP"]
    for code, name in enumerate(expect):
        assert lib.hdt_status_string(code).decode() == name
    assert lib.hdt_status_string(99).decode() == "HDT_ERR_UNKNOWN"


def test_build_layout_argument_errors_without_gpu(lib):
    h = ctypes.c_void_p(0)
    assert lib.hdt_build_layout(None, None, 1, 8, None, None, None) == 1          # out == NULL
    assert lib.hdt_build_layout(None, None, -1, 8, None, None, ctypes.byref(h)) == 1
    assert b"negative" in lib.hdt_last_error()
    assert lib.hdt_build_layout(None, None, 1, -8, None, None, ctypes.byref(h)) == 1
    assert lib.hdt_build_layout(None, None, 1, (1 << 19) + 1, None, None, ctypes.byref(h)) == 2   # SHAPE
    assert lib.hdt_build_layout(None, None, 1, 8, None, None, ctypes.byref(h)) == 1          # NULL id arrays
    from paper_2407_08330_amd.binding import _Opts
    for tm, tn in [(48, 64), (128, 16), (256, 64), (128, 160)]:
        opts = _Opts(tm, tn, 0, 0, 0, 0)
        assert lib.hdt_build_layout(None, None, 0, 0, ctypes.byref(opts), None, ctypes.byref(h)) == 4  # UNSUPPORTED
    opts = _Opts(0, 0, 0, 0, 0, 8)   # an edge kind that does not exist
    assert lib.hdt_build_layout(None, None, 0, 0, ctypes.byref(opts), None, ctypes.byref(h)) == 1
    opts = _Opts(0, 0, 0, 0, 0, 0, 0, 0, -5)   # a negative capacity
    assert lib.hdt_build_layout(None, None, 0, 0, ctypes.byref(opts), None, ctypes.byref(h)) == 1
    assert h.value is None or h.value == 0


def test_empty_layout_and_calls_on_it_are_noops_without_gpu(lib):
    from paper_2407_08330_amd.binding import _Info
    for batch, n_pos in [(0, 128), (3, 0), (0, 0)]:
        h = ctypes.c_void_p(0)
        assert lib.hdt_build_layout(None, None, batch, n_pos, None, None, ctypes.byref(h)) == 0
        info = _Info()
        assert lib.hdt_layout_info(h, ctypes.byref(info)) == 0
        assert (info.batch, info.n_pos, info.n_tiles, info.nnz) == (batch, n_pos, 0, 0)
        assert (info.tile_m, info.tile_n) == (128, 64)
        need = ctypes.c_int64(-7)
        assert lib.hdt_layout_status(h, ctypes.byref(need)) == 0 and need.value == 0   # nothing deferred, nothing needed
        assert lib.hdt_layout_status(h, None) == 0
        assert lib.hdt_attn_bwd_no_alloc(h, None, None, None, None, None, None, None, None, None, 4, 64, 0,
                                         ctypes.c_float(0.125), None) == 0
        # attention on an empty layout: nothing to do, pointers are not looked at
        assert lib.hdt_attn_fwd(h, None, None, None, None, None, 4, 64, 0, ctypes.c_float(0.125), None) == 0
        assert lib.hdt_attn_bwd(h, None, None, None, None, None, None, None, None, None, 4, 64, 0,
                                ctypes.c_float(0.125), None, 0, None) == 0
        assert lib.hdt_attn_bwd_workspace_bytes(h, 4, 64, 0) == 0
        # but bad scalar arguments are still refused
        assert lib.hdt_attn_fwd(h, None, None, None, None, None, 4, 96, 0, ctypes.c_float(0.125), None) == 4
        assert lib.hdt_attn_fwd(h, None, None, None, None, None, 4, 64, 0, ctypes.c_float(-1.0), None) == 1
        assert lib.hdt_attn_fwd(h, None, None, None, None, None, 4, 64, 7, ctypes.c_float(0.125), None) == 4
        assert lib.hdt_attn_fwd(h, None, None, None, None, None, -1, 64, 0, ctypes.c_float(0.125), None) == 1
        if batch > 0:
            a, b = ctypes.c_int64(-1), ctypes.c_int64(-1)
            assert lib.hdt_layout_sample_info(h, 0, ctypes.byref(a), ctypes.byref(b)) == 0 and a.value == 0
            assert lib.hdt_layout_sample_info(h, batch, ctypes.byref(a), ctypes.byref(b)) == 2
        assert lib.hdt_layout_destroy(h) == 0
    assert lib.hdt_layout_destroy(None) == 0 and lib.hdt_layout_destroy_completed(None) == 0


def test_invalid_layout_handles_are_refused(lib):
    from paper_2407_08330_amd.binding import _Info
    junk = (ctypes.c_char * 512)()
    info = _Info()
    assert lib.hdt_layout_info(None, ctypes.byref(info)) == 1
    assert lib.hdt_layout_info(junk, ctypes.byref(info)) == 1
    assert lib.hdt_layout_status(junk, None) == 1 and lib.hdt_layout_status(None, None) == 1
    assert lib.hdt_attn_fwd(junk, None, None, None, None, None, 1, 64, 0, ctypes.c_float(0.1), None) == 1
    assert lib.hdt_attn_bwd_workspace_bytes(junk, 1, 64, 0) == 0
    assert lib.hdt_layout_destroy(junk) == 1 and lib.hdt_layout_destroy_completed(junk) == 1


def test_timing_calls_without_gpu(lib):
    assert lib.hdt_timing_enable(0) == 0
    assert lib.hdt_timing_reset() == 0
    assert lib.hdt_timing_read(None, None, None, 0) == 0
    assert lib.hdt_release_cached_memory() == 0
    flop = ctypes.c_double(-1.0)
    assert lib.hdt_status_string(lib.hdt_probe_mfma_bf16(0, 10, None, ctypes.byref(flop), None)).decode() == "HDT_ERR_INVALID_ARG"
    assert lib.hdt_status_string(lib.hdt_probe_mfma_bf16(4, 10, None, None, None)).decode() == "HDT_ERR_INVALID_ARG"


def test_hpe_argument_errors_without_gpu(lib):
    assert lib.hdt_index_vectors_workspace_bytes(0, 128) == 0
    assert lib.hdt_index_vectors_workspace_bytes(2, 100) >= 4 * (2 * 101 + 2 * 100)
    assert lib.hdt_index_vectors(None, None, -1, 8, 3, None, None, 0, None) == 1
    assert lib.hdt_index_vectors(None, None, 1, 8, 0, None, None, 0, None) == 1        # n_levels < 1
    assert lib.hdt_index_vectors(None, None, 1, 8, 32, None, None, 0, None) == 1       # n_levels too large
    assert lib.hdt_index_vectors(None, None, 0, 8, 3, None, None, 0, None) == 0        # empty: nothing to do
    assert lib.hdt_index_vectors(None, None, 1, 8, 3, None, None, 0, None) == 1        # NULL pointers
    assert lib.hdt_hpe_table(None, 4, 12, None) == 1                                   # d_model % 8
    assert lib.hdt_hpe_table(None, 0, 16, None) == 0
    assert lib.hdt_hpe_table(None, 4, 16, None) == 1
    assert lib.hdt_hpe_add(None, 0, 8, 3, None, 0, None, 16, 0, None) == 0
    assert lib.hdt_hpe_add(None, 1, 8, 3, None, 0, None, 12, 0, None) == 1
    assert lib.hdt_hpe_add(None, 1, 8, 3, None, 0, None, 16, 5, None) == 4             # dtype
    assert lib.hdt_hpe_add(None, 1, 8, 3, None, 0, None, 16, 0, None) == 1             # NULL pointers
