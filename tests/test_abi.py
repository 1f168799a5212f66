"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares, and its pure host
functions behave.  No kernel is launched here."""
import os
import re

import pytest

from paper_2402_05099_amd import binding as hb
from paper_2402_05099_amd import build as hbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(hb.LIB_PATH):
        hbuild.build(verbose=False)
    return hb.lib()


def declared_functions():
    names = set()
    for header in ("hydragen.h", "hydragen_debug.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(hg_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_attention_header_declares_no_debug_entry_point():
    text = open(os.path.join(ROOT, "include", "hydragen.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    assert not re.findall(r"\bhg_debug_[a-z0-9_]+\s*\(", text)


def test_header_and_binding_agree():
    assert declared_functions() == sorted(hb.EXPORTS)


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_workspace_bytes_and_strerror(lib):
    assert hb.hg_workspace_bytes(1024, 40, 128, 3) == (3 * 1024 * 40 * 129 * 4 + 255) // 256 * 256
    assert hb.hg_workspace_bytes(0, 40, 128, 3) == 0
    assert hb.strerror(hb.HG_OK) == "ok"
    assert hb.strerror(hb.HG_ERR_UNSUPPORTED) == "unsupported shape or dtype"
    assert hb.strerror(12345) == "unknown error"


def test_constants_match_header():
    text = open(os.path.join(ROOT, "include", "hydragen.h")).read()
    for name in ("HG_OK", "HG_ERR_INVALID_ARG", "HG_ERR_UNSUPPORTED", "HG_ERR_WORKSPACE", "HG_ERR_HIP", "HG_ERR_STATIC_LIMIT", "HG_STATIC_SCRATCH_BYTES", "HG_F32", "HG_BF16",
                 "HG_MAX_LEVELS", "HG_MAX_PARTS", "HG_OPT_PREFIX_SPLITS", "HG_OPT_SUFFIX_CHUNK", "HG_OPT_OVERLAP",
                 "HG_OPT_NAIVE_CHUNK", "HG_OPT_STAGE_TIMING", "HG_OPT_PREFIX_KERNEL", "HG_TIMING_RING", "HG_OPT_WIDE_SLOTS",
                 "HG_OPT_NUM_QUERIES", "HG_OPT_SUFFIX_KERNEL", "HG_OPT_SUFFIX_ITEMS_PER_WAVE", "HG_OPT_SUFFIX_TILE_ROWS", "HG_OPT_FUSED_KERNEL", "HG_KV_BF16", "HG_KV_E4M3"):
        m = re.search(rf"\b{name}\s*=\s*(\d+)", text)
        assert m, name
        assert int(m.group(1)) == getattr(hb, name), name


def test_paged_struct_layout_matches_header():
    """hg_paged_kv is passed by pointer: the ctypes mirror must have the header's fields in the header's order."""
    text = open(os.path.join(ROOT, "include", "hydragen.h")).read()
    body = re.search(r"typedef struct \{([^}]*)\} hg_paged_kv;", text).group(1)
    names = re.findall(r"(\w+);", body)
    assert names == [f[0] for f in hb.hg_paged_kv._fields_]
    body = re.search(r"typedef struct \{([^}]*)\} hg_level;", text).group(1)
    assert re.findall(r"(\w+);", body) == [f[0] for f in hb.hg_level._fields_]


def test_calls_without_a_context_are_rejected_before_any_device_work(lib):
    """Every compute entry point checks its context first: a null context is an argument error, with no GPU present."""
    import ctypes
    z = ctypes.c_void_p(0)
    kv = hb.hg_paged_kv(0, 0, 0, 16, 1, 1, 0, 1.0, 1.0)
    lv = hb.hg_level()
    bad = hb.HG_ERR_INVALID_ARG
    assert lib.hg_prefix_attn(z, z, z, z, 1, 1, 1, 128, 1, 0.0, z, 0, z) == bad
    assert lib.hg_suffix_attn(z, z, z, z, z, z, 1, 1, 1, 1, 128, 0.0, z, 0, z) == bad
    assert lib.hg_suffix_attn_fp8(z, z, z, z, 1.0, 1.0, z, z, 1, 1, 1, 1, 128, 0.0, z, 0, z) == bad
    assert lib.hg_hydragen_attn(z, z, 0, ctypes.byref(lv), z, z, z, z, 1, 1, 1, 1, 128, 0.0, z, 0, z) == bad
    assert lib.hg_hydragen_attn_fp8(z, z, 0, ctypes.byref(lv), z, z, 1.0, 1.0, z, z, 1, 1, 1, 1, 128, 0.0, z, 0, z) == bad
    assert lib.hg_naive_attn(z, z, 0, ctypes.byref(lv), z, z, z, z, 1, 1, 1, 1, 128, 0.0, z, 0, z) == bad
    assert lib.hg_hydragen_attn_static(z, z, 0, ctypes.byref(lv), z, z, z, z, 1, 1, 1, 1, 128, 0.0, z, 0, z) == bad
    assert lib.hg_suffix_attn_paged(z, z, ctypes.byref(kv), z, 1, 1, 1, 1, 128, 0.0, z, 0, z) == bad
    assert lib.hg_kv_append(z, z, z, z, z, z, z, 1, 1, 1, 128) == bad
    assert lib.hg_kv_append_fp8(z, z, z, z, z, 1.0, 1.0, z, z, 1, 1, 1, 128) == bad
    # scales are checked even before the context
    assert lib.hg_suffix_attn_fp8(z, z, z, z, 0.0, 1.0, z, z, 1, 1, 1, 1, 128, 0.0, z, 0, z) == bad
    assert lib.hg_kv_append_fp8(z, z, z, z, z, 1.0, float("nan"), z, z, 1, 1, 1, 128) == bad
