"""CPU-side checks of the C-ABI library: it loads, exports every function include/gta.h
declares, and its host-only argument checks answer without touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2604_16715_amd as gta
    return gta.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "gta.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(gta_[a-z_]+)\s*\(", text)
    return sorted(set(names))


def test_header_symbols_are_exported(lib):
    names = declared_functions()
    assert {"gta_plan_create", "gta_attn_fwd", "gta_attn_bwd", "gta_plan_destroy",
            "gta_attn_scratch_bytes", "gta_plan_workspace_bytes"} <= set(names)
    for name in names:
        assert hasattr(lib, name), f"{name} declared in gta.h but not exported"


def test_version_and_error_strings(lib):
    assert b"gfx950" in lib.gta_version()
    assert isinstance(lib.gta_last_error(), bytes)


def test_workspace_query_is_host_only(lib):
    from paper_2604_16715_amd.binding import _PlanOpts
    assert lib.gta_plan_workspace_bytes(1000, 1500, 20000, None) > 20000 * 8
    assert lib.gta_plan_workspace_bytes(-1, 10, 10, None) == 0
    assert lib.gta_plan_workspace_bytes(10, 10, 1 << 31, None) == 0
    assert lib.gta_plan_workspace_bytes(10, 10, (1 << 31) - 1023, None) == 0   # 32-bit positions + loop strides
    assert lib.gta_plan_workspace_bytes(10, 10, (1 << 31) - 1024, None) > 0
    bad = _PlanOpts(0, 48, 0, 0, 0)         # not a power of two
    assert lib.gta_plan_workspace_bytes(10, 10, 10, ctypes.byref(bad)) == 0
    bad = _PlanOpts(0, 512, 256, 0, 0)      # hub_chunk < wave_max_deg
    assert lib.gta_plan_workspace_bytes(10, 10, 10, ctypes.byref(bad)) == 0
    small = _PlanOpts(0, 4, 8, 0, 0)
    assert lib.gta_plan_workspace_bytes(10, 10, 100, ctypes.byref(small)) > 0


def test_null_arguments_are_rejected_before_any_gpu_call(lib):
    handle = ctypes.c_void_p()
    rc = lib.gta_plan_create(ctypes.byref(handle), None, None, 4, 4, 8, None, None, 0, None)
    assert rc == 1 and b"null" in lib.gta_last_error()
    rc = lib.gta_plan_create(None, None, None, 4, 4, 8, None, None, 0, None)
    assert rc == 1
    assert lib.gta_attn_scratch_bytes(None, 4, 16, 0) == 0
    rc = lib.gta_attn_fwd(None, None, None, None, None, None, None, None, 0, 0, 4, 16, 0, 0.0, None, 0, None)
    assert rc == 1 and b"plan" in lib.gta_last_error()
    rc = lib.gta_attn_bwd(None, None, None, None, None, None, None, None, None, None, None, None,
                          0, 0, 4, 16, 0, 0.0, None, 0, None)
    assert rc == 1
    assert lib.gta_plan_get_info(None, None) == 1
    # halo forms: the split is validated before anything else
    rc = lib.gta_attn_fwd_halo(None, None, None, None, None, None, None, None, 5, None, None, 0, 4, 4, 16, 0,
                               0.0, None, 0, None)
    assert rc == 1 and b"n_local" in lib.gta_last_error()
    rc = lib.gta_attn_fwd_halo(None, None, None, None, None, None, None, None, 2, None, None, 0, 4, 4, 16, 0,
                               0.0, None, 0, None)
    assert rc == 1 and b"halo" in lib.gta_last_error()
    rc = lib.gta_attn_bwd_halo(None, None, None, None, None, None, None, None, 4, None, None, None, None, None,
                               None, None, None, 0, 4, 4, 16, 0, 0.0, None, 0, None)
    assert rc == 1 and b"plan" in lib.gta_last_error()


def test_newer_entry_points_reject_bad_arguments_on_the_host(lib):
    import ctypes
    # the forward without scratch argument: same plan checks as gta_attn_fwd, before anything else
    rc = lib.gta_attn_fwd_noalloc(None, None, None, None, None, None, None, None, 0, 0, 4, 16, 0, 0.0, None)
    assert rc == 1 and b"plan" in lib.gta_last_error()
    assert lib.gta_plan_compact(None, None, 0, None) == 1
    assert lib.gta_plan_retained_bytes(-1, 1, 1, None) == 0
    keep, whole = lib.gta_plan_retained_bytes(1000, 1500, 20000, None), lib.gta_plan_workspace_bytes(1000, 1500, 20000, None)
    assert 20000 * 12 <= keep < whole          # three int32 arrays per entry stay, the sort buffers do not
    # grouped projections: sizes, grouping and dtype are checked before any pointer is touched
    assert lib.gta_linear_group_scratch_bytes(256, 1, 3) >= 3 * 256 * 256 * 2
    assert lib.gta_linear_group_scratch_bytes(256, 5, 1) == 0
    rc = lib.gta_linear_group(None, 1, None, 1, None, None, 10, 256, 0, 0, None, 0, None)      # fp32
    assert rc == 2 and b"bfloat16" in lib.gta_last_error()
    rc = lib.gta_linear_group(None, 1, None, 1, None, None, 10, 96, 1, 0, None, 0, None)       # d = 96
    assert rc == 2
    rc = lib.gta_linear_group(None, 1, None, 1, None, None, 10, 256, 1, 0, None, 0, None)      # null arrays
    assert rc == 1
    # grouped weight gradients: the product count and the pointer arrays
    assert lib.gta_linear_dw_group_scratch_bytes(1000, 64, 64, 3) == 3 * lib.gta_linear_dw_scratch_bytes(1000, 64, 64)
    assert lib.gta_linear_dw_group_scratch_bytes(1000, 64, 64, 5) == 0
    rc = lib.gta_linear_dw_group(None, None, None, 5, 10, 64, 64, 1, None, 0, None)
    assert rc == 2 and b"products" in lib.gta_last_error()
    rc = lib.gta_linear_dw_group(None, None, None, 2, 10, 64, 64, 1, None, 0, None)
    assert rc == 1
    rc = lib.gta_stream_probe(3, None, None, None, 0, None)
    assert rc == 1 and b"mode" in lib.gta_last_error()
