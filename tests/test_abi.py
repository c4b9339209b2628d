"""The C-ABI library builds, loads without a GPU and exports every function that the
headers under include/ declare; the Python binding knows the same names."""
import ctypes
import glob
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared():
    text = "\n".join(open(h).read() for h in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"^(?:int32_t|uint64_t|const char\*)\s+(\w+)\s*\(", text, flags=re.M)))


def test_header_declares_the_four_entry_points():
    names = declared()
    for n in ("tr_verify_step", "tree_attention", "accept_path", "kv_compact"):
        assert n in names
    # the method's header carries no experiment knobs or measurement aids
    main = open(os.path.join(ROOT, "include", "trjacobi.h")).read()
    for n in ("trj_set_tunable", "trj_profile_begin", "trj_copy_probe", "trj_linear"):
        assert n not in main


def test_library_exports_every_declared_symbol():
    from paper_2406_17404_amd import binding
    assert os.path.exists(binding.LIB_PATH), "build the library first (__graft_entry__.build())"
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in declared():
        assert hasattr(lib, n), n
    assert sorted(binding.exported_symbols()) == declared()


def test_version_and_host_side_errors_need_no_gpu():
    from paper_2406_17404_amd import binding as b
    assert "gfx950" in b.trj_version()
    l = b.lib()
    # null pointers and bad shapes are rejected before anything touches a device
    n = ctypes.c_size_t(0)
    assert l.trj_workspace_bytes(None, 64, 1, 1088, ctypes.byref(n)) == -1
    d = b.ModelDesc(2, 256, 4, 64, 1024, 2048, 1e-5, 1e4, b.F32)
    assert l.trj_workspace_bytes(ctypes.byref(d), 15, 1, 143, ctypes.byref(n)) == 0 and n.value > 0
    d.dtype = 7
    assert l.trj_workspace_bytes(ctypes.byref(d), 15, 1, 143, ctypes.byref(n)) == -3
    d.dtype, d.d_model = b.BF16, 250
    assert l.trj_workspace_bytes(ctypes.byref(d), 15, 1, 143, ctypes.byref(n)) == -2
    # output widths that are not whole 32-row weight tiles are refused up front, in both modes
    for dt in (b.BF16, b.F32):
        for dm, ff in ((48, 1024), (256, 1040)):
            bad = b.ModelDesc(2, dm, 4, 64, ff, 2048, 1e-5, 1e4, dt)
            assert l.trj_workspace_bytes(ctypes.byref(bad), 15, 1, 143, ctypes.byref(n)) == -2, (dt, dm, ff)
    assert l.trj_tree_mask(None, None, 1, 1, None, None, None, None) == -1
    assert l.accept_path(None, 1, 1, 1, 1, 1000, 8, 1, 1, 1, 1, 1, 1, None) == -4
    assert l.kv_compact(None, None, 0, None, None, None, None, 1, 1, 1, 64, 64, 0, None, None) == -1


def test_tunables_refuse_unknown_names_and_unusable_values():
    from paper_2406_17404_amd import binding as b
    l = b.lib()
    assert l.trj_set_tunable(b"no_such_knob", 1) == -2
    assert l.trj_set_tunable(b"attn_target_wgs", 0) == -2      # would divide by zero in the plan
    assert l.trj_set_tunable(b"gemm_cfg", 9) == -2
    assert l.trj_set_tunable(None, 1) == -1
    assert l.trj_set_tunable(b"attn_target_wgs", 256) == 0
