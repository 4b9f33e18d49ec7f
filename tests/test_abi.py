"""The C-ABI library loads and exports every function include/orch.h declares
(no compute calls: this runs without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "orch.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(orch_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = declared_functions()
    for want in ("orch_balance", "orch_pack", "orch_pack_composed", "orch_pack_composed_workspace", "orch_balance_padded", "orch_balance_tolerance", "orch_comm_volume", "orch_varlen_attn_fwd", "orch_balance_workspace",
                 "orch_pack_workspace", "orch_varlen_attn_workspace", "orch_varlen_attn_bwd",
                 "orch_varlen_attn_bwd_workspace", "orch_last_error"):
        assert want in names


def test_library_exports_every_declared_symbol():
    import paper_2503_23830_amd as orch
    from paper_2503_23830_amd import binding

    if not os.path.exists(orch.library_path()):
        from paper_2503_23830_amd import build
        build.build_library()
    lib = ctypes.CDLL(orch.library_path())
    for name in declared_functions():
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == declared_functions()


def test_workspace_queries_and_host_side_errors():
    """Host-checkable argument errors return before any launch, so they can be
    exercised without a GPU."""
    import paper_2503_23830_amd as orch
    from paper_2503_23830_amd import binding as B

    lib = orch.load_library()
    assert lib.orch_balance_workspace(32768, 256) >= 32768 * 40
    assert lib.orch_pack_workspace(32768, 256) >= 32768 * 24
    assert lib.orch_varlen_attn_workspace(128, 352000, 32) >= 129 * 4 + (352000 // 256 + 128) * 32 * 4
    fake = ctypes.c_void_p(256)
    asg = B._Assignment(256, 256, 256, 256, 256, 256, 256)
    rc = lib.orch_balance(fake, -1, 4, B._Phase(1, 1), asg, fake, 1 << 20, None)
    assert rc == -1 and b"n = -1" in lib.orch_last_error()
    rc = lib.orch_balance(fake, 8, 0, B._Phase(1, 1), asg, fake, 1 << 20, None)
    assert rc == -1
    rc = lib.orch_balance(fake, 8, 5000, B._Phase(1, 1), asg, fake, 1 << 20, None)
    assert rc == -3
    rc = lib.orch_balance(fake, 8, 4, B._Phase(1, 1), asg, fake, 16, None)
    assert rc == -2 and b"workspace" in lib.orch_last_error()
    rc = lib.orch_balance(fake, 8, 4, B._Phase(1, 1), B._Assignment(256, 0, 256, 256, 256, 256, 256),
                          fake, 1 << 20, None)
    assert rc == -1
    rc = lib.orch_balance_padded(fake, 8, 0, B._Phase(1, 1), asg, None, fake, 1 << 20, None)
    assert rc == -1 and b"D = 0" in lib.orch_last_error()
    rc = lib.orch_balance_padded(fake, 8, 5000, B._Phase(1, 1), asg, None, fake, 1 << 20, None)
    assert rc == -3
    rc = lib.orch_balance_padded(fake, 8, 4, B._Phase(1, 1), asg, None, fake, 16, None)
    assert rc == -2 and b"workspace" in lib.orch_last_error()
    rc = lib.orch_balance_tolerance(fake, 8, 2000, 5, B._Phase(1, 1), asg, fake, 1 << 20, None)
    assert rc == -3 and b"1024" in lib.orch_last_error()
    rc = lib.orch_balance_tolerance(fake, -2, 4, 5, B._Phase(1, 1), asg, fake, 1 << 20, None)
    assert rc == -1
    rc = lib.orch_comm_volume(fake, 8, 0, None, 4, asg, fake, 0, None, None)
    assert rc == -1 and b"D_src" in lib.orch_last_error()
    rc = lib.orch_comm_volume(fake, 8, 4, None, 4, asg, None, 0, None, None)
    assert rc == -1 and b"V is NULL" in lib.orch_last_error()
    rc = lib.orch_pack(fake, fake, fake, 8, 4, 10, 0, 10, asg, 0, 4, fake, 1 << 20, None)
    assert rc == -1
    rc = lib.orch_pack(fake, fake, fake, 8, 4, 10, 64, 10, asg, 2, 5, fake, 1 << 20, None)
    assert rc == -1
    assert lib.orch_pack_composed_workspace(32768) >= 32768 * 32
    rc = lib.orch_pack_composed(fake, fake, fake, fake, 8, 0, None, 4, asg, 10, 64, 10, 2, 5, fake, 1 << 20, None)
    assert rc == -1 and b"instance range" in lib.orch_last_error()
    rc = lib.orch_pack_composed(fake, fake, fake, fake, 8, 0, ctypes.byref(asg), 4, asg, 10, 64, 10, 0, 4, fake,
                                1 << 20, None)
    assert rc == -1 and b"D_src" in lib.orch_last_error()
    rc = lib.orch_pack_composed(fake, fake, fake, None, 8, 0, None, 4, asg, 10, 64, 10, 0, 4, fake, 1 << 20, None)
    assert rc == -1 and b"sub_off" in lib.orch_last_error()
    rc = lib.orch_pack_composed(fake, fake, fake, fake, 8, 0, None, 4, asg, 10, 64, 10, 0, 4, fake, 64, None)
    assert rc == -2 and b"workspace" in lib.orch_last_error()
    rc = lib.orch_varlen_attn_fwd(fake, fake, fake, fake, None, fake, 2, 64, 0, 8, 3, 64, 0.0, 1, None, fake,
                                  1 << 20, None)
    assert rc == -1
    rc = lib.orch_varlen_attn_fwd(fake, fake, fake, fake, None, fake, 2, 64, 0, 8, 4, 96, 0.0, 1, None, fake,
                                  1 << 20, None)
    assert rc == -3 and b"head_dim" in lib.orch_last_error()
    rc = lib.orch_varlen_attn_fwd(fake, fake, fake, fake, None, fake, 2, 64, 0, 8, 4, 64, 0.0, 1, None, fake,
                                  8, None)
    assert rc == -2
    assert lib.orch_varlen_attn_bwd_workspace(4, 1000, 8) >= 1000 * 8 * 4
    bwd = lambda lse, d, wsb: lib.orch_varlen_attn_bwd(fake, fake, fake, fake, lse, fake, fake, fake, fake, fake,
                                                       2, 64, 0, 8, 4, d, 0.0, 1, None, fake, wsb, None)
    assert bwd(None, 64, 1 << 20) == -1 and b"lse" in lib.orch_last_error()
    assert bwd(fake, 96, 1 << 20) == -3
    assert bwd(fake, 64, 8) == -2
