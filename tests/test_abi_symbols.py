"""The C-ABI library loads and exports every function include/moe.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions(header="moe.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_hot_path_calls():
    names = declared_functions()
    for n in ["moe_gate_topk", "moe_permute", "moe_grouped_ffn_fwd", "moe_grouped_ffn_bwd",
              "moe_unpermute_combine", "moe_combine_bwd", "moe_gate_topk_bwd", "moe_workspace_bytes"]:
        assert n in names


def test_library_exports_every_declared_symbol():
    from paper_2602_11686_amd import binding as B
    if not os.path.exists(B.LIB_PATH):
        pytest.skip("libmoe.so not built (run python -m paper_2602_11686_amd.build)")
    L = ctypes.CDLL(B.LIB_PATH)
    for n in declared_functions():
        assert hasattr(L, n), n
    assert sorted(B.EXPORTS) == declared_functions()
    from paper_2602_11686_amd import planner
    for n in declared_functions("moe_planner.h"):
        assert hasattr(L, n), n
    assert sorted(planner.PLANNER_EXPORTS) == declared_functions("moe_planner.h")
    from paper_2602_11686_amd import fsep
    for n in declared_functions("moe_fsep.h"):
        assert hasattr(L, n), n
    assert sorted(fsep.FSEP_EXPORTS) == declared_functions("moe_fsep.h")


def test_host_side_validation_needs_no_gpu():
    """Bad shapes are rejected on the host before anything is launched."""
    from paper_2602_11686_amd import binding as B
    import torch
    if not os.path.exists(B.LIB_PATH):
        pytest.skip("libmoe.so not built")
    assert B.moe_workspace_bytes(B.Shape(256, 128, 256, 8, 2, torch.float32)) > 0
    for bad in [B.Shape(0, 128, 256, 8, 2, torch.float32), B.Shape(16, 128, 256, 8, 9, torch.float32),
                B.Shape(16, 130, 256, 8, 2, torch.bfloat16), B.Shape(16, 128, 256, 1000, 2, torch.bfloat16)]:
        with pytest.raises(B.MoeError):
            B.moe_workspace_bytes(bad)
    L = B.lib()
    c = B.Shape(16, 128, 256, 8, 2, torch.float32).c()
    # NULL pointer -> MOE_ERR_INVALID_ARG (1), nothing launched
    st = L.moe_unpermute_combine(ctypes.byref(c), None, None, None, None, None)
    assert st == 1 and b"NULL" in L.moe_last_error()
    # misaligned pointer
    st = L.moe_unpermute_combine(ctypes.byref(c), ctypes.c_void_p(8), ctypes.c_void_p(16), None, ctypes.c_void_p(16), None)
    assert st == 1 and b"aligned" in L.moe_last_error()
    # workspace too small -> 3
    st = L.moe_permute(ctypes.byref(c), ctypes.c_void_p(16), ctypes.c_void_p(16), ctypes.c_void_p(16), ctypes.c_void_p(16),
                       ctypes.c_void_p(16), ctypes.c_void_p(16), ctypes.c_void_p(16), ctypes.c_void_p(16), ctypes.c_size_t(1), None)
    assert st == 3
    assert L.moe_status_string(3) == b"workspace too small"


def test_grouped_gemm_calls_refuse_to_run_without_a_supported_device():
    """Where no GPU can be queried the grouped-GEMM entry points return MOE_ERR_DEVICE before launching anything
    (on a GPU machine this test is skipped: the fake pointers below must never reach a kernel)."""
    from paper_2602_11686_amd import binding as B
    import torch
    if not os.path.exists(B.LIB_PATH):
        pytest.skip("libmoe.so not built")
    if torch.cuda.is_available():
        pytest.skip("a GPU is present: the device check passes and the call would launch")
    L = B.lib()
    c = B.Shape(64, 128, 256, 4, 2, torch.bfloat16).c()
    p = ctypes.c_void_p(4096)
    big = ctypes.c_size_t(1 << 40)
    st = L.moe_grouped_ffn_fwd(ctypes.byref(c), p, p, p, p, p, p, None, None, p, big, None)
    assert st == 4 and b"GPU" in L.moe_last_error()
    st = L.moe_grouped_ffn_bwd(ctypes.byref(c), p, p, p, p, p, None, None, p, p, p, p, p, p, big, None)
    assert st == 4
    st = L.moe_gate_topk_bwd(ctypes.byref(c), p, p, p, p, p, p, p, p, big, None)
    assert st == 4
    # argument errors still come first
    st = L.moe_grouped_ffn_fwd(ctypes.byref(c), None, p, p, p, p, p, None, None, p, big, None)
    assert st == 1
    # the pair that saves products: all three saved tensors are required; no workspace in the forward call
    st = L.moe_grouped_ffn_fwd_products(ctypes.byref(c), p, p, p, p, p, p, p, p, p, None)
    assert st == 4 and b"GPU" in L.moe_last_error()
    st = L.moe_grouped_ffn_fwd_products(ctypes.byref(c), p, p, p, p, p, p, p, None, p, None)
    assert st == 1 and b"p_save" in L.moe_last_error()
    st = L.moe_grouped_ffn_bwd_products(ctypes.byref(c), p, p, p, p, p, p, p, p, p, p, p, p, p, p, big, None)
    assert st == 4
    st = L.moe_grouped_ffn_bwd_products(ctypes.byref(c), p, p, p, p, p, None, p, p, p, p, p, p, p, p, big, None)
    assert st == 1 and b"h_save" in L.moe_last_error()
    st = L.moe_grouped_ffn_bwd_products(ctypes.byref(c), p, p, p, p, p, p, p, p, p, p, p, p, p, p, ctypes.c_size_t(8), None)
    assert st in (3, 4)   # (the workspace check sits behind the device check)


def test_one_time_kernel_attributes_are_set_under_a_lock():
    """The launch helpers hold no unsynchronised `static bool` flags any more."""
    csrc = os.path.join(ROOT, "paper_2602_11686_amd", "csrc")
    for name in os.listdir(csrc):
        text = open(os.path.join(csrc, name)).read()
        assert not re.search(r"static\s+(thread_local\s+)?bool\s+attr", text), name
