"""The C-ABI library loads and exports every function include/flowprefill.h declares (no compute
call is made here, so this runs without a GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "flowprefill.h")
LIB = os.path.join(ROOT, "paper_2602_16603_amd", "libflowprefill.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fp_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_boundary_calls():
    names = declared_functions()
    for must in ("fp_model_create", "fp_prefill_begin", "fp_prefill_advance", "fp_preempt", "fp_resume"):
        assert must in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        from paper_2602_16603_amd.csrc.build import build
        build(verbose=False)
    lib = ctypes.CDLL(LIB)
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in the header but not exported"


def test_binding_covers_every_declared_symbol():
    from paper_2602_16603_amd import binding
    assert sorted(binding.EXPORTED) == declared_functions()
    assert binding.fp_version().startswith("flowprefill")


def test_status_paths_that_need_no_device():
    from paper_2602_16603_amd import binding as B
    import pytest
    shape = B.fp_shape(1, 64, 2, 2, 24, 64, 1e-5, 1e4, 1, 16, 4, 16)     # head_dim 24: invalid
    with pytest.raises(B.FlowPrefillError) as e:
        B.fp_model_create(shape, [dict(attn_norm=16, w_qkv=16, w_o=16, mlp_norm=16, w_gate_up=16, w_down=16)])
    assert e.value.status == B.FP_ERR_INVALID
    shape = B.fp_shape(1, 64, 3, 2, 64, 64, 1e-5, 1e4, 1, 16, 4, 16)     # 3 q heads over 2 kv heads
    with pytest.raises(B.FlowPrefillError):
        B.fp_model_create(shape, [dict(attn_norm=16, w_qkv=16, w_o=16, mlp_norm=16, w_gate_up=16, w_down=16)])
    assert "multiple" in B.fp_last_error()
