"""CPU-side checks of the boundary: the shared library loads, exports every
function include/d2c.h declares, and fails loudly (no fallback) without a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "d2c.h")
TOOLS_HEADER = os.path.join(ROOT, "include", "d2c_tools.h")
LIB = os.path.join(ROOT, "paper_2509_23094_amd", "libd2c.so")


def _declared_functions(path=HEADER):
    text = open(path).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(d2c_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_four_calls():
    names = _declared_functions()
    for need in ("d2c_init", "d2c_select", "d2c_refresh_layer", "d2c_step", "d2c_destroy", "d2c_last_error"):
        assert need in names


@pytest.mark.skipif(not os.path.exists(LIB), reason="libd2c.so not built (run __graft_entry__.build())")
def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(LIB)
    for name in _declared_functions() + _declared_functions(TOOLS_HEADER):
        assert getattr(lib, name) is not None


@pytest.mark.skipif(not os.path.exists(LIB), reason="libd2c.so not built (run __graft_entry__.build())")
def test_binding_names_match_header():
    from paper_2509_23094_amd import binding
    assert sorted(binding.EXPORTS) == _declared_functions()
    assert sorted(binding.TOOL_EXPORTS) == _declared_functions(TOOLS_HEADER)
    for name in ("d2c_select", "d2c_refresh_layer", "d2c_step", "d2c_attention", "d2c_influence", "d2c_seq_reset", "d2c_linear"):
        assert hasattr(binding.Context, name)


@pytest.mark.skipif(not os.path.exists(LIB), reason="libd2c.so not built (run __graft_entry__.build())")
def test_argument_errors_need_no_gpu():
    from paper_2509_23094_amd import binding as B
    lib = B._lib
    out = ctypes.c_void_p()
    assert lib.d2c_init(None, None, ctypes.byref(out)) == B.D2C_EINVAL
    d = B.d2c_dims(2, 256, 4, 4, 64, 688, 1024, 128, 7, 1e-5, 1e4, 1023)          # dtype 7 does not exist
    w = B.d2c_weights()
    assert lib.d2c_init(ctypes.byref(d), ctypes.byref(w), ctypes.byref(out)) == B.D2C_EINVAL
    assert b"dtype" in lib.d2c_last_error(None)
    d.dtype = B.D2C_F32
    d.n_kv_heads = 3                                                              # 4 heads over 3 KV heads
    assert lib.d2c_init(ctypes.byref(d), ctypes.byref(w), ctypes.byref(out)) == B.D2C_EINVAL
    d.n_kv_heads = 4
    assert lib.d2c_init(ctypes.byref(d), ctypes.byref(w), ctypes.byref(out)) == B.D2C_EINVAL   # null weights
    assert b"weight" in lib.d2c_last_error(None)
    assert lib.d2c_step(None, None, None, 1, None) == B.D2C_EINVAL
    assert lib.d2c_destroy(None) == B.D2C_OK
    assert lib.d2c_ctx_set_tunable(None, b"gemm_waves", 8) == B.D2C_EINVAL
    bad = (B.d2c_tunable * 1)(B.d2c_tunable(b"no_such_knob", 1))
    d2 = B.d2c_dims(2, 256, 4, 4, 64, 688, 1024, 128, B.D2C_F32, 1e-5, 1e4, 1023)
    assert lib.d2c_init_tuned(ctypes.byref(d2), ctypes.byref(w), bad, 1, ctypes.byref(out)) == B.D2C_EINVAL
    assert b"no_such_knob" in lib.d2c_last_error(None)
