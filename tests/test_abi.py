"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, sizes buffers as documented and turns bad arguments into error codes."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2306_08960_amd", "libapb.so")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="libapb.so not built (run __graft_entry__.build())")


def _declared():
    text = open(os.path.join(ROOT, "include", "apb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(apb_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = ctypes.CDLL(LIB)
    names = _declared()
    assert len(names) >= 10
    for n in names:
        assert hasattr(lib, n), n


def test_binding_names_match_header():
    from paper_2306_08960_amd import binding
    assert sorted(binding.EXPORTS) == _declared()
    for n in binding.EXPORTS:
        if n not in ("apb_layer_free", "apb_w2_free", "apb_strerror", "apb_last_hip_error"):
            assert hasattr(binding, n), n


def test_acts_bytes():
    from paper_2306_08960_amd import binding as b
    assert b.apb_acts_bytes(32, 64, 1) == 4 * 64 * (1 + 1)
    assert b.apb_acts_bytes(33, 65, 2) == 4 * 128 * (2 * 2 + 1)
    assert b.apb_acts_bytes(576, 131072, 2) == 4 * 131072 * (2 * 18 + 1)
    assert b.apb_acts_bytes(0, 5, 1) == 0 and b.apb_acts_bytes(5, -1, 1) == 0
    assert b.apb_acts_bytes(5, 5, 3) == 0 and b.apb_acts_bytes(2 ** 30, 5, 1) == 0


def test_argument_errors_without_touching_the_gpu():
    from paper_2306_08960_amd import binding as b
    lib = b.load()
    out = ctypes.c_void_p(123)
    nan = float("nan")
    assert lib.apb_compress(None, 4, 4, 0.1, nan, None, ctypes.byref(out)) == b.APB_ERR_NULL
    assert out.value is None
    fake = ctypes.c_void_p(4096)       # never dereferenced: every call below fails validation first
    assert lib.apb_compress(fake, 4, 4, 0.1, nan, None, None) == b.APB_ERR_NULL
    assert lib.apb_compress(fake, 0, 4, 0.1, nan, None, ctypes.byref(out)) == b.APB_ERR_SHAPE
    assert lib.apb_compress(fake, 4, -1, 0.1, nan, None, ctypes.byref(out)) == b.APB_ERR_SHAPE
    assert lib.apb_compress(fake, 65536, 65536, 0.1, nan, None, ctypes.byref(out)) == b.APB_ERR_SHAPE
    assert lib.apb_compress(fake, 4, 4, nan, 0.1, None, ctypes.byref(out)) == b.APB_ERR_VALUE
    assert lib.apb_compress(fake, 4, 4, 0.1, -1.0, None, ctypes.byref(out)) == b.APB_ERR_VALUE
    assert lib.apb_compress(fake, 4, 4, 0.1, float("inf"), None, ctypes.byref(out)) == b.APB_ERR_VALUE
    assert lib.apb_quantize_acts(None, 4, 4, 1, 1.0, fake, None) == b.APB_ERR_NULL
    assert lib.apb_quantize_acts(fake, 4, 4, 1, 1.0, None, None) == b.APB_ERR_NULL
    assert lib.apb_quantize_acts(fake, 0, 4, 1, 1.0, fake, None) == b.APB_ERR_SHAPE
    assert lib.apb_quantize_acts(fake, 4, 4, 3, 1.0, fake, None) == b.APB_ERR_BITS
    for bad in (0.0, -1.0, nan, float("inf")):
        assert lib.apb_quantize_acts(fake, 4, 4, 2, bad, fake, None) == b.APB_ERR_VALUE
    assert lib.apb_forward(None, fake, 4, 1, 1.0, fake, None) == b.APB_ERR_NULL
    assert lib.apb_forward_int(None, fake, 4, 1, fake, None) == b.APB_ERR_NULL
    assert lib.apb_quantize_forward(None, fake, 4, 1, 1.0, fake, fake, None) == b.APB_ERR_NULL
    assert lib.apb_quantize_forward_is_one_kernel(None, 4, 1) == 0
    assert lib.apb_forward_requant(None, fake, 4, 1, 1.0, None, None, 2, 1.0, fake, None) == b.APB_ERR_NULL
    assert lib.apb_forward_conv3x3(None, fake, 1, 4, 4, 1, 2, 1.0, None, 0, fake, None) == b.APB_ERR_NULL
    assert lib.apb_forward_conv3x3_requant(None, fake, 1, 4, 4, 1, 2, 1.0, None, None, 2, 1.0, None, 0, fake, None) == b.APB_ERR_NULL
    assert lib.apb_layer_info(None, None, None, None, None, None) == b.APB_ERR_NULL
    assert lib.apb_layer_export(None, None, None, None, None, None, None) == b.APB_ERR_NULL
    lib.apb_layer_free(None)
    # 2/2 routine
    assert lib.apb_w2_pack(None, 4, 4, 0.1, None, ctypes.byref(out)) == b.APB_ERR_NULL
    assert lib.apb_w2_pack(fake, 4, 4, 0.1, None, None) == b.APB_ERR_NULL
    assert lib.apb_w2_pack(fake, 0, 4, 0.1, None, ctypes.byref(out)) == b.APB_ERR_SHAPE
    for bad in (0.0, -1.0, nan, float("inf")):
        assert lib.apb_w2_pack(fake, 4, 4, bad, None, ctypes.byref(out)) == b.APB_ERR_VALUE
    assert out.value is None
    assert lib.apb_w2_export(None, fake, None) == b.APB_ERR_NULL
    assert lib.apb_gemm_2_2_int(None, fake, 4, fake, None) == b.APB_ERR_NULL
    assert lib.apb_gemm_2_2(None, fake, 4, 1.0, fake, None) == b.APB_ERR_NULL
    lib.apb_w2_free(None)
    for code in range(-6, 1):
        assert b.strerror(code) and "unknown" not in b.strerror(code)
    assert "unknown" in b.strerror(-99)


def test_product_and_oracle_share_nothing():
    """Neither side imports the other; the oracle is not reachable from the product package."""
    pkg = os.path.join(ROOT, "paper_2306_08960_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                assert "oracle" not in open(os.path.join(dirpath, f)).read().lower() or f == "synth.py", f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            assert "paper_2306_08960_amd" not in open(os.path.join(ROOT, "oracle", f)).read(), f
