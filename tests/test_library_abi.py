"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and rejects bad arguments before anything is launched (no GPU needed)."""
import ctypes
import os
import re

import pytest

import paper_2511_23225_amd as tw
from paper_2511_23225_amd import build as tw_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(tw.LIB_PATH):
        tw_build.build_library()
    return tw.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "tweo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tweo_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert len(names) >= 11
    for n in names:
        assert hasattr(lib, n), n
    assert set(tw.binding.EXPORTS) == set(names)


def test_status_strings(lib):
    seen = {tw.status_string(i) for i in range(5)}
    assert len(seen) == 5 and "ok" in seen


def test_workspace_bytes(lib):
    for op in range(6):
        b = tw.tweo_workspace_bytes(op, 8192, 2304, 768)
        assert b >= 256 and b % 256 == 0
    assert tw.tweo_workspace_bytes(0, 16384, 6144, 2048) >= 4 * (16384 // 256) * (6144 // 256)
    assert tw.tweo_workspace_bytes(0, 0, 0, 0) == 256


def test_invalid_arguments_are_rejected_without_a_gpu(lib):
    vp = ctypes.c_void_p
    buf = ctypes.create_string_buffer(4096)
    p = vp((ctypes.addressof(buf) + 15) & ~15)
    odd = vp(p.value + 2)
    assert lib.tweo_amax(None, 8, p, None) == tw.TWEO_ERR_INVALID_ARG
    assert lib.tweo_amax(p, 0, p, None) == tw.TWEO_ERR_INVALID_ARG
    assert lib.tweo_amax(odd, 8, p, None) == tw.TWEO_ERR_INVALID_ARG
    assert lib.tweo_quantize_e4m3(p, 8, 12, p, p, None, None, None, None) == tw.TWEO_ERR_UNSUPPORTED
    assert lib.tweo_quantize_e4m3(p, 8, 16, None, p, None, None, None, None) == tw.TWEO_ERR_INVALID_ARG
    assert lib.tweo_fp8_linear_fwd(p, p, p, p, None, 16, 16, 24, p, None, None, None, 0, None) == \
        tw.TWEO_ERR_UNSUPPORTED
    assert lib.tweo_fp8_linear_fwd(p, p, p, p, None, 16, -1, 16, p, None, None, None, 0, None) == \
        tw.TWEO_ERR_INVALID_ARG
    pen = tw.binding.PenaltyCfg(3.0, 1e-6, 4)
    assert lib.tweo_fp8_linear_fwd(p, p, p, p, None, 16, 16, 16, p, ctypes.byref(pen), p, None, 0,
                                   None) == tw.TWEO_ERR_WORKSPACE
    assert lib.tweo_fp8_linear_fwd(p, p, p, p, None, 16, 16, 16, p, ctypes.byref(pen), p, p, 4,
                                   None) == tw.TWEO_ERR_WORKSPACE
    bad = tw.binding.PenaltyCfg(3.0, 1e-6, 11)
    assert lib.tweo_fp8_linear_fwd(p, p, p, p, None, 16, 16, 16, p, ctypes.byref(bad), p, p, 4096,
                                   None) == tw.TWEO_ERR_UNSUPPORTED
    neg = tw.binding.PenaltyCfg(-1.0, 1e-6, 4)
    assert lib.tweo_fp8_linear_fwd(p, p, p, p, None, 16, 16, 16, p, ctypes.byref(neg), p, p, 4096,
                                   None) == tw.TWEO_ERR_INVALID_ARG
    assert lib.tweo_fp8_linear_bwd(p, p, p, p, p, p, p, 16, 16, 16, None, None, None, 0, None) == \
        tw.TWEO_ERR_INVALID_ARG
    assert lib.tweo_fp8_linear_bwd(p, p, p, p, p, p, p, 16, 24, 16, p, None, None, 0, None) == \
        tw.TWEO_ERR_UNSUPPORTED
    assert lib.tweo_quantize_i8(p, 12, 1.0, p, None) == tw.TWEO_ERR_UNSUPPORTED
    assert lib.tweo_quantize_i8(p, 16, float("nan"), p, None) == tw.TWEO_ERR_INVALID_ARG
    assert lib.tweo_w8a8_linear(p, p, 4, 16, 8, 1.0, p, None, 0, None) == tw.TWEO_ERR_UNSUPPORTED
    assert lib.tweo_w8a8_linear(p, None, 4, 16, 16, 1.0, p, None, 0, None) == tw.TWEO_ERR_INVALID_ARG
    # LayerNorm -> cast: every check comes before the first launch
    ln = lib.tweo_layernorm_quantize_e4m3
    assert ln(p, None, p, None, 16, 16, 1e-5, None, None, None, p, None, None, None, None, 0, None) == \
        tw.TWEO_ERR_WORKSPACE
    assert ln(p, None, p, None, 16, 16, 1e-5, None, None, None, p, None, None, None, p, 64, None) == \
        tw.TWEO_ERR_WORKSPACE
    assert ln(p, None, None, None, 16, 16, 1e-5, None, None, None, p, None, None, None, p, 4096, None) == \
        tw.TWEO_ERR_INVALID_ARG
    assert ln(p, p, p, None, 16, 16, 1e-5, None, None, None, p, None, None, None, p, 4096, None) == \
        tw.TWEO_ERR_INVALID_ARG      # a residual without a place for h
    assert ln(p, None, p, None, 16, 24, 1e-5, None, None, None, p, None, None, None, p, 4096, None) == \
        tw.TWEO_ERR_UNSUPPORTED
    assert ln(p, None, p, None, 16, 16, float("nan"), None, None, None, p, None, None, None, p, 4096, None) == \
        tw.TWEO_ERR_INVALID_ARG
    assert lib.tweo_layernorm_quantize_e4m3_delayed(p, None, p, None, 16, 16, 1e-5, None, 0, None, None, p, None, p,
                                                    4096, None) == tw.TWEO_ERR_INVALID_ARG   # no state
    assert tw.tweo_workspace_bytes(tw.TWEO_OP_LAYERNORM_QUANTIZE, 16384, 1, 1) == 2304 + 16384 * 16
    assert lib.tweo_set_gemm_tile(99) == tw.TWEO_ERR_INVALID_ARG
    assert lib.tweo_set_gemm_tile(12) == tw.TWEO_ERR_INVALID_ARG   # a retired variant
    assert lib.tweo_set_gemm_tile(17) == tw.TWEO_OK
    assert lib.tweo_set_gemm_tile(0) == tw.TWEO_OK


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2511_23225_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "tweo_oracle" not in text, f
