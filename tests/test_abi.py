"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching a GPU."""
import ctypes as C
import os
import re

import pytest

import paper_2507_16099_amd as fp8

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "fp8mi355.h")


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(fp8_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    lib = fp8.load_library()
    names = _declared()
    assert {"fp8_amax", "fp8_scale", "fp8_cast", "fp8_scaled_mm", "fp8_linear_fwd", "fp8_linear_bwd",
            "fp8_quantize", "fp8_quantize_row_col", "fp8_linear_fwd_prequantized", "fp8_grad_weight_hp", "fp8_mx_quantize", "fp8_mx_scaled_mm", "fp8_mx_linear_fwd", "fp8_mx_linear_workspace_bytes",
            "fp8_layernorm_quantize", "fp8_block_quantize", "fp8_block_linear_workspace_bytes", "fp8_block_linear_fwd", "fp8_block_quantize_t", "fp8_block_quantize_row_col", "fp8_block_linear_bwd_workspace_bytes", "fp8_block_linear_bwd", "fp8_linear_bwd_sigmoid", "fp8_linear_bwd_sigmoid_workspace_bytes", "fp8_mx_quantize_t", "fp8_mx_quantize_row_col", "fp8_mx_linear_bwd", "fp8_mx_linear_bwd_workspace_bytes",
            "fp8_linear_prequantized_workspace_bytes", "fp8_linear_workspace_bytes", "fp8_last_error", "fp8_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert "gfx950" in fp8.fp8_version()


def test_binding_has_the_same_names():
    for n in _declared():
        assert callable(getattr(fp8, n)), n


def test_enum_values_match_header():
    src = open(HEADER).read()
    for name in ("FP8_E4M3FN", "FP8_E5M2", "FP8_TENSOR", "FP8_ROW", "FP8_COL", "FP8_POW2_SCALE",
                 "FP8_TRANSPOSE_OUT", "FP8_OUT_FP32", "FP8_GRAD_WEIGHT_HP", "FP8_SAVE_FOR_BWD", "FP8_EPILOGUE_SIGMOID"):
        m = re.search(name + r"\s*=\s*(-?\d+)", src)
        assert m and int(m.group(1)) == getattr(fp8, name), name


def test_argument_errors_are_reported_without_a_gpu():
    L = fp8.load_library()
    buf = (C.c_char * 4096)()
    p = C.addressof(buf)
    p16 = (p + 15) // 16 * 16
    # NULL input
    assert L.fp8_amax(None, 4, 8, 8, 0, p16, None) == -1
    assert "NULL" in fp8.fp8_last_error()
    # unknown granularity / format / flag bits
    assert L.fp8_amax(p16, 4, 8, 8, 7, p16, None) == -3
    assert L.fp8_scale(p16, 4, 9, 0, p16, None) == -3
    assert L.fp8_cast(p16, 4, 8, 8, p16, 0, 0, 64, p16, 16, None) == -3
    # shapes
    assert L.fp8_amax(p16, -1, 8, 8, 0, p16, None) == -2
    assert L.fp8_amax(p16, 4, 16, 8, 0, p16, None) == -2            # ld < cols
    assert L.fp8_scaled_mm(p16, 16, 0, p16, 0, p16, 16, 0, p16, 0, 4, 4, 8, p16, 8, 0, None) == -2   # K % 16
    # alignment
    assert L.fp8_amax(p16 + 2, 4, 8, 8, 0, p16, None) == -4
    assert L.fp8_amax(p16, 4, 8, 12, 0, p16, None) == -4            # ld % 8
    assert L.fp8_cast(p16, 4, 16, 16, p16, 0, 0, 0, p16, 24, None) == -4   # ld_out % 16
    assert fp8.fp8_last_error() != ""
    # recipe checks and workspace size
    r = fp8.Recipe(gran=fp8.FP8_COL).c()
    assert L.fp8_linear_workspace_bytes(64, 64, 64, C.byref(r), 0) == 0
    r = fp8.Recipe(gran=fp8.FP8_ROW).c()
    n = L.fp8_linear_workspace_bytes(64, 128, 32, C.byref(r), 0)
    assert n >= 64 * 128 + 32 * 128 + 4 * (64 + 32)
    nb = L.fp8_linear_workspace_bytes(64, 128, 32, C.byref(r), 1)
    assert nb >= 2 * 64 * 32 + 128 * 32 + 128 * 64
    assert L.fp8_linear_fwd(p16, p16, 64, 128, 32, C.byref(r), p16, p16, 16, None) in (-4, -5)
    assert L.fp8_linear_fwd(p16, p16, 64, 120, 32, C.byref(r), p16, p16, 1 << 20, None) == -2


def test_argument_errors_of_the_later_entry_points():
    """The entry points added for the weight-gradient-in-bf16 recipe, inference
    with pre-quantized weights and MX block scaling reject bad arguments on the
    host, before any launch."""
    L = fp8.load_library()
    buf = (C.c_char * 8192)()
    p = (C.addressof(buf) + 255) // 256 * 256
    # fp8_quantize_row_col: format, leading dimensions
    assert L.fp8_quantize_row_col(p, 64, 64, 64, 5, 0, p, 64, p, p, 64, p, None) == -3
    assert L.fp8_quantize_row_col(p, 64, 64, 32, 0, 0, p, 64, p, p, 64, p, None) == -2
    # fp8_grad_weight_hp: NULL output, ragged dims
    assert L.fp8_grad_weight_hp(p, p, 64, 64, 64, None, None) == -1
    assert L.fp8_grad_weight_hp(p, p, 64, 60, 64, p, None) == -2
    # prequantized forward: granularity of the weight scales, workspace too small
    assert L.fp8_linear_fwd_prequantized(p, 16, 64, 0, 1, 0, p, 64, 0, p, 2, 32, p, 32, p, 1 << 20, None) == -3
    assert L.fp8_linear_fwd_prequantized(p, 16, 64, 0, 1, 0, p, 64, 0, p, 1, 32, p, 32, p, 16, None) == -5
    assert L.fp8_linear_prequantized_workspace_bytes(16, 64) >= 16 * 64 + 16 * 4
    # the variant with the static scratch buffer: same checks, and sizes beyond the buffer are refused on the host
    assert L.fp8_linear_fwd_prequantized_static(p, 16, 64, 0, 1, 0, p, 64, 0, p, 2, 32, p, 32, None) == -3
    assert L.fp8_linear_fwd_prequantized_static(p, 4096, 4096, 0, 1, 0, p, 4096, 0, p, 1, 64, p, 64, None) == -5
    assert "static buffer" in fp8.fp8_last_error()
    # MX: block size, scale leading dimension, contraction length of the GEMM
    assert L.fp8_mx_quantize(p, 4, 48, 48, 0, p, 48, p, 4, None) == -2
    assert L.fp8_mx_quantize(p, 4, 64, 64, 0, p, 64, p, 2, None) == -2           # ld_e % 4
    assert L.fp8_mx_quantize_t(p, 48, 64, 64, 0, p, 48, p, 4, None) == -2         # rows % 32
    assert L.fp8_mx_quantize_t(p, 64, 64, 64, 7, p, 64, p, 4, None) == -3
    assert L.fp8_mx_scaled_mm(p, 64, 0, p, 4, p, 64, 0, p, 4, 16, 16, 64, p, 16, 0, None) == -2   # K % 128
    assert L.fp8_mx_scaled_mm(p, 128, 0, p, 4, p, 128, 0, p, 4, 16, 16, 128, p, 16, 8, None) == -3  # unknown flag
    # scale slabs (negative ld_e): whole slabs of sixteen blocks, enough rows per slab, both operands of a product alike
    assert L.fp8_mx_quantize(p, 4, 256, 256, 0, p, 256, p, -4, None) == -2        # 8 blocks per row: not a multiple of 16
    assert "512" in fp8.fp8_last_error()
    assert L.fp8_mx_quantize(p, 4, 512, 512, 0, p, 512, p, -3, None) == -2        # 3 rows per slab for 4 rows
    assert L.fp8_mx_quantize(p + 4, 4, 512, 512, 0, p, 512, p + 4, -4, None) == -4    # slabs 16-byte aligned
    assert L.fp8_mx_quantize_t(p, 512, 8, 8, 0, p, 512, p, -7, None) == -2        # 8 scale rows
    assert L.fp8_mx_scaled_mm(p, 512, 0, p, -16, p, 512, 0, p, 16, 16, 16, 512, p, 16, 0, None) == -2   # slabs and plain rows mixed
    assert "both" in fp8.fp8_last_error()
    assert L.fp8_mx_scaled_mm(p, 512, 0, p, -8, p, 512, 0, p, -16, 16, 16, 512, p, 16, 0, None) == -2   # 8 rows per slab for M = 16
    assert L.fp8_mx_scaled_mm(p, 256, 0, p, -16, p, 256, 0, p, -16, 16, 16, 256, p, 16, 0, None) == -2  # K % 512
    assert L.fp8_mx_linear_workspace_bytes(16, 96, 16) == 0
    assert L.fp8_mx_linear_bwd_workspace_bytes(100, 64, 128) == 0                # M % 32
    assert L.fp8_mx_linear_bwd_workspace_bytes(96, 64, 160) >= 96 * 256 + 64 * 256 + 160 * 128 + 64 * 128   # padded to 128
    assert L.fp8_block_linear_bwd_workspace_bytes(96, 64, 128) == 0              # blockwise tiles: M % 128
    assert L.fp8_mx_linear_bwd_workspace_bytes(128, 64, 256) >= 2 * 128 * 256 + 64 * 256 + 64 * 128
    assert L.fp8_mx_linear_bwd(p, p, p, 128, 64, 128, 0, 0, 9, p, p, p, 1 << 20, None) == -3
    assert L.fp8_mx_linear_bwd(p, p, p, 128, 64, 128, 0, 0, 0, p, p, p, 16, None) == -5
    assert L.fp8_mx_linear_bwd(p, p, p, 128, 64, 128, 0, 0, 0, None, None, p, 16, None) == 0   # nothing asked for
    assert "workspace" in fp8.fp8_last_error() or fp8.fp8_last_error() == ""


def test_missing_library_fails_loudly(monkeypatch):
    import paper_2507_16099_amd.fp8 as mod
    monkeypatch.setattr(mod, "_lib", None)
    monkeypatch.setattr(mod, "_LIB_PATH", "/nonexistent/libfp8mi355.so")
    with pytest.raises(ImportError):
        mod.load_library()


def test_product_does_not_reach_the_oracle():
    """No file of the GPU package mentions the oracle, and vice versa."""
    pkg = os.path.join(ROOT, "paper_2507_16099_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                assert "oracle" not in open(os.path.join(dirpath, f)).read().lower(), f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            txt = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2507_16099_amd" not in txt and "fp8mi355" not in txt, f
