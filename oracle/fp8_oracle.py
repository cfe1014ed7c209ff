"""ctypes front end of the CPU oracle (``fp8_oracle.c``) plus the linear-layer
compositions.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's ``cpu_baseline`` leg.  The GPU library never imports this module
and this module never imports the GPU library.

Arrays are numpy: bfloat16 tensors are ``uint16`` bit patterns, fp8 tensors are
``uint8`` codes, scales are ``float32``.

The compositions follow the paper's Appendix A: a tensorwise recipe keeps one
scale per tensor; the rowwise recipe scales the left operand of each GEMM per
row and the right operand per column, i.e. every operand is (re)quantized
along the contraction axis of the GEMM it feeds.  The three GEMMs of a linear
layer are Y = X W^T, dX = dY W and dW = dY^T X.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

E4M3FN, E5M2 = 0, 1
TENSOR, ROW, COL = 0, 1, 2
POW2_SCALE, TRANSPOSE_OUT = 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fp8_oracle.c")
_LIB = os.path.join(_HERE, "libfp8oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off: every fp32 operation
    rounds once, no fused multiply-add."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        i64, vp, ci, f32 = C.c_int64, C.c_void_p, C.c_int, C.c_float
        L.orc_bf16_to_f32.restype = f32
        L.orc_bf16_to_f32.argtypes = [C.c_uint16]
        L.orc_f32_to_bf16.restype = C.c_uint16
        L.orc_f32_to_bf16.argtypes = [f32]
        L.orc_num_threads.restype = ci
        L.orc_fp8_max.restype = f32
        L.orc_fp8_max.argtypes = [ci]
        L.orc_fp8_decode.restype = f32
        L.orc_fp8_decode.argtypes = [C.c_uint8, ci]
        L.orc_fp8_encode_search.restype = C.c_uint8
        L.orc_fp8_encode_search.argtypes = [f32, ci]
        L.orc_fp8_encode_bits.restype = C.c_uint8
        L.orc_fp8_encode_bits.argtypes = [f32, ci]
        L.orc_fp8_encode_array.restype = None
        L.orc_fp8_encode_array.argtypes = [vp, i64, ci, ci, vp]
        L.orc_f32_to_bf16_array.restype = None
        L.orc_f32_to_bf16_array.argtypes = [vp, i64, vp]
        L.orc_amax.restype = None
        L.orc_amax.argtypes = [vp, i64, i64, i64, ci, vp]
        L.orc_scale.restype = None
        L.orc_scale.argtypes = [vp, i64, ci, ci, vp]
        L.orc_cast.restype = None
        L.orc_cast.argtypes = [vp, i64, i64, i64, vp, ci, ci, ci, vp, i64, ci]
        L.orc_cast_stats.restype = None
        L.orc_cast_stats.argtypes = [vp, i64, i64, i64, vp, ci, ci, vp]
        L.orc_scaled_mm.restype = None
        L.orc_scaled_mm.argtypes = [vp, i64, ci, vp, ci, vp, i64, ci, vp, ci,
                                    i64, i64, i64, vp, i64, vp, vp, vp]
        L.orc_mx_quantize.restype = None
        L.orc_mx_quantize.argtypes = [vp, i64, i64, i64, ci, vp, i64, vp, i64]
        L.orc_block_quantize.restype = None
        L.orc_block_quantize.argtypes = [vp, i64, i64, i64, i64, i64, ci, vp, i64, vp, i64]
        L.orc_mx_value.restype = C.c_double
        L.orc_mx_value.argtypes = [C.c_uint8, ci, C.c_uint8]
        L.orc_mx_mm.restype = None
        L.orc_mx_mm.argtypes = [vp, i64, ci, vp, i64, vp, i64, ci, vp, i64, i64, i64, i64, vp, i64, vp, vp, vp]
        L.orc_bf16_mm_f64.restype = None
        L.orc_bf16_mm_f64.argtypes = [vp, i64, vp, i64, i64, i64, i64, vp, i64, vp]
        L.orc_f64_to_bf16.restype = C.c_uint16
        L.orc_f64_to_bf16.argtypes = [C.c_double]
        L.orc_sigmoid_bwd.restype = None
        L.orc_sigmoid_bwd.argtypes = [vp, vp, i64, vp]
        L.orc_sigmoid_bf16.restype = None
        L.orc_sigmoid_bf16.argtypes = [vp, i64, vp]
        L.orc_layernorm.restype = None
        L.orc_layernorm.argtypes = [vp, i64, i64, i64, vp, vp, C.c_double, vp, i64, vp, vp]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def num_threads() -> int:
    return int(lib().orc_num_threads())


def fp8_max(fmt: int) -> float:
    return float(lib().orc_fp8_max(fmt))


# ------------------------------------------------------------------ scalars

def decode(code: int, fmt: int) -> float:
    return float(lib().orc_fp8_decode(int(code) & 0xFF, fmt))


def decode_table(fmt: int) -> np.ndarray:
    """float32 value of each of the 256 codes."""
    return np.array([lib().orc_fp8_decode(c, fmt) for c in range(256)], dtype=np.float32)


def encode_search(v: float, fmt: int) -> int:
    return int(lib().orc_fp8_encode_search(float(np.float32(v)), fmt))


def encode_bits(v: float, fmt: int) -> int:
    return int(lib().orc_fp8_encode_bits(float(np.float32(v)), fmt))


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_bf16(x: np.ndarray) -> np.ndarray:
    """Oracle's own bfloat16 rounding, element by element in C."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    lib().orc_f32_to_bf16_array(_p(x), x.size, _p(out))
    return out


def encode_array(v: np.ndarray, fmt: int, use_search: bool = False) -> np.ndarray:
    v = np.ascontiguousarray(v, dtype=np.float32)
    out = np.empty(v.shape, dtype=np.uint8)
    lib().orc_fp8_encode_array(_p(v), v.size, fmt, int(use_search), _p(out))
    return out


# ------------------------------------------------------------------- steps

def _check2d(x, dtype):
    assert x.ndim == 2 and x.dtype == dtype and x.strides[1] == x.itemsize, (x.shape, x.dtype, x.strides)
    return x.shape[0], x.shape[1], x.strides[0] // x.itemsize


def amax(x: np.ndarray, gran: int) -> np.ndarray:
    rows, cols, ld = _check2d(x, np.uint16)
    n = 1 if gran == TENSOR else (rows if gran == ROW else cols)
    out = np.empty(n, dtype=np.float32)
    lib().orc_amax(_p(x), rows, cols, ld, gran, _p(out))
    return out


def scale(amax_: np.ndarray, fmt: int, flags: int = 0) -> np.ndarray:
    a = np.ascontiguousarray(amax_, dtype=np.float32)
    out = np.empty_like(a)
    lib().orc_scale(_p(a), a.size, fmt, flags, _p(out))
    return out


def cast(x: np.ndarray, scale_: np.ndarray, gran: int, fmt: int, flags: int = 0,
         use_search: bool = False) -> np.ndarray:
    rows, cols, ld = _check2d(x, np.uint16)
    s = np.ascontiguousarray(scale_, dtype=np.float32)
    assert s.size == (1 if gran == TENSOR else (rows if gran == ROW else cols))
    q = np.empty((cols, rows) if flags & TRANSPOSE_OUT else (rows, cols), dtype=np.uint8)
    lib().orc_cast(_p(x), rows, cols, ld, _p(s), gran, fmt, flags, _p(q), q.shape[1], int(use_search))
    return q


@dataclass
class CastStats:
    n_sat: int
    n_zero: int
    n_subnormal: int
    sqnr_db: float


def cast_stats(x: np.ndarray, scale_: np.ndarray, gran: int, fmt: int) -> CastStats:
    rows, cols, ld = _check2d(x, np.uint16)
    s = np.ascontiguousarray(scale_, dtype=np.float32)
    st = np.zeros(5, dtype=np.float64)
    lib().orc_cast_stats(_p(x), rows, cols, ld, _p(s), gran, fmt, _p(st))
    sqnr = float("inf") if st[4] == 0 else 10.0 * np.log10(st[3] / st[4])
    return CastStats(int(st[0]), int(st[1]), int(st[2]), float(sqnr))


def quantize(x: np.ndarray, gran: int, fmt: int, flags: int = 0):
    """amax -> scale -> cast.  Returns (codes, scales)."""
    s = scale(amax(x, gran), fmt, flags & POW2_SCALE)
    return cast(x, s, gran, fmt, flags & TRANSPOSE_OUT), s


@dataclass
class MMResult:
    out32: np.ndarray   # fp32 result (dequantized)
    out16: np.ndarray   # bfloat16 bits of out32
    acc64: np.ndarray   # binary64 shadow result


def scaled_mm(a: np.ndarray, fmt_a: int, scale_a: np.ndarray, gran_a: int,
              b: np.ndarray, fmt_b: int, scale_b: np.ndarray, gran_b: int,
              rows: np.ndarray | None = None) -> MMResult:
    """out[m, n] = sum_k dec(a[m,k]) dec(b[n,k]) / (sa sb); a [M,K], b [N,K]."""
    M, K, lda = _check2d(a, np.uint8)
    N, Kb, ldb = _check2d(b, np.uint8)
    assert K == Kb and gran_a in (TENSOR, ROW) and gran_b in (TENSOR, ROW)
    sa = np.ascontiguousarray(scale_a, dtype=np.float32)
    sb = np.ascontiguousarray(scale_b, dtype=np.float32)
    assert sa.size == (1 if gran_a == TENSOR else M) and sb.size == (1 if gran_b == TENSOR else N)
    idx = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    R = M if idx is None else idx.size
    o32 = np.empty((R, N), np.float32)
    o16 = np.empty((R, N), np.uint16)
    a64 = np.empty((R, N), np.float64)
    lib().orc_scaled_mm(_p(a), lda, fmt_a, _p(sa), gran_a, _p(b), ldb, fmt_b, _p(sb), gran_b,
                        M, N, K, _p(idx), R, _p(o32), _p(o16), _p(a64))
    return MMResult(o32, o16, a64)


def bf16_mm_f64(a: np.ndarray, b: np.ndarray, rows: np.ndarray | None = None) -> np.ndarray:
    M, K, lda = _check2d(a, np.uint16)
    N, Kb, ldb = _check2d(b, np.uint16)
    assert K == Kb
    idx = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    R = M if idx is None else idx.size
    out = np.empty((R, N), np.float64)
    lib().orc_bf16_mm_f64(_p(a), lda, _p(b), ldb, M, N, K, _p(idx), R, _p(out))
    return out


# ------------------------------------------------------- O7: linear fwd/bwd

@dataclass(frozen=True)
class Recipe:
    gran: int = TENSOR          # TENSOR or ROW
    fmt_x: int = E4M3FN
    fmt_w: int = E4M3FN
    fmt_dy: int = E5M2
    pow2: bool = False

    @property
    def flags(self) -> int:
        return POW2_SCALE if self.pow2 else 0


@dataclass
class Operand:
    q: np.ndarray
    s: np.ndarray
    gran: int
    fmt: int


def _operand(x, recipe: Recipe, fmt: int, along_cols: bool) -> Operand:
    """Quantize a GEMM operand so that its contraction axis is contiguous.
    along_cols=True : contraction runs over x's columns -> scale per row.
    along_cols=False: contraction runs over x's rows -> scale per column and
    the codes are written transposed (each output row carries one scale)."""
    fl = recipe.flags
    if recipe.gran == TENSOR:
        s = scale(amax(x, TENSOR), fmt, fl)
        q = cast(x, s, TENSOR, fmt, 0 if along_cols else TRANSPOSE_OUT)
        return Operand(q, s, TENSOR, fmt)
    if along_cols:
        q, s = quantize(x, ROW, fmt, fl)
    else:
        q, s = quantize(x, COL, fmt, fl | TRANSPOSE_OUT)
    return Operand(q, s, ROW, fmt)


def _mm(a: Operand, b: Operand, rows=None) -> MMResult:
    return scaled_mm(a.q, a.fmt, a.s, a.gran, b.q, b.fmt, b.s, b.gran, rows)


def linear_fwd(x, w, recipe: Recipe, rows=None):
    """Y[M,N] = X[M,K] W[N,K]^T; both operands quantized along K.
    Returns (MMResult, Xq operand, Wq operand)."""
    xo = _operand(x, recipe, recipe.fmt_x, True)
    wo = _operand(w, recipe, recipe.fmt_w, True)
    return _mm(xo, wo, rows), xo, wo


def linear_bwd_dx(dy, w, recipe: Recipe, rows=None):
    """dX[M,K] = dY[M,N] W[N,K]; contraction over N: dY per row, W per column
    (written transposed as [K,N])."""
    go = _operand(dy, recipe, recipe.fmt_dy, True)
    wo = _operand(w, recipe, recipe.fmt_w, False)
    return _mm(go, wo, rows), go, wo


def linear_bwd_dw(dy, x, recipe: Recipe, rows=None):
    """dW[N,K] = dY[M,N]^T X[M,K]; contraction over M: both operands are
    quantized per column and written transposed ([N,M] and [K,M])."""
    go = _operand(dy, recipe, recipe.fmt_dy, False)
    xo = _operand(x, recipe, recipe.fmt_x, False)
    return _mm(go, xo, rows), go, xo


# ------------------------------------------------------------- MX blocks

MX_BLOCK = 32


def mx_quantize(x: np.ndarray, fmt: int):
    """Blocks of 32 along the last axis -> (codes [rows, cols], E8M0 bytes [rows, cols / 32])."""
    rows, cols, ld = _check2d(x, np.uint16)
    assert cols % MX_BLOCK == 0
    q = np.empty((rows, cols), np.uint8)
    e = np.empty((rows, cols // MX_BLOCK), np.uint8)
    lib().orc_mx_quantize(_p(x), rows, cols, ld, fmt, _p(q), cols, _p(e), cols // MX_BLOCK)
    return q, e


def block_quantize(x: np.ndarray, br: int, bc: int, fmt: int):
    """Blockwise FP8 (blocks of br x bc, power-of-two scales) -> (codes [rows, cols], E8M0 bytes
    [rows, cols / 32] in the layout of the MX scales: a block's byte repeated over its rows and
    its groups of 32 columns)."""
    rows, cols, ld = _check2d(x, np.uint16)
    assert br >= 1 and bc % MX_BLOCK == 0 and cols % bc == 0
    q = np.empty((rows, cols), np.uint8)
    e = np.empty((rows, cols // MX_BLOCK), np.uint8)
    lib().orc_block_quantize(_p(x), rows, cols, ld, br, bc, fmt, _p(q), cols, _p(e), cols // MX_BLOCK)
    return q, e


def block_linear_fwd(x, w, fmt_x=E4M3FN, fmt_w=E4M3FN, rows=None) -> MMResult:
    """Y = X W^T, X in tiles of 1 x 128 along K, W in blocks of 128 x 128 (DeepSeek-style blockwise FP8)."""
    xq, xe = block_quantize(x, 1, 128, fmt_x)
    wq, we = block_quantize(w, 128, 128, fmt_w)
    return mx_mm(xq, fmt_x, xe, wq, fmt_w, we, rows)


def block_linear_bwd(dy, x, w, fmt_dy=E4M3FN, fmt_x=E4M3FN, fmt_w=E4M3FN, rows_dx=None, rows_dw=None):
    """Backward of the blockwise linear layer, each operand with its blocks along the contraction axis of
    the product it feeds (the activation-like operands in tiles of 1 x 128 along that axis, the weight in
    its 128 x 128 blocks):
      dX[m,k] = sum_n dY[m,n] W[n,k]:  dY [M,N] in tiles along N, W^T [K,N] in blocks of 128 x 128;
      dW[n,k] = sum_m dY[m,n] X[m,k]:  dY^T [N,M] and X^T [K,M] in tiles along M.
    Returns (dx, dw) as MMResult; rows_dx / rows_dw select output rows."""
    dyq, dye = block_quantize(dy, 1, 128, fmt_dy)
    wtq, wte = block_quantize(np.ascontiguousarray(w.T), 128, 128, fmt_w)
    dx = mx_mm(dyq, fmt_dy, dye, wtq, fmt_w, wte, rows_dx)
    dytq, dyte = block_quantize(np.ascontiguousarray(dy.T), 1, 128, fmt_dy)
    xtq, xte = block_quantize(np.ascontiguousarray(x.T), 1, 128, fmt_x)
    dw = mx_mm(dytq, fmt_dy, dyte, xtq, fmt_x, xte, rows_dw)
    return dx, dw


def mx_value(code: int, fmt: int, e8m0: int) -> float:
    return float(lib().orc_mx_value(code, fmt, e8m0))


def mx_mm(a, fmt_a, ea, b, fmt_b, eb, rows=None) -> MMResult:
    """out[m, n] = sum over blocks of 2^(ea-127) 2^(eb-127) sum_k dec(a) dec(b); a [M,K], b [N,K]."""
    M, K, lda = _check2d(a, np.uint8)
    N, Kb, ldb = _check2d(b, np.uint8)
    assert K == Kb and K % MX_BLOCK == 0
    ea = np.ascontiguousarray(ea, dtype=np.uint8)
    eb = np.ascontiguousarray(eb, dtype=np.uint8)
    assert ea.shape == (M, K // MX_BLOCK) and eb.shape == (N, K // MX_BLOCK)
    idx = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    R = M if idx is None else idx.size
    o32 = np.empty((R, N), np.float32)
    o16 = np.empty((R, N), np.uint16)
    a64 = np.empty((R, N), np.float64)
    lib().orc_mx_mm(_p(a), lda, fmt_a, _p(ea), K // MX_BLOCK, _p(b), ldb, fmt_b, _p(eb), K // MX_BLOCK,
                    M, N, K, _p(idx), R, _p(o32), _p(o16), _p(a64))
    return MMResult(o32, o16, a64)


def mx_linear_fwd(x, w, fmt_x=E4M3FN, fmt_w=E4M3FN, rows=None) -> MMResult:
    """Y = X W^T with both operands in MX blocks of 32 along K."""
    xq, xe = mx_quantize(x, fmt_x)
    wq, we = mx_quantize(w, fmt_w)
    return mx_mm(xq, fmt_x, xe, wq, fmt_w, we, rows)


def mx_linear_bwd(dy, x, w, fmt_dy=E4M3FN, fmt_x=E4M3FN, fmt_w=E4M3FN, rows_dx=None, rows_dw=None):
    """Backward of the MX linear layer.  The blocks of 32 run along each
    product's own contraction axis (OCP MX v1.0 Section 6.2: the scaled dot
    product is defined over blocks of the contracted index), so every operand is
    re-quantized from its bfloat16 original in the orientation the product needs:
      dX[m,k] = sum_n dY[m,n] W[n,k]:  dY in blocks along N, W^T [K,N] in blocks along N;
      dW[n,k] = sum_m dY[m,n] X[m,k]:  dY^T [N,M] and X^T [K,M] in blocks along M.
    Returns (dx, dw) as MMResult; rows_dx / rows_dw select output rows."""
    dyq, dye = mx_quantize(dy, fmt_dy)
    wtq, wte = mx_quantize(np.ascontiguousarray(w.T), fmt_w)
    dx = mx_mm(dyq, fmt_dy, dye, wtq, fmt_w, wte, rows_dx)
    dytq, dyte = mx_quantize(np.ascontiguousarray(dy.T), fmt_dy)
    xtq, xte = mx_quantize(np.ascontiguousarray(x.T), fmt_x)
    dw = mx_mm(dytq, fmt_dy, dyte, xtq, fmt_x, xte, rows_dw)
    return dx, dw


def linear_bwd_dw_hp(dy, x, rows=None):
    """Weight gradient of the rowwise_gw_hp recipe (Appendix A: the grad_weight
    GEMM stays in bfloat16): dW[n,k] = sum_m dY[m,n] X[m,k] on the unquantized
    inputs.  The definition written out: binary64 sums of the exact products
    (orc_bf16_mm_f64 on the transposed operands), rounded to binary32 and then
    to bfloat16.  Returns (out32, out16); rows selects output rows n."""
    acc = bf16_mm_f64(np.ascontiguousarray(dy.T), np.ascontiguousarray(x.T), rows)
    out32 = acc.astype(np.float32)
    return out32, f32_to_bf16(out32)


def f64_to_bf16(d: float) -> int:
    return int(lib().orc_f64_to_bf16(float(d)))


def sigmoid_bf16(v: np.ndarray) -> np.ndarray:
    """bfloat16 bits of 1 / (1 + exp(-v)) for fp32 v (binary64 evaluation, one rounding)."""
    v = np.ascontiguousarray(v, dtype=np.float32)
    out = np.empty(v.shape, np.uint16)
    lib().orc_sigmoid_bf16(_p(v), v.size, _p(out))
    return out


def sigmoid_bwd(dy: np.ndarray, y: np.ndarray) -> np.ndarray:
    """bfloat16 bits of dz = dy * y * (1 - y) (binary32, one operation at a time), same shape as dy."""
    dy = np.ascontiguousarray(dy, dtype=np.uint16)
    y = np.ascontiguousarray(y, dtype=np.uint16)
    assert dy.shape == y.shape
    dz = np.empty(dy.shape, np.uint16)
    lib().orc_sigmoid_bwd(_p(dy), _p(y), dy.size, _p(dz))
    return dz


def layernorm(x: np.ndarray, gamma: np.ndarray, beta: np.ndarray | None, eps: float):
    """LayerNorm over the last axis in binary64, output rounded once to bfloat16:
    (h bits [rows, cols], mean [rows] f64, rstd [rows] f64)."""
    rows, cols, ld = _check2d(x, np.uint16)
    gamma = np.ascontiguousarray(gamma, dtype=np.uint16)
    assert gamma.shape == (cols,)
    if beta is not None:
        beta = np.ascontiguousarray(beta, dtype=np.uint16)
        assert beta.shape == (cols,)
    h = np.empty((rows, cols), np.uint16)
    mean = np.empty(rows, np.float64)
    rstd = np.empty(rows, np.float64)
    lib().orc_layernorm(_p(x), rows, cols, ld, _p(gamma), _p(beta), float(eps), _p(h), cols, _p(mean), _p(rstd))
    return h, mean, rstd


def layernorm_quantize(x, gamma, beta, eps, fmt=E4M3FN, pow2=False):
    """The normalised bfloat16 tensor and its rowwise dynamic quantization (codes, scales)."""
    h, mean, rstd = layernorm(x, gamma, beta, eps)
    q, s = quantize(h, ROW, fmt, POW2_SCALE if pow2 else 0)
    return h, q, s, mean, rstd


def rel_frobenius(got: np.ndarray, ref: np.ndarray) -> float:
    g = np.asarray(got, dtype=np.float64)
    r = np.asarray(ref, dtype=np.float64)
    den = np.sqrt((r * r).sum())
    return float(np.sqrt(((g - r) ** 2).sum()) / den) if den > 0 else float(np.sqrt(((g - r) ** 2).sum()))
