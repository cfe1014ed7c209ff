"""ctypes binding of the C ABI declared in include/fp8mi355.h.

Same names as the C entry points.  Tensors are torch CUDA (ROCm) tensors:
bfloat16 inputs as ``torch.bfloat16`` (or raw ``uint16``/``int16`` bits), fp8
codes as ``torch.uint8``, scales as ``torch.float32``.  Work is enqueued on
torch's current stream.  There is no fallback: if the library cannot be loaded
an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

FP8_E4M3FN, FP8_E5M2 = 0, 1
FP8_TENSOR, FP8_ROW, FP8_COL = 0, 1, 2
FP8_POW2_SCALE, FP8_TRANSPOSE_OUT, FP8_OUT_FP32, FP8_GRAD_WEIGHT_HP, FP8_SAVE_FOR_BWD = 1, 2, 4, 8, 16
FP8_EPILOGUE_SIGMOID = 32

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfp8mi355.so")
_lib = None


class Fp8Error(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"fp8mi355 error {code}: {msg}")
        self.code = code


class _CRecipe(C.Structure):
    _fields_ = [("gran", C.c_int), ("fmt_x", C.c_int), ("fmt_w", C.c_int), ("fmt_dy", C.c_int), ("flags", C.c_int)]


@dataclass(frozen=True)
class Recipe:
    gran: int = FP8_TENSOR
    fmt_x: int = FP8_E4M3FN
    fmt_w: int = FP8_E4M3FN
    fmt_dy: int = FP8_E5M2
    flags: int = 0

    def c(self) -> _CRecipe:
        return _CRecipe(self.gran, self.fmt_x, self.fmt_w, self.fmt_dy, self.flags)


def library_path() -> str:
    return _LIB_PATH


def load_library() -> C.CDLL:
    """Load libfp8mi355.so (built in-tree by paper_2507_16099_amd/build.py)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -m paper_2507_16099_amd.build` "
                          "(or __graft_entry__.build()); there is no fallback path")
    L = C.CDLL(_LIB_PATH)
    i64, vp, ci = C.c_int64, C.c_void_p, C.c_int
    L.fp8_last_error.restype = C.c_char_p
    L.fp8_last_error.argtypes = []
    L.fp8_version.restype = C.c_char_p
    L.fp8_version.argtypes = []
    L.fp8_amax.restype = ci
    L.fp8_amax.argtypes = [vp, i64, i64, i64, ci, vp, vp]
    L.fp8_scale.restype = ci
    L.fp8_scale.argtypes = [vp, i64, ci, ci, vp, vp]
    L.fp8_cast.restype = ci
    L.fp8_cast.argtypes = [vp, i64, i64, i64, vp, ci, ci, ci, vp, i64, vp]
    L.fp8_quantize.restype = ci
    L.fp8_quantize.argtypes = [vp, i64, i64, i64, ci, ci, ci, vp, i64, vp, vp]
    L.fp8_quantize_row_col.restype = ci
    L.fp8_quantize_row_col.argtypes = [vp, i64, i64, i64, ci, ci, vp, i64, vp, vp, i64, vp, vp]
    L.fp8_scaled_mm.restype = ci
    L.fp8_scaled_mm.argtypes = [vp, i64, ci, vp, ci, vp, i64, ci, vp, ci, i64, i64, i64, vp, i64, ci, vp]
    L.fp8_linear_workspace_bytes.restype = C.c_size_t
    L.fp8_linear_workspace_bytes.argtypes = [i64, i64, i64, C.POINTER(_CRecipe), ci]
    L.fp8_linear_fwd.restype = ci
    L.fp8_linear_fwd.argtypes = [vp, vp, i64, i64, i64, C.POINTER(_CRecipe), vp, vp, C.c_size_t, vp]
    L.fp8_linear_prequantized_workspace_bytes.restype = C.c_size_t
    L.fp8_linear_prequantized_workspace_bytes.argtypes = [i64, i64]
    L.fp8_linear_fwd_prequantized.restype = ci
    L.fp8_linear_fwd_prequantized.argtypes = [vp, i64, i64, ci, ci, ci, vp, i64, ci, vp, ci, i64, vp, i64, vp,
                                              C.c_size_t, vp]
    L.fp8_linear_fwd_prequantized_static.restype = ci
    L.fp8_linear_fwd_prequantized_static.argtypes = [vp, i64, i64, ci, ci, ci, vp, i64, ci, vp, ci, i64, vp, i64, vp]
    L.fp8_linear_bwd_sigmoid_workspace_bytes.restype = C.c_size_t
    L.fp8_linear_bwd_sigmoid_workspace_bytes.argtypes = [i64, i64, i64, vp]
    L.fp8_linear_bwd_sigmoid.restype = ci
    L.fp8_linear_bwd_sigmoid.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, vp, vp, vp, C.c_size_t, vp]
    L.fp8_layernorm_quantize.restype = ci
    L.fp8_layernorm_quantize.argtypes = [vp, i64, i64, i64, vp, vp, C.c_double, ci, ci, vp, i64, vp, i64, vp, vp, vp, vp]
    L.fp8_block_quantize.restype = ci
    L.fp8_block_quantize.argtypes = [vp, i64, i64, i64, ci, ci, vp, i64, vp, i64, vp]
    L.fp8_block_linear_workspace_bytes.restype = C.c_size_t
    L.fp8_block_linear_workspace_bytes.argtypes = [i64, i64, i64]
    L.fp8_block_linear_fwd.restype = ci
    L.fp8_block_linear_fwd.argtypes = [vp, vp, i64, i64, i64, ci, ci, vp, vp, C.c_size_t, vp]
    L.fp8_block_quantize_t.restype = ci
    L.fp8_block_quantize_t.argtypes = [vp, i64, i64, i64, ci, ci, vp, i64, vp, i64, vp]
    L.fp8_block_linear_bwd_workspace_bytes.restype = C.c_size_t
    L.fp8_block_linear_bwd_workspace_bytes.argtypes = [i64, i64, i64]
    L.fp8_block_linear_bwd.restype = ci
    L.fp8_block_linear_bwd.argtypes = [vp, vp, vp, i64, i64, i64, ci, ci, ci, vp, vp, vp, C.c_size_t, vp]
    L.fp8_block_quantize_row_col.restype = ci
    L.fp8_block_quantize_row_col.argtypes = [vp, i64, i64, i64, ci, vp, i64, vp, i64, vp, i64, vp, i64, vp]
    L.fp8_mx_quantize.restype = ci
    L.fp8_mx_quantize.argtypes = [vp, i64, i64, i64, ci, vp, i64, vp, i64, vp]
    L.fp8_mx_quantize_t.restype = ci
    L.fp8_mx_quantize_t.argtypes = [vp, i64, i64, i64, ci, vp, i64, vp, i64, vp]
    L.fp8_mx_quantize_row_col.restype = ci
    L.fp8_mx_quantize_row_col.argtypes = [vp, i64, i64, i64, ci, vp, i64, vp, i64, vp, i64, vp, i64, vp]
    L.fp8_mx_linear_bwd_workspace_bytes.restype = C.c_size_t
    L.fp8_mx_linear_bwd_workspace_bytes.argtypes = [i64, i64, i64]
    L.fp8_mx_linear_bwd.restype = ci
    L.fp8_mx_linear_bwd.argtypes = [vp, vp, vp, i64, i64, i64, ci, ci, ci, vp, vp, vp, C.c_size_t, vp]
    L.fp8_mx_scaled_mm.restype = ci
    L.fp8_mx_scaled_mm.argtypes = [vp, i64, ci, vp, i64, vp, i64, ci, vp, i64, i64, i64, i64, vp, i64, ci, vp]
    L.fp8_mx_linear_workspace_bytes.restype = C.c_size_t
    L.fp8_mx_linear_workspace_bytes.argtypes = [i64, i64, i64]
    L.fp8_mx_linear_fwd.restype = ci
    L.fp8_mx_linear_fwd.argtypes = [vp, vp, i64, i64, i64, ci, ci, vp, vp, C.c_size_t, vp]
    L.fp8_grad_weight_hp.restype = ci
    L.fp8_grad_weight_hp.argtypes = [vp, vp, i64, i64, i64, vp, vp]
    L.fp8_linear_bwd.restype = ci
    L.fp8_linear_bwd.argtypes = [vp, vp, vp, i64, i64, i64, C.POINTER(_CRecipe), vp, vp, vp, C.c_size_t, vp]
    L.fp8_internal_set_knob.restype = ci
    L.fp8_internal_set_knob.argtypes = [C.c_char_p, ci]
    _lib = L
    return L


def set_knob(name: str, value: int | None) -> None:
    """Force one of the library's tuning / test switches (GEMM_VARIANT, SNAKE_HALF, SKINNY_NW, SKINNY_DMA,
    MX_VARIANT, MX_SLAB, BF16_VARIANT, GEMM_STREAM, GEMM_TILE_M) for the rest of the process; None restores the default.  The
    library reads FP8MI355_<NAME> from the environment once, on first use; afterwards only this call changes a switch."""
    if load_library().fp8_internal_set_knob(name.encode(), -1 if value is None else int(value)) != 0:
        raise ValueError(f"unknown switch {name!r}")


def fp8_last_error() -> str:
    return load_library().fp8_last_error().decode()


def fp8_version() -> str:
    return load_library().fp8_version().decode()


def _check(rc: int) -> None:
    if rc != 0:
        raise Fp8Error(rc, fp8_last_error())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _mat(t: torch.Tensor, itemsize: int):
    """(rows, cols, ld) of a 2-D tensor whose last dimension is contiguous."""
    assert t.is_cuda and t.dim() == 2 and t.element_size() == itemsize, (t.shape, t.dtype, t.device)
    assert t.shape[1] <= 1 or t.stride(1) == 1, "last dimension must be contiguous"
    if t.numel() == 0:
        return t.shape[0], t.shape[1], (t.shape[1] + 15) // 16 * 16
    ld = t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])
    return t.shape[0], t.shape[1], ld


def _groups(gran: int, rows: int, cols: int) -> int:
    return 1 if gran == FP8_TENSOR else (rows if gran == FP8_ROW else cols)


def _pad16(n: int) -> int:
    return (n + 15) // 16 * 16


def fp8_amax(x: torch.Tensor, gran: int, out: torch.Tensor | None = None) -> torch.Tensor:
    rows, cols, ld = _mat(x, 2)
    if out is None:
        out = torch.empty(max(_groups(gran, rows, cols), 0), dtype=torch.float32, device=x.device)
    _check(load_library().fp8_amax(_ptr(x), rows, cols, ld, gran, _ptr(out), _stream()))
    return out


def fp8_scale(amax: torch.Tensor, fmt: int, flags: int = 0, out: torch.Tensor | None = None) -> torch.Tensor:
    assert amax.is_cuda and amax.dtype == torch.float32 and amax.is_contiguous()
    if out is None:
        out = torch.empty_like(amax)
    _check(load_library().fp8_scale(_ptr(amax), amax.numel(), fmt, flags, _ptr(out), _stream()))
    return out


def _alloc_q(rows: int, cols: int, flags: int, device) -> torch.Tensor:
    """fp8 output with a leading dimension padded to 16 (returned as a view)."""
    r, c = (cols, rows) if flags & FP8_TRANSPOSE_OUT else (rows, cols)
    return torch.empty((r, _pad16(c)), dtype=torch.uint8, device=device)[:, :c]


def fp8_cast(x: torch.Tensor, scale: torch.Tensor, gran: int, fmt: int, flags: int = 0,
             out: torch.Tensor | None = None) -> torch.Tensor:
    rows, cols, ld = _mat(x, 2)
    if out is None:
        out = _alloc_q(rows, cols, flags, x.device)
    _, _, ld_out = _mat(out, 1)
    _check(load_library().fp8_cast(_ptr(x), rows, cols, ld, _ptr(scale), gran, fmt, flags, _ptr(out), ld_out, _stream()))
    return out


def fp8_quantize(x: torch.Tensor, gran: int, fmt: int, flags: int = 0, out: torch.Tensor | None = None,
                 scale_out: torch.Tensor | None = None):
    rows, cols, ld = _mat(x, 2)
    if out is None:
        out = _alloc_q(rows, cols, flags, x.device)
    if scale_out is None:
        scale_out = torch.empty(_groups(gran, rows, cols), dtype=torch.float32, device=x.device)
    _, _, ld_out = _mat(out, 1)
    _check(load_library().fp8_quantize(_ptr(x), rows, cols, ld, gran, fmt, flags, _ptr(out), ld_out,
                                       _ptr(scale_out), _stream()))
    return out, scale_out


def fp8_quantize_row_col(x: torch.Tensor, fmt: int, flags: int = 0, q_row: torch.Tensor | None = None,
                         scale_row: torch.Tensor | None = None, q_col_t: torch.Tensor | None = None,
                         scale_col: torch.Tensor | None = None):
    """Rowwise codes [rows, cols] + scales [rows] and per-column codes, transposed [cols, rows], + scales [cols]."""
    rows, cols, ld = _mat(x, 2)
    if q_row is None:
        q_row = _alloc_q(rows, cols, 0, x.device)
    if q_col_t is None:
        q_col_t = _alloc_q(rows, cols, FP8_TRANSPOSE_OUT, x.device)
    if scale_row is None:
        scale_row = torch.empty(rows, dtype=torch.float32, device=x.device)
    if scale_col is None:
        scale_col = torch.empty(cols, dtype=torch.float32, device=x.device)
    _, _, ld_row = _mat(q_row, 1)
    _, _, ld_col_t = _mat(q_col_t, 1)
    _check(load_library().fp8_quantize_row_col(_ptr(x), rows, cols, ld, fmt, flags, _ptr(q_row), ld_row, _ptr(scale_row),
                                               _ptr(q_col_t), ld_col_t, _ptr(scale_col), _stream()))
    return q_row, scale_row, q_col_t, scale_col


def fp8_scaled_mm(a: torch.Tensor, fmt_a: int, scale_a: torch.Tensor, gran_a: int,
                  b: torch.Tensor, fmt_b: int, scale_b: torch.Tensor, gran_b: int,
                  flags: int = 0, out: torch.Tensor | None = None) -> torch.Tensor:
    M, K, lda = _mat(a, 1)
    N, Kb, ldb = _mat(b, 1)
    assert K == Kb, (a.shape, b.shape)
    if out is None:
        dt = torch.float32 if flags & FP8_OUT_FP32 else torch.bfloat16
        pad = 4 if flags & FP8_OUT_FP32 else 8
        out = torch.empty((M, (N + pad - 1) // pad * pad), dtype=dt, device=a.device)[:, :N]
    _, _, ld_out = _mat(out, out.element_size())
    _check(load_library().fp8_scaled_mm(_ptr(a), lda, fmt_a, _ptr(scale_a), gran_a, _ptr(b), ldb, fmt_b,
                                        _ptr(scale_b), gran_b, M, N, K, _ptr(out), ld_out, flags, _stream()))
    return out


def fp8_linear_workspace_bytes(M: int, K: int, N: int, recipe: Recipe, bwd: bool) -> int:
    r = recipe.c()
    n = load_library().fp8_linear_workspace_bytes(M, K, N, C.byref(r), int(bwd))
    if n == 0:
        raise Fp8Error(-2, fp8_last_error())
    return int(n)


def fp8_linear_fwd(x: torch.Tensor, w: torch.Tensor, recipe: Recipe, y: torch.Tensor | None = None,
                   workspace: torch.Tensor | None = None) -> torch.Tensor:
    M, K, ldx = _mat(x, 2)
    N, Kw, ldw = _mat(w, 2)
    assert K == Kw and ldx == K and ldw == K, "x and w must be dense [M,K] / [N,K]"
    assert workspace is not None or not (recipe.flags & FP8_SAVE_FOR_BWD), "pass the workspace the backward will reuse"
    if workspace is None:
        workspace = torch.empty(fp8_linear_workspace_bytes(M, K, N, recipe, False), dtype=torch.uint8, device=x.device)
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    r = recipe.c()
    _check(load_library().fp8_linear_fwd(_ptr(x), _ptr(w), M, K, N, C.byref(r), _ptr(y), _ptr(workspace),
                                         workspace.numel(), _stream()))
    return y


def fp8_linear_bwd(dy: torch.Tensor, x: torch.Tensor, w: torch.Tensor, recipe: Recipe,
                   dx: torch.Tensor | None = None, dw: torch.Tensor | None = None,
                   workspace: torch.Tensor | None = None, need_dx: bool = True, need_dw: bool = True):
    """x, w: the layer's inputs, or (with FP8_SAVE_FOR_BWD, where the forward left their fp8 copies in
    the workspace) just their shapes as tuples (M, K) and (N, K)."""
    M, N, _ = _mat(dy, 2)
    K = x.shape[1] if isinstance(x, torch.Tensor) else x[1]
    if recipe.flags & FP8_SAVE_FOR_BWD:
        assert workspace is not None, "the backward reuses the forward's workspace"
        assert tuple(x.shape if isinstance(x, torch.Tensor) else x) == (M, K)
        assert tuple(w.shape if isinstance(w, torch.Tensor) else w) == (N, K)
        x = x if isinstance(x, torch.Tensor) else None
        w = w if isinstance(w, torch.Tensor) else None
    else:
        assert x.shape == (M, K) and w.shape == (N, K) and x.is_contiguous() and w.is_contiguous()
    assert dy.is_contiguous()
    if workspace is None:
        workspace = torch.empty(fp8_linear_workspace_bytes(M, K, N, recipe, True), dtype=torch.uint8, device=dy.device)
    if dx is None and need_dx:
        dx = torch.empty((M, K), dtype=torch.bfloat16, device=dy.device)
    if dw is None and need_dw:
        dw = torch.empty((N, K), dtype=torch.bfloat16, device=dy.device)
    r = recipe.c()
    _check(load_library().fp8_linear_bwd(_ptr(dy), _ptr(x), _ptr(w), M, K, N, C.byref(r), _ptr(dx), _ptr(dw),
                                         _ptr(workspace), workspace.numel(), _stream()))
    return dx, dw


def fp8_linear_bwd_sigmoid_workspace_bytes(M: int, K: int, N: int, recipe: Recipe) -> int:
    r = recipe.c()
    n = load_library().fp8_linear_bwd_sigmoid_workspace_bytes(M, K, N, C.byref(r))
    if n == 0:
        raise Fp8Error(-2, fp8_last_error())
    return int(n)


def fp8_linear_bwd_sigmoid(dy: torch.Tensor, y: torch.Tensor, x, w, recipe: Recipe, dx: torch.Tensor | None = None,
                           dw: torch.Tensor | None = None, workspace: torch.Tensor | None = None,
                           need_dx: bool = True, need_dw: bool = True):
    """Backward through Sigmoid + Linear: as fp8_linear_bwd with dY = dy * y * (1 - y), y the stored sigmoid output."""
    M, N, _ = _mat(dy, 2)
    assert tuple(y.shape) == (M, N) and dy.is_contiguous() and y.is_contiguous() and y.element_size() == 2
    K = x.shape[1] if isinstance(x, torch.Tensor) else x[1]
    x = x if isinstance(x, torch.Tensor) else None
    w = w if isinstance(w, torch.Tensor) else None
    assert x is None or (tuple(x.shape) == (M, K) and x.is_contiguous())
    assert w is None or (tuple(w.shape) == (N, K) and w.is_contiguous())
    if workspace is None:
        workspace = torch.empty(fp8_linear_bwd_sigmoid_workspace_bytes(M, K, N, recipe), dtype=torch.uint8, device=dy.device)
    if dx is None and need_dx:
        dx = torch.empty((M, K), dtype=torch.bfloat16, device=dy.device)
    if dw is None and need_dw:
        dw = torch.empty((N, K), dtype=torch.bfloat16, device=dy.device)
    r = recipe.c()
    _check(load_library().fp8_linear_bwd_sigmoid(_ptr(dy), _ptr(y), _ptr(x), _ptr(w), M, K, N, C.byref(r), _ptr(dx), _ptr(dw),
                                                 _ptr(workspace), workspace.numel(), _stream()))
    return dx, dw


def fp8_linear_prequantized_workspace_bytes(M: int, K: int) -> int:
    n = load_library().fp8_linear_prequantized_workspace_bytes(M, K)
    if n == 0:
        raise Fp8Error(-2, fp8_last_error())
    return n


def fp8_linear_fwd_prequantized(x: torch.Tensor, wq: torch.Tensor, fmt_w: int, scale_w: torch.Tensor, gran_w: int,
                                fmt_x: int = FP8_E4M3FN, gran_x: int = FP8_ROW, flags: int = 0,
                                y: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Y = X W^T with a weight quantized beforehand (codes wq [N, K], scales scale_w) and x quantized per call."""
    M, K, ldx = _mat(x, 2)
    N, Kw, ldw = _mat(wq, 1)
    assert K == Kw and ldx == K, (x.shape, wq.shape)
    if y is None:
        y = torch.empty((M, (N + 7) // 8 * 8), dtype=torch.bfloat16, device=x.device)[:, :N]
    _, _, ld_y = _mat(y, 2)
    if workspace is None:
        workspace = torch.empty(fp8_linear_prequantized_workspace_bytes(M, K), dtype=torch.uint8, device=x.device)
    _check(load_library().fp8_linear_fwd_prequantized(_ptr(x), M, K, fmt_x, gran_x, flags, _ptr(wq), ldw, fmt_w,
                                                      _ptr(scale_w), gran_w, N, _ptr(y), ld_y, _ptr(workspace),
                                                      workspace.numel(), _stream()))
    return y


FP8_STATIC_SCRATCH_BYTES = 8 << 20


def fp8_linear_fwd_prequantized_static(x: torch.Tensor, wq: torch.Tensor, fmt_w: int, scale_w: torch.Tensor, gran_w: int,
                                       y: torch.Tensor, fmt_x: int = FP8_E4M3FN, gran_x: int = FP8_ROW,
                                       flags: int = 0) -> torch.Tensor:
    """fp8_linear_fwd_prequantized without a workspace: the library's static device buffer holds the activation
    codes.  The caller passes y; nothing is allocated here or in the library."""
    M, K, ldx = _mat(x, 2)
    N, Kw, ldw = _mat(wq, 1)
    assert K == Kw and ldx == K, (x.shape, wq.shape)
    _, _, ld_y = _mat(y, 2)
    _check(load_library().fp8_linear_fwd_prequantized_static(_ptr(x), M, K, fmt_x, gran_x, flags, _ptr(wq), ldw, fmt_w,
                                                             _ptr(scale_w), gran_w, N, _ptr(y), ld_y, _stream()))
    return y


def fp8_grad_weight_hp(dy: torch.Tensor, x: torch.Tensor, dw: torch.Tensor | None = None) -> torch.Tensor:
    """dW [N, K] = dY [M, N]^T X [M, K] in bfloat16 (fp32 accumulate), no quantization."""
    M, N, ldg = _mat(dy, 2)
    Mx, K, ldx = _mat(x, 2)
    assert M == Mx and (M == 0 or (ldg == N and ldx == K)), (dy.shape, x.shape)
    if dw is None:
        dw = torch.empty((N, K), dtype=torch.bfloat16, device=dy.device)
    assert dw.is_contiguous() and tuple(dw.shape) == (N, K)
    _check(load_library().fp8_grad_weight_hp(_ptr(dy), _ptr(x), M, K, N, _ptr(dw), _stream()))
    return dw


def fp8_layernorm_quantize(x: torch.Tensor, gamma: torch.Tensor, beta: torch.Tensor | None, eps: float,
                           fmt: int = FP8_E4M3FN, flags: int = 0, want_h: bool = True, want_stats: bool = True, out=None):
    """LayerNorm over the last axis with the rowwise fp8 quantization of its bfloat16 result fused in.
    Returns (h or None, q, scale, mean or None, rstd or None); out: the same five to write into."""
    rows, cols, ld = _mat(x, 2)
    assert gamma.is_contiguous() and gamma.numel() == cols and gamma.element_size() == 2
    assert beta is None or (beta.is_contiguous() and beta.numel() == cols and beta.element_size() == 2)
    if out is None:
        h = torch.empty((rows, cols), dtype=torch.bfloat16, device=x.device) if want_h else None
        q = _alloc_q(rows, cols, 0, x.device)
        s = torch.empty(rows, dtype=torch.float32, device=x.device)
        mean = torch.empty(rows, dtype=torch.float32, device=x.device) if want_stats else None
        rstd = torch.empty(rows, dtype=torch.float32, device=x.device) if want_stats else None
    else:
        h, q, s, mean, rstd = out
    ld_h = _mat(h, 2)[2] if h is not None else 0
    _check(load_library().fp8_layernorm_quantize(_ptr(x), rows, cols, ld, _ptr(gamma), _ptr(beta), float(eps), fmt, flags,
                                                 _ptr(h), ld_h, _ptr(q), _mat(q, 1)[2], _ptr(s), _ptr(mean), _ptr(rstd),
                                                 _stream()))
    return h, q, s, mean, rstd


def _alloc_e8m0(rows: int, nb: int, slabs: bool, device) -> torch.Tensor:
    """Room for the E8M0 bytes of `rows` scale rows of `nb` blocks: plain rows [rows, nb] (row pitch a multiple
    of 4), or, with slabs, [nb / 16, rows, 16] (see the layout note in fp8mi355.h)."""
    if slabs:
        if nb % 16 != 0:
            raise ValueError("scale slabs need a multiple of 16 blocks (512 elements) per row")
        return torch.empty((nb // 16, rows, 16), dtype=torch.uint8, device=device)
    return torch.empty((rows, (nb + 3) // 4 * 4), dtype=torch.uint8, device=device)[:, :nb]


def _e8m0_ld(e: torch.Tensor) -> int:
    """The ld_e argument for a scale tensor: its row pitch, or minus the rows per slab for a 3-D slab tensor."""
    if e.dim() == 3:
        assert e.dtype == torch.uint8 and e.shape[2] == 16 and e.is_contiguous(), "slab tensor must be [nb/16, rows, 16] uint8, contiguous"
        return -int(e.shape[1])
    return _mat(e, 1)[2]


def e8m0_plain_rows(e: torch.Tensor) -> torch.Tensor:
    """A scale tensor as plain rows [rows, nb], whatever its layout (a copy for slabs)."""
    if e.dim() == 3:
        return e.permute(1, 0, 2).reshape(e.shape[1], e.shape[0] * 16)
    return e


def fp8_mx_quantize(x: torch.Tensor, fmt: int, q: torch.Tensor | None = None, e8m0: torch.Tensor | None = None,
                    slabs: bool = False):
    """MX blocks of 32 along the last axis: codes [rows, cols] and E8M0 bytes [rows, cols / 32]
    (slabs: [cols / 512, rows, 16])."""
    rows, cols, ld = _mat(x, 2)
    if q is None:
        q = _alloc_q(rows, cols, 0, x.device)
    if e8m0 is None:
        e8m0 = _alloc_e8m0(rows, cols // 32, slabs, x.device)
    _, _, ld_q = _mat(q, 1)
    ld_e = _e8m0_ld(e8m0)
    _check(load_library().fp8_mx_quantize(_ptr(x), rows, cols, ld, fmt, _ptr(q), ld_q, _ptr(e8m0), ld_e, _stream()))
    return q, e8m0


def fp8_block_quantize(x: torch.Tensor, block_rows: int, fmt: int, q: torch.Tensor | None = None,
                       e8m0: torch.Tensor | None = None, slabs: bool = False):
    """Blockwise FP8: tiles of 1 x 128 (block_rows = 1) or blocks of 128 x 128 (block_rows = 128) with power-of-two
    scales; codes [rows, cols] and E8M0 bytes [rows, cols / 32] in the layout of the MX scales."""
    rows, cols, ld = _mat(x, 2)
    if q is None:
        q = _alloc_q(rows, cols, 0, x.device)
    if e8m0 is None:
        e8m0 = _alloc_e8m0(rows, cols // 32, slabs, x.device)
    _, _, ld_q = _mat(q, 1)
    ld_e = _e8m0_ld(e8m0)
    _check(load_library().fp8_block_quantize(_ptr(x), rows, cols, ld, block_rows, fmt, _ptr(q), ld_q, _ptr(e8m0), ld_e,
                                             _stream()))
    return q, e8m0


def fp8_block_linear_workspace_bytes(M: int, K: int, N: int) -> int:
    n = load_library().fp8_block_linear_workspace_bytes(M, K, N)
    if n == 0:
        raise Fp8Error(-2, fp8_last_error())
    return int(n)


def fp8_block_linear_fwd(x: torch.Tensor, w: torch.Tensor, fmt_x: int = FP8_E4M3FN, fmt_w: int = FP8_E4M3FN,
                         y: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Y = X W^T with X in tiles of 1 x 128 along K and W in blocks of 128 x 128 (blockwise FP8)."""
    M, K = x.shape
    N = w.shape[0]
    assert w.shape == (N, K) and x.is_contiguous() and w.is_contiguous()
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    if workspace is None:
        workspace = torch.empty(fp8_block_linear_workspace_bytes(M, K, N), dtype=torch.uint8, device=x.device)
    _check(load_library().fp8_block_linear_fwd(_ptr(x), _ptr(w), M, K, N, fmt_x, fmt_w, _ptr(y), _ptr(workspace),
                                               workspace.numel(), _stream()))
    return y


def fp8_block_quantize_t(x: torch.Tensor, block_rows: int, fmt: int, qt: torch.Tensor | None = None,
                         e8m0_t: torch.Tensor | None = None, slabs: bool = False):
    """Blockwise FP8 of the transposed matrix, written transposed: codes [cols, rows], E8M0 bytes [cols, rows / 32]
    (block_rows = 1: tiles of 128 rows x 1 column of x; 128: blocks of 128 x 128)."""
    rows, cols, ld = _mat(x, 2)
    if qt is None:
        qt = _alloc_q(cols, rows, 0, x.device)
    if e8m0_t is None:
        e8m0_t = _alloc_e8m0(cols, rows // 32, slabs, x.device)
    _, _, ld_q = _mat(qt, 1)
    ld_e = _e8m0_ld(e8m0_t)
    _check(load_library().fp8_block_quantize_t(_ptr(x), rows, cols, ld, block_rows, fmt, _ptr(qt), ld_q, _ptr(e8m0_t), ld_e,
                                               _stream()))
    return qt, e8m0_t


def fp8_block_linear_bwd_workspace_bytes(M: int, K: int, N: int) -> int:
    n = load_library().fp8_block_linear_bwd_workspace_bytes(M, K, N)
    if n == 0:
        raise Fp8Error(-2, fp8_last_error())
    return int(n)


def fp8_block_linear_bwd(dy: torch.Tensor, x: torch.Tensor, w: torch.Tensor, fmt_dy: int = FP8_E4M3FN,
                         fmt_x: int = FP8_E4M3FN, fmt_w: int = FP8_E4M3FN, need_dx: bool = True, need_dw: bool = True,
                         dx: torch.Tensor | None = None, dw: torch.Tensor | None = None,
                         workspace: torch.Tensor | None = None):
    """dX = dY W and dW = dY^T X of the blockwise linear layer (tiles of 1 x 128 along each product's contraction
    axis, the weight in its 128 x 128 blocks)."""
    M, N = dy.shape
    K = x.shape[1]
    assert x.shape == (M, K) and w.shape == (N, K) and dy.is_contiguous() and x.is_contiguous() and w.is_contiguous()
    if need_dx and dx is None:
        dx = torch.empty((M, K), dtype=torch.bfloat16, device=dy.device)
    if need_dw and dw is None:
        dw = torch.empty((N, K), dtype=torch.bfloat16, device=dy.device)
    if workspace is None:
        workspace = torch.empty(fp8_block_linear_bwd_workspace_bytes(M, K, N), dtype=torch.uint8, device=dy.device)
    _check(load_library().fp8_block_linear_bwd(_ptr(dy), _ptr(x), _ptr(w), M, K, N, fmt_dy, fmt_x, fmt_w,
                                               _ptr(dx) if need_dx else None, _ptr(dw) if need_dw else None,
                                               _ptr(workspace), workspace.numel(), _stream()))
    return dx, dw


def fp8_mx_quantize_t(x: torch.Tensor, fmt: int, qt: torch.Tensor | None = None, e8m0_t: torch.Tensor | None = None,
                      slabs: bool = False):
    """MX blocks of 32 down the columns, transposed output: codes [cols, rows], E8M0 bytes [cols, rows / 32]."""
    rows, cols, ld = _mat(x, 2)
    if qt is None:
        qt = _alloc_q(cols, rows, 0, x.device)
    if e8m0_t is None:
        e8m0_t = _alloc_e8m0(cols, rows // 32, slabs, x.device)
    _, _, ld_q = _mat(qt, 1)
    ld_e = _e8m0_ld(e8m0_t)
    _check(load_library().fp8_mx_quantize_t(_ptr(x), rows, cols, ld, fmt, _ptr(qt), ld_q, _ptr(e8m0_t), ld_e, _stream()))
    return qt, e8m0_t


def fp8_mx_quantize_row_col(x: torch.Tensor, fmt: int, out=None, slabs: bool = False):
    """Both MX orientations from one read: (q_row [rows, cols], e_row [rows, cols/32], q_col_t [cols, rows],
    e_col_t [cols, rows/32]); out: the same four tensors to write into."""
    rows, cols, ld = _mat(x, 2)
    if out is None:
        nb_r, nb_c = cols // 32, rows // 32
        out = (_alloc_q(rows, cols, 0, x.device), _alloc_e8m0(rows, nb_r, slabs, x.device),
               _alloc_q(cols, rows, 0, x.device), _alloc_e8m0(cols, nb_c, slabs, x.device))
    q_row, e_row, q_col_t, e_col_t = out
    _check(load_library().fp8_mx_quantize_row_col(_ptr(x), rows, cols, ld, fmt, _ptr(q_row), _mat(q_row, 1)[2], _ptr(e_row),
                                                  _e8m0_ld(e_row), _ptr(q_col_t), _mat(q_col_t, 1)[2], _ptr(e_col_t),
                                                  _e8m0_ld(e_col_t), _stream()))
    return q_row, e_row, q_col_t, e_col_t


def fp8_block_quantize_row_col(x: torch.Tensor, fmt: int, out=None, slabs: bool = False):
    """Blockwise tiles of 1 x 128 along the rows and, transposed, of 128 x 1 down the columns from one read:
    (q_row [rows, cols], e_row [rows, cols/32], q_col_t [cols, rows], e_col_t [cols, rows/32])."""
    rows, cols, ld = _mat(x, 2)
    if out is None:
        nb_r, nb_c = cols // 32, rows // 32
        out = (_alloc_q(rows, cols, 0, x.device), _alloc_e8m0(rows, nb_r, slabs, x.device),
               _alloc_q(cols, rows, 0, x.device), _alloc_e8m0(cols, nb_c, slabs, x.device))
    q_row, e_row, q_col_t, e_col_t = out
    _check(load_library().fp8_block_quantize_row_col(_ptr(x), rows, cols, ld, fmt, _ptr(q_row), _mat(q_row, 1)[2], _ptr(e_row),
                                                     _e8m0_ld(e_row), _ptr(q_col_t), _mat(q_col_t, 1)[2], _ptr(e_col_t),
                                                     _e8m0_ld(e_col_t), _stream()))
    return q_row, e_row, q_col_t, e_col_t


def fp8_mx_scaled_mm(a: torch.Tensor, fmt_a: int, ea: torch.Tensor, b: torch.Tensor, fmt_b: int, eb: torch.Tensor,
                     flags: int = 0, out: torch.Tensor | None = None) -> torch.Tensor:
    M, K, lda = _mat(a, 1)
    N, Kb, ldb = _mat(b, 1)
    assert K == Kb, (a.shape, b.shape)
    ld_ea, ld_eb = _e8m0_ld(ea), _e8m0_ld(eb)      # (3-D slab tensors give negative values)
    if out is None:
        dt = torch.float32 if flags & FP8_OUT_FP32 else torch.bfloat16
        pad = 4 if flags & FP8_OUT_FP32 else 8
        out = torch.empty((M, (N + pad - 1) // pad * pad), dtype=dt, device=a.device)[:, :N]
    _, _, ld_out = _mat(out, out.element_size())
    _check(load_library().fp8_mx_scaled_mm(_ptr(a), lda, fmt_a, _ptr(ea), ld_ea, _ptr(b), ldb, fmt_b, _ptr(eb), ld_eb,
                                           M, N, K, _ptr(out), ld_out, flags, _stream()))
    return out


def fp8_mx_linear_workspace_bytes(M: int, K: int, N: int) -> int:
    n = load_library().fp8_mx_linear_workspace_bytes(M, K, N)
    if n == 0:
        raise Fp8Error(-2, fp8_last_error())
    return n


def fp8_mx_linear_fwd(x: torch.Tensor, w: torch.Tensor, fmt_x: int = FP8_E4M3FN, fmt_w: int = FP8_E4M3FN,
                      y: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    M, K = x.shape
    N = w.shape[0]
    assert w.shape == (N, K) and x.is_contiguous() and w.is_contiguous()
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    if workspace is None:
        workspace = torch.empty(fp8_mx_linear_workspace_bytes(M, K, N), dtype=torch.uint8, device=x.device)
    _check(load_library().fp8_mx_linear_fwd(_ptr(x), _ptr(w), M, K, N, fmt_x, fmt_w, _ptr(y), _ptr(workspace),
                                            workspace.numel(), _stream()))
    return y


def fp8_mx_linear_bwd_workspace_bytes(M: int, K: int, N: int) -> int:
    n = load_library().fp8_mx_linear_bwd_workspace_bytes(M, K, N)
    if n == 0:
        raise Fp8Error(-2, fp8_last_error())
    return n


def fp8_mx_linear_bwd(dy: torch.Tensor, x: torch.Tensor, w: torch.Tensor, fmt_dy: int = FP8_E4M3FN,
                      fmt_x: int = FP8_E4M3FN, fmt_w: int = FP8_E4M3FN, need_dx: bool = True, need_dw: bool = True,
                      dx: torch.Tensor | None = None, dw: torch.Tensor | None = None,
                      workspace: torch.Tensor | None = None):
    """dX = dY W and dW = dY^T X with every operand in MX blocks along the contracted axis."""
    M, N = dy.shape
    K = x.shape[1]
    assert x.shape == (M, K) and w.shape == (N, K) and dy.is_contiguous() and x.is_contiguous() and w.is_contiguous()
    if need_dx and dx is None:
        dx = torch.empty((M, K), dtype=torch.bfloat16, device=dy.device)
    if need_dw and dw is None:
        dw = torch.empty((N, K), dtype=torch.bfloat16, device=dy.device)
    if workspace is None:
        workspace = torch.empty(fp8_mx_linear_bwd_workspace_bytes(M, K, N), dtype=torch.uint8, device=dy.device)
    _check(load_library().fp8_mx_linear_bwd(_ptr(dy), _ptr(x), _ptr(w), M, K, N, fmt_dy, fmt_x, fmt_w,
                                            _ptr(dx) if need_dx else None, _ptr(dw) if need_dw else None,
                                            _ptr(workspace), workspace.numel(), _stream()))
    return dx, dw
