"""GPU parity: blockwise FP8 (tiles of 1 x 128 for activations, blocks of
128 x 128 for weights, power-of-two scales as E8M0 bytes) vs the CPU oracle.
Codes and scale bytes bit for bit; the forward product by relative Frobenius
error <= 1e-3 and bit-identical to fp8_mx_scaled_mm on the same operands."""
import numpy as np
import pytest
import torch

import synthetic_inputs as si
from oracle import fp8_oracle as orc
from tests.gpu_util import dev_bf16, host_bf16_bits, host_u8

pytestmark = pytest.mark.gpu

import paper_2507_16099_amd as fp8  # noqa: E402

TOL = 1e-3
FMTS = [orc.E4M3FN, orc.E5M2]


def _check(x, br, fmt, ld=None):
    q, e = fp8.fp8_block_quantize(dev_bf16(x, ld), br, fmt)
    wq, we = orc.block_quantize(x, br, 128, fmt)
    ge, gq = host_u8(e), host_u8(q)
    assert (ge == we).all(), (np.argwhere(ge != we)[:4], ge[ge != we][:4], we[ge != we][:4])
    assert (gq == wq).all(), np.argwhere(gq != wq)[:4]


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("br", [1, 128])
def test_block_quantize_all_bf16_patterns(br, fmt):
    """Every finite bfloat16 value: sorted (blocks of similar magnitude) and permuted (mixed magnitudes)."""
    allp = si.all_bf16_patterns().reshape(-1)
    finite = allp[np.isfinite(si.bf16_bits_to_f32(allp))]
    rng = np.random.default_rng(3)
    for arr in (finite[:65280], rng.permutation(finite)[:65280]):
        _check(np.ascontiguousarray(arr.reshape(-1, 384)), br, fmt)           # 170 rows of three tiles


@pytest.mark.parametrize("rows,cols,ld", [(1, 128, 128), (5, 256, 264), (130, 384, 384), (300, 1024, 1040),
                                          (257, 4096, 4096), (1024, 14336, 14336)])
@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("br", [1, 128])
def test_block_quantize_shapes(rows, cols, ld, br, fmt):
    x = si.student_t_outlier_bf16((rows, cols), 3.0, 0.01, 100.0, seed=6, stream=rows + br)
    x[rows // 2, :128] = 0                   # an all-zero tile
    x[:128, cols - 128:] = 0x8000            # an all-(negative-)zero block
    _check(x, br, fmt, ld)


@pytest.mark.parametrize("fmt", FMTS)
def test_every_bfloat16_magnitude_as_block_maximum(fmt):
    """The kernels derive the power-of-two scale from the exponent and mantissa of the block maximum instead of
    dividing: every finite bfloat16 magnitude (zero and subnormals included) as the maximum of a 1 x 128 tile, and a
    sample of 4096 of them, with the decision boundaries, as the maximum of a 128 x 128 block."""
    mags = np.arange(0, 0x7F80, dtype=np.uint16)                        # 32640 magnitudes, Inf / NaN excluded
    rng = np.random.default_rng(10)
    x = np.zeros((mags.size, 128), np.uint16)
    x[:, 0] = mags | (rng.integers(0, 2, mags.size).astype(np.uint16) << 15)
    x[:, 1] = mags // 2                                                  # a smaller companion in every tile
    _check(np.ascontiguousarray(x.reshape(-1, 512)), 1, fmt)
    pick = np.unique(np.concatenate([np.linspace(0, 0x7F7F, 3900).astype(np.int64),
                                     np.arange(0x2B80, 0x2BA0),                                   # around 1e-12
                                     (np.arange(60, 200)[:, None] * 128 + np.array([95, 96, 97])).ravel()]))[:4096]
    y = np.zeros((128, pick.size * 128), np.uint16)
    y[rng.integers(0, 128, pick.size), np.arange(pick.size) * 128 + rng.integers(0, 128, pick.size)] = mags[pick]
    _check(y, 128, fmt)


SHAPES = [(16, 16, 128), (33, 136, 256), (200, 304, 384), (257, 136, 1280), (1024, 768, 512)]


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_block_linear_forward(M, N, K):
    wl = si.scaled_down(si.WORKLOADS["c2_llama3_8b_ffn_rowwise"], M, K, N)
    x, w = wl.x(), wl.w()
    y = fp8.fp8_block_linear_fwd(dev_bf16(x), dev_bf16(w))
    want = orc.block_linear_fwd(x, w)
    got = host_bf16_bits(y)
    assert orc.rel_frobenius(si.bf16_bits_to_f32(got), si.bf16_bits_to_f32(want.out16)) <= TOL
    assert float((got == want.out16).mean()) > 0.97
    # the same operands through the block-scaled GEMM entry point: identical bits
    xq, xe = fp8.fp8_block_quantize(dev_bf16(x), 1, fp8.FP8_E4M3FN)
    wq, we = fp8.fp8_block_quantize(dev_bf16(w), 128, fp8.FP8_E4M3FN)
    y2 = fp8.fp8_mx_scaled_mm(xq, 0, xe, wq, 0, we)
    assert torch.equal(y.view(torch.int16), y2.contiguous().view(torch.int16))


def test_block_linear_exact_on_small_integers():
    """Integer operands: every product and partial sum is exact, so the result must be the integer matrix product."""
    rng = np.random.default_rng(4)
    M, N, K = 96, 160, 256
    xi = rng.integers(-3, 4, (M, K)).astype(np.float32)
    wi = rng.integers(-2, 3, (N, K)).astype(np.float32)
    x, w = si.f32_to_bf16_bits(xi), si.f32_to_bf16_bits(wi)
    y = fp8.fp8_block_linear_fwd(dev_bf16(x), dev_bf16(w))
    want = si.f32_to_bf16_bits((xi.astype(np.float64) @ wi.astype(np.float64).T).astype(np.float32))
    assert (host_bf16_bits(y) == want).all()


def test_block_arguments_are_checked():
    x = dev_bf16(si.normal_bf16((16, 256), 1.0, seed=1, stream=1))
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_block_quantize(x, 64, fp8.FP8_E4M3FN)                     # block_rows
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_block_quantize(x[:, :192].contiguous(), 1, fp8.FP8_E4M3FN)  # cols % 128
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_block_quantize(x, 1, 9)                                   # format
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_block_linear_workspace_bytes(16, 192, 16)                 # K % 128
    q, e = fp8.fp8_block_quantize(x[:0], 128, fp8.FP8_E4M3FN)             # empty: accepted, nothing written
    assert q.shape[0] == 0 and e.shape[0] == 0


def test_block_full_size_llama_ffn_forward_sampled_rows():
    """Benchmark shape: X [16384, 4096] in tiles, W [14336, 4096] in blocks: codes and scale bytes on the whole
    tensors, the product on a stratified sample of rows."""
    wl = si.WORKLOADS[si.BENCH_WORKLOAD]
    x, w = wl.x(), wl.w()
    xd, wd = dev_bf16(x), dev_bf16(w)
    xq, xe = fp8.fp8_block_quantize(xd, 1, fp8.FP8_E4M3FN)
    wq, we = fp8.fp8_block_quantize(wd, 128, fp8.FP8_E4M3FN)
    oxq, oxe = orc.block_quantize(x, 1, 128, orc.E4M3FN)
    owq, owe = orc.block_quantize(w, 128, 128, orc.E4M3FN)
    assert (host_u8(xq) == oxq).all() and (host_u8(xe) == oxe).all()
    assert (host_u8(wq) == owq).all() and (host_u8(we) == owe).all()
    y = fp8.fp8_block_linear_fwd(xd, wd)
    rows = si.tile_band_rows(wl.M, 128)     # first and last row of every band of 256 rows
    want = orc.mx_mm(oxq, orc.E4M3FN, oxe, owq, orc.E4M3FN, owe, rows)
    got = host_bf16_bits(y[torch.from_numpy(rows).cuda()])
    assert orc.rel_frobenius(si.bf16_bits_to_f32(got), si.bf16_bits_to_f32(want.out16)) <= TOL
    assert float((got == want.out16).mean()) > 0.97


# ----------------------------------------------------------------- backward
@pytest.mark.parametrize("rows,cols,ld", [(128, 8, 8), (128, 136, 136), (256, 384, 392), (384, 1000, 1000), (1024, 4096, 4096)])
@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("br", [1, 128])
def test_block_quantize_t_shapes(rows, cols, ld, br, fmt):
    """Transposed output == the oracle's blockwise quantization of the transposed matrix."""
    x = si.student_t_outlier_bf16((rows, cols), 3.0, 0.01, 100.0, seed=8, stream=rows + br)
    x[:128, 0] = 0                           # an all-zero tile of 128 rows x 1 column
    x[:, cols - 1] = 0x8000
    qt, et = fp8.fp8_block_quantize_t(dev_bf16(x, ld), br, fmt)
    wq, we = orc.block_quantize(np.ascontiguousarray(x.T), br, 128, fmt)
    ge, gq = host_u8(et), host_u8(qt)
    assert (ge == we).all(), (np.argwhere(ge != we)[:4], ge[ge != we][:4], we[ge != we][:4])
    assert (gq == wq).all(), np.argwhere(gq != wq)[:4]


@pytest.mark.parametrize("fmt", FMTS)
def test_block_quantize_t_every_magnitude_as_maximum(fmt):
    mags = np.arange(0, 0x7F80, dtype=np.uint16)
    rng = np.random.default_rng(12)
    xt = np.zeros((mags.size, 128), np.uint16)                          # x^T: one tile of 1 x 128 per row
    xt[np.arange(mags.size), rng.integers(0, 128, mags.size)] = mags | (rng.integers(0, 2, mags.size).astype(np.uint16) << 15)
    x = np.ascontiguousarray(xt.T)                                      # [128, 32640]
    qt, et = fp8.fp8_block_quantize_t(dev_bf16(x), 1, fmt)
    wq, we = orc.block_quantize(xt, 1, 128, fmt)
    assert (host_u8(et) == we).all() and (host_u8(qt) == wq).all()


@pytest.mark.parametrize("rows,cols,ld", [(128, 128, 128), (256, 384, 392), (384, 1024, 1024), (1024, 4096, 4096)])
@pytest.mark.parametrize("fmt", FMTS)
def test_block_quantize_row_col_from_one_read(rows, cols, ld, fmt):
    x = si.student_t_outlier_bf16((rows, cols), 3.0, 0.01, 100.0, seed=9, stream=rows)
    x[5, :128] = 0
    x[:128, 7] = 0x8000
    q_row, e_row, q_col_t, e_col_t = fp8.fp8_block_quantize_row_col(dev_bf16(x, ld), fmt)
    wq, we = orc.block_quantize(x, 1, 128, fmt)
    assert (host_u8(e_row) == we).all() and (host_u8(q_row) == wq).all()
    wq, we = orc.block_quantize(np.ascontiguousarray(x.T), 1, 128, fmt)
    assert (host_u8(e_col_t) == we).all() and (host_u8(q_col_t) == wq).all()
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_block_quantize_row_col(dev_bf16(x[:, :cols - 64] if cols > 128 else x[:64]), fmt)   # a dimension not % 128


@pytest.mark.parametrize("M,N,K", [(128, 128, 128), (128, 256, 136), (384, 128, 520), (256, 384, 1000), (1024, 768, 512)])
def test_block_linear_backward(M, N, K):
    wl = si.scaled_down(si.WORKLOADS["c2_llama3_8b_ffn_rowwise"], M, K, N)
    x, w, dy = wl.x(), wl.w(), wl.dy()
    dx, dw = fp8.fp8_block_linear_bwd(dev_bf16(dy), dev_bf16(x), dev_bf16(w))
    wx, ww = orc.block_linear_bwd(dy, x, w)
    for got_t, want in ((dx, wx), (dw, ww)):
        got = host_bf16_bits(got_t)
        assert orc.rel_frobenius(si.bf16_bits_to_f32(got), si.bf16_bits_to_f32(want.out16)) <= TOL
        assert float((got == want.out16).mean()) > 0.97
    # one output only: the same bits
    a, none = fp8.fp8_block_linear_bwd(dev_bf16(dy), dev_bf16(x), dev_bf16(w), need_dw=False)
    assert none is None and torch.equal(a.view(torch.int16), dx.view(torch.int16))
    none, b = fp8.fp8_block_linear_bwd(dev_bf16(dy), dev_bf16(x), dev_bf16(w), need_dx=False)
    assert none is None and torch.equal(b.view(torch.int16), dw.view(torch.int16))
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_block_linear_bwd_workspace_bytes(M + 64, K, N)          # M % 128


def test_block_full_size_llama_ffn_backward_sampled_rows():
    """Benchmark shape: the four re-quantized operands bit for bit on the whole tensors, both gradients on a
    stratified sample of output rows."""
    wl = si.WORKLOADS[si.BENCH_WORKLOAD]
    x, w, dy = wl.x(), wl.w(), wl.dy()
    xd, wd, dyd = dev_bf16(x), dev_bf16(w), dev_bf16(dy)
    for name, src, host, br in (("w", wd, w, 128), ("x", xd, x, 1), ("dy", dyd, dy, 1)):
        qt, et = fp8.fp8_block_quantize_t(src, br, fp8.FP8_E4M3FN)
        oq, oe = orc.block_quantize(np.ascontiguousarray(host.T), br, 128, orc.E4M3FN)
        assert (host_u8(qt) == oq).all() and (host_u8(et) == oe).all(), name
        del qt, et, oq, oe
    q, e, qt, et = fp8.fp8_block_quantize_row_col(dyd, fp8.FP8_E4M3FN)          # the gradient, one read
    oq, oe = orc.block_quantize(dy, 1, 128, orc.E4M3FN)
    assert (host_u8(q) == oq).all() and (host_u8(e) == oe).all()
    oq, oe = orc.block_quantize(np.ascontiguousarray(dy.T), 1, 128, orc.E4M3FN)
    assert (host_u8(qt) == oq).all() and (host_u8(et) == oe).all()
    del q, e, qt, et, oq, oe
    dx, dw = fp8.fp8_block_linear_bwd(dyd, xd, wd)
    rx, rw = si.tile_band_rows(wl.M, 128), si.tile_band_rows(wl.N, 112)   # first and last row of every band of 256
    wx, ww = orc.block_linear_bwd(dy, x, w, rows_dx=rx, rows_dw=rw)
    for got, want in ((host_bf16_bits(dx[torch.from_numpy(rx).cuda()]), wx), (host_bf16_bits(dw[torch.from_numpy(rw).cuda()]), ww)):
        assert orc.rel_frobenius(si.bf16_bits_to_f32(got), si.bf16_bits_to_f32(want.out16)) <= TOL
        assert float((got == want.out16).mean()) > 0.97
