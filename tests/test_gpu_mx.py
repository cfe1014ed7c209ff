"""GPU parity: MX (microscaling) block quantization, the block-scaled FP8 GEMM
and the MX forward vs the CPU oracle.  Codes and E8M0 bytes bit for bit; the
GEMM by relative Frobenius error <= 1e-3 (the matrix cores add the scaled
products in an order of their own), bit for bit where every partial sum is
exactly representable."""
import numpy as np
import pytest
import torch

import synthetic_inputs as si
from oracle import fp8_oracle as orc
from tests.gpu_util import dev_bf16, dev_u8, host_bf16_bits, host_f32, host_u8, knobs

pytestmark = pytest.mark.gpu

import paper_2507_16099_amd as fp8  # noqa: E402

TOL = 1e-3
FMTS = [orc.E4M3FN, orc.E5M2]


def _dev_e(e):
    rows, nb = e.shape
    full = torch.zeros((rows, (nb + 3) // 4 * 4), dtype=torch.uint8, device="cuda")
    full[:, :nb] = torch.from_numpy(np.ascontiguousarray(e)).cuda()
    return full[:, :nb]


@pytest.mark.parametrize("fmt", FMTS)
def test_mx_quantize_all_bf16_patterns(fmt):
    """Every finite bfloat16 value, in blocks that mix magnitudes (a permutation
    of all patterns) and in blocks of similar magnitude (sorted order)."""
    allp = si.all_bf16_patterns().reshape(-1)
    finite = allp[np.isfinite(si.bf16_bits_to_f32(allp))]
    n = finite.size // 32 * 32
    rng = np.random.default_rng(1)
    for arr in (finite[:n], rng.permutation(finite)[:n]):
        x = np.ascontiguousarray(arr.reshape(-1, 960))          # 65280 finite patterns = 68 rows of 30 blocks
        q, e = fp8.fp8_mx_quantize(dev_bf16(x), fmt)
        wq, we = orc.mx_quantize(x, fmt)
        assert (host_u8(e) == we).all(), np.argwhere(host_u8(e) != we)[:4]
        assert (host_u8(q) == wq).all(), np.argwhere(host_u8(q) != wq)[:4]


@pytest.mark.parametrize("rows,cols,ld", [(1, 32, 32), (7, 96, 104), (300, 1024, 1024), (33, 4128, 4128), (5, 14336, 14336)])
@pytest.mark.parametrize("fmt", FMTS)
def test_mx_quantize_shapes(rows, cols, ld, fmt):
    x = si.student_t_outlier_bf16((rows, cols), 3.0, 0.01, 100.0, seed=4, stream=rows)
    x[rows // 2, :32] = 0
    x[0, cols - 32:] = 0x8000
    q, e = fp8.fp8_mx_quantize(dev_bf16(x, ld), fmt)
    wq, we = orc.mx_quantize(x, fmt)
    assert (host_u8(e) == we).all() and (host_u8(q) == wq).all()


SHAPES = [(16, 16, 128), (33, 17, 256), (200, 300, 384), (256, 512, 512), (257, 129, 1280), (500, 70, 1024)]


@pytest.fixture(params=["0", "1"], ids=["staged", "snake"])
def mx_variant(request):
    """Both MX GEMM kernels on every shape (the dispatch would pick by problem size)."""
    with knobs(MX_VARIANT=int(request.param)):
        yield request.param


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_mx_gemm_exact_on_small_integers(mx_variant, M, N, K):
    """Integer codes and power-of-two block scales: exact, so every mistake in the
    assignment of blocks, scale bytes and rows to lanes shows up."""
    rng = np.random.default_rng(M + N + K)
    ai, bi = rng.integers(-3, 4, size=(M, K)), rng.integers(-3, 4, size=(N, K))
    for fa, fb in ((orc.E4M3FN, orc.E4M3FN), (orc.E5M2, orc.E4M3FN), (orc.E4M3FN, orc.E5M2)):
        a = orc.encode_array(ai.astype(np.float32), fa)
        b = orc.encode_array(bi.astype(np.float32), fb)
        # block scales within a factor of 4 of each other: with |sum per block| < 2^9 and at most 40
        # blocks every partial sum then fits the 24-bit significand whatever the order of addition
        ea = rng.integers(126, 129, size=(M, K // 32)).astype(np.uint8)
        eb = rng.integers(126, 129, size=(N, K // 32)).astype(np.uint8)
        want = orc.mx_mm(a, fa, ea, b, fb, eb)
        got32 = host_f32(fp8.fp8_mx_scaled_mm(dev_u8(a), fa, _dev_e(ea), dev_u8(b), fb, _dev_e(eb), fp8.FP8_OUT_FP32))
        assert (got32 == want.out32).all(), (M, N, K, fa, fb, np.argwhere(got32 != want.out32)[:4])
        got16 = host_bf16_bits(fp8.fp8_mx_scaled_mm(dev_u8(a), fa, _dev_e(ea), dev_u8(b), fb, _dev_e(eb)))
        assert (got16 == want.out16).all()


@pytest.mark.parametrize("M,N,K", [(4096, 4096, 4096), (4096, 4352, 4224), (2048, 2304, 14336)])
def test_mx_gemm_long_contraction_exact_every_element(M, N, K):
    """32, 33 and 112 K steps per tile with every CU busy: the refills of data and scale buffers overlap
    the reads for the whole contraction.  Integer codes, block scales of 1/2, 1 or 2: every partial sum
    fits the significand in any order, so the dequantized product in binary32 is exact; every element
    is checked and three launches must agree bit for bit."""
    rng = np.random.default_rng(M + N + K)
    ai = rng.integers(-3, 4, size=(M, K)).astype(np.float32)
    bi = rng.integers(-3, 4, size=(N, K)).astype(np.float32)
    a, b = orc.encode_array(ai, orc.E5M2), orc.encode_array(bi, orc.E4M3FN)
    ea = rng.integers(126, 129, size=(M, K // 32)).astype(np.uint8)
    eb = rng.integers(126, 129, size=(N, K // 32)).astype(np.uint8)
    ad = ai * np.repeat(np.exp2(ea.astype(np.float32) - 127.0), 32, axis=1)
    bd = bi * np.repeat(np.exp2(eb.astype(np.float32) - 127.0), 32, axis=1)
    exact = (ad @ bd.T).astype(np.float32)        # |sums| < 2^18 in units of 1/4: exact
    # the oracle proper on a sample of rows
    rows = si.stratified_rows(M, 8)
    want = orc.mx_mm(a, orc.E5M2, ea, b, orc.E4M3FN, eb, rows)
    assert (want.out32 == exact[rows]).all()
    for _ in range(3):
        got32 = host_f32(fp8.fp8_mx_scaled_mm(dev_u8(a), orc.E5M2, _dev_e(ea), dev_u8(b), orc.E4M3FN, _dev_e(eb), fp8.FP8_OUT_FP32))
        assert (got32 == exact).all()
        got16 = host_bf16_bits(fp8.fp8_mx_scaled_mm(dev_u8(a), orc.E5M2, _dev_e(ea), dev_u8(b), orc.E4M3FN, _dev_e(eb)))
        assert (got16 == orc.f32_to_bf16(exact)).all()


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_mx_gemm_random_codes(mx_variant, M, N, K):
    rng = np.random.default_rng(M + 3 * N + K)
    a = rng.integers(0, 0x78, size=(M, K)).astype(np.uint8) | (rng.integers(0, 2, size=(M, K)).astype(np.uint8) << 7)
    b = rng.integers(0, 0x78, size=(N, K)).astype(np.uint8) | (rng.integers(0, 2, size=(N, K)).astype(np.uint8) << 7)
    ea = rng.integers(100, 150, size=(M, K // 32)).astype(np.uint8)
    eb = rng.integers(100, 150, size=(N, K // 32)).astype(np.uint8)
    want = orc.mx_mm(a, orc.E4M3FN, ea, b, orc.E4M3FN, eb)
    got32 = host_f32(fp8.fp8_mx_scaled_mm(dev_u8(a), 0, _dev_e(ea), dev_u8(b), 0, _dev_e(eb), fp8.FP8_OUT_FP32))
    assert orc.rel_frobenius(got32, want.out32) <= TOL
    assert orc.rel_frobenius(got32, want.acc64) <= TOL


@pytest.mark.parametrize("M,K,N", [(64, 128, 64), (384, 256, 512), (208, 1152, 272), (1024, 384, 640)])
def test_mx_linear_forward(M, K, N):
    wl = si.scaled_down(si.WORKLOADS["c2_llama3_8b_ffn_rowwise"], M, K, N)
    x, w = wl.x(), wl.w()
    y = fp8.fp8_mx_linear_fwd(dev_bf16(x), dev_bf16(w))
    want = orc.mx_linear_fwd(x, w)
    got = host_bf16_bits(y)
    assert orc.rel_frobenius(si.bf16_bits_to_f32(got), si.bf16_bits_to_f32(want.out16)) <= TOL
    assert float((got == want.out16).mean()) > 0.95


def test_mx_rejects_bad_arguments():
    x = torch.zeros((4, 48), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_mx_quantize(x, fp8.FP8_E4M3FN)                    # cols not a multiple of 32
    a = torch.zeros((16, 64), dtype=torch.uint8, device="cuda")
    e = torch.zeros((16, 4), dtype=torch.uint8, device="cuda")[:, :2]
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_mx_scaled_mm(a, 0, e, a, 0, e)                     # K not a multiple of 128
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_mx_linear_workspace_bytes(16, 96, 16)


def test_mx_full_size_llama_ffn_forward_sampled_rows():
    """Benchmark shape: X [16384, 4096], W [14336, 4096]; codes and scale bytes of
    both operands on the whole tensors, the product on a stratified sample of rows."""
    wl = si.WORKLOADS[si.BENCH_WORKLOAD]
    x, w = wl.x(), wl.w()
    xq, xe = fp8.fp8_mx_quantize(dev_bf16(x), fp8.FP8_E4M3FN)
    wq, we = fp8.fp8_mx_quantize(dev_bf16(w), fp8.FP8_E4M3FN)
    oxq, oxe = orc.mx_quantize(x, orc.E4M3FN)
    owq, owe = orc.mx_quantize(w, orc.E4M3FN)
    assert (host_u8(xq) == oxq).all() and (host_u8(xe) == oxe).all()
    assert (host_u8(wq) == owq).all() and (host_u8(we) == owe).all()
    y = fp8.fp8_mx_scaled_mm(xq, 0, xe, wq, 0, we)
    rows = si.tile_band_rows(wl.M, 128)     # first and last row of every band of 256 rows
    want = orc.mx_mm(oxq, orc.E4M3FN, oxe, owq, orc.E4M3FN, owe, rows)
    got = host_bf16_bits(y[torch.from_numpy(rows).cuda()])
    assert orc.rel_frobenius(si.bf16_bits_to_f32(got), si.bf16_bits_to_f32(want.out16)) <= TOL
    assert float((got == want.out16).mean()) > 0.97


# ----------------------------------------------------------------- backward
@pytest.mark.parametrize("fmt", FMTS)
def test_mx_quantize_t_all_bf16_patterns(fmt):
    """Blocks down the columns, transposed output == the oracle on the transposed matrix."""
    allp = si.all_bf16_patterns().reshape(-1)
    finite = allp[np.isfinite(si.bf16_bits_to_f32(allp))]
    rng = np.random.default_rng(2)
    for arr in (finite[:65280], rng.permutation(finite)[:65280]):
        xt = np.ascontiguousarray(arr.reshape(-1, 960))           # [68, 960]: the transposed matrix, blocks along its rows
        x = np.ascontiguousarray(xt.T)                            # [960, 68]
        qt, et = fp8.fp8_mx_quantize_t(dev_bf16(x, 72), fmt)
        wq, we = orc.mx_quantize(xt, fmt)
        assert (host_u8(et) == we).all(), np.argwhere(host_u8(et) != we)[:4]
        assert (host_u8(qt) == wq).all(), np.argwhere(host_u8(qt) != wq)[:4]


@pytest.mark.parametrize("rows,cols,ld", [(32, 8, 8), (96, 7, 8), (128, 128, 128), (160, 300, 304), (1024, 1000, 1000),
                                          (4128, 33, 40), (2080, 2056, 2056)])
@pytest.mark.parametrize("fmt", FMTS)
def test_mx_quantize_t_shapes(rows, cols, ld, fmt):
    x = si.student_t_outlier_bf16((rows, cols), 3.0, 0.01, 100.0, seed=6, stream=rows)
    x[:32, cols // 2] = 0
    x[rows - 32:, 0] = 0x8000
    qt, et = fp8.fp8_mx_quantize_t(dev_bf16(x, ld), fmt)
    wq, we = orc.mx_quantize(np.ascontiguousarray(x.T), fmt)
    assert tuple(qt.shape) == (cols, rows) and tuple(et.shape) == (cols, rows // 32)
    assert (host_u8(et) == we).all() and (host_u8(qt) == wq).all()


@pytest.mark.parametrize("rows,cols,ld", [(32, 32, 32), (96, 160, 168), (128, 128, 128), (160, 288, 288), (1024, 992, 992),
                                          (4128, 64, 64), (2080, 2080, 2080)])
@pytest.mark.parametrize("fmt", FMTS)
def test_mx_quantize_row_col_shapes(rows, cols, ld, fmt):
    """Both orientations from one read == the two single-orientation conversions of the oracle."""
    x = si.student_t_outlier_bf16((rows, cols), 3.0, 0.01, 100.0, seed=7, stream=rows + cols)
    x[:32, cols // 2] = 0
    x[rows // 2, :32] = 0x8000
    q_row, e_row, q_col_t, e_col_t = fp8.fp8_mx_quantize_row_col(dev_bf16(x, ld), fmt)
    wq, we = orc.mx_quantize(x, fmt)
    wqt, wet = orc.mx_quantize(np.ascontiguousarray(x.T), fmt)
    assert (host_u8(e_row) == we).all() and (host_u8(q_row) == wq).all()
    assert (host_u8(e_col_t) == wet).all() and (host_u8(q_col_t) == wqt).all()


# (the last four: token and feature counts that are whole blocks of 32 but not whole K steps of 128 - the contraction
# axes are padded inside the workspace)
@pytest.mark.parametrize("M,K,N", [(128, 64, 128), (256, 8, 128), (384, 272, 512), (1024, 384, 640), (128, 1152, 256),
                                   (96, 64, 160), (416, 272, 288), (1056, 384, 672), (32, 8, 32)])
def test_mx_linear_backward(M, K, N):
    wl = si.scaled_down(si.WORKLOADS["c2_llama3_8b_ffn_rowwise"], M, K, N)
    x, w, dy = wl.x(), wl.w(), wl.dy()
    for fmt_dy in FMTS:
        dx, dw = fp8.fp8_mx_linear_bwd(dev_bf16(dy), dev_bf16(x), dev_bf16(w), fmt_dy=fmt_dy)
        wx, ww = orc.mx_linear_bwd(dy, x, w, fmt_dy=fmt_dy)
        for got, want in ((host_bf16_bits(dx), wx), (host_bf16_bits(dw), ww)):
            assert got.shape == want.out16.shape
            assert orc.rel_frobenius(si.bf16_bits_to_f32(got), si.bf16_bits_to_f32(want.out16)) <= TOL
            assert float((got == want.out16).mean()) > 0.95


def test_mx_linear_backward_exact_on_integers_and_single_outputs():
    rng = np.random.default_rng(8)
    M, K, N = 256, 96, 128
    dyi, xi, wi = rng.integers(-3, 4, size=(M, N)), rng.integers(-3, 4, size=(M, K)), rng.integers(-3, 4, size=(N, K))
    dy, x, w = (si.f32_to_bf16_bits(a.astype(np.float32)) for a in (dyi, xi, wi))
    dx, dw = fp8.fp8_mx_linear_bwd(dev_bf16(dy), dev_bf16(x), dev_bf16(w))
    assert (si.bf16_bits_to_f32(host_bf16_bits(dx)) == si.bf16_bits_to_f32(orc.f32_to_bf16((dyi @ wi).astype(np.float32)))).all()
    assert (si.bf16_bits_to_f32(host_bf16_bits(dw)) == si.bf16_bits_to_f32(orc.f32_to_bf16((dyi.T @ xi).astype(np.float32)))).all()
    only_dx, none = fp8.fp8_mx_linear_bwd(dev_bf16(dy), dev_bf16(x), dev_bf16(w), need_dw=False)
    assert none is None and torch.equal(only_dx, dx)
    none, only_dw = fp8.fp8_mx_linear_bwd(dev_bf16(dy), dev_bf16(x), dev_bf16(w), need_dx=False)
    assert none is None and torch.equal(only_dw, dw)
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_mx_linear_bwd_workspace_bytes(100, 64, 128)          # M not a multiple of 32
    xb = torch.zeros((48, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_mx_quantize_t(xb, fp8.FP8_E4M3FN)                   # rows not a multiple of 32


def test_mx_full_size_llama_ffn_backward_sampled_rows():
    """Benchmark shape: the four re-quantized operands bit for bit on the whole
    tensors, both gradients on a stratified sample of output rows."""
    wl = si.WORKLOADS[si.BENCH_WORKLOAD]
    x, w, dy = wl.x(), wl.w(), wl.dy()
    dxd, dwd = dev_bf16(x), dev_bf16(w)
    dyd = dev_bf16(dy)
    for name, src, host in (("w", dwd, w), ("x", dxd, x), ("dy", dyd, dy)):
        qt, et = fp8.fp8_mx_quantize_t(src, fp8.FP8_E4M3FN)
        oq, oe = orc.mx_quantize(np.ascontiguousarray(host.T), orc.E4M3FN)
        assert (host_u8(qt) == oq).all() and (host_u8(et) == oe).all(), name
        del qt, et, oq, oe
    q_row, e_row, q_col_t, e_col_t = fp8.fp8_mx_quantize_row_col(dyd, fp8.FP8_E4M3FN)       # the gradient, one read
    oq, oe = orc.mx_quantize(dy, orc.E4M3FN)
    assert (host_u8(q_row) == oq).all() and (host_u8(e_row) == oe).all()
    oq, oe = orc.mx_quantize(np.ascontiguousarray(dy.T), orc.E4M3FN)
    assert (host_u8(q_col_t) == oq).all() and (host_u8(e_col_t) == oe).all()
    del q_row, e_row, q_col_t, e_col_t, oq, oe
    dx, dw = fp8.fp8_mx_linear_bwd(dyd, dxd, dwd)
    rx, rw = si.tile_band_rows(wl.M, 128), si.tile_band_rows(wl.N, 112)   # first and last row of every band of 256
    wx, ww = orc.mx_linear_bwd(dy, x, w, rows_dx=rx, rows_dw=rw)
    for got, want in ((host_bf16_bits(dx[torch.from_numpy(rx).cuda()]), wx), (host_bf16_bits(dw[torch.from_numpy(rw).cuda()]), ww)):
        assert orc.rel_frobenius(si.bf16_bits_to_f32(got), si.bf16_bits_to_f32(want.out16)) <= TOL
        assert float((got == want.out16).mean()) > 0.97


@pytest.mark.parametrize("M,K,N", [(640, 1024, 896), (512, 640, 1024), (1536, 512, 1024), (1024, 1024, 640)])
def test_scale_slabs_between_quantizers_and_gemm(M, K, N):
    """Inside the MX and blockwise linear entry points the E8M0 scales travel in slabs of sixteen blocks
    ([blocks / 16][rows][16 bytes]) whenever the product that reads them runs on the LDS-DMA kernel with a
    contraction that is a multiple of 512.  Forced here on small ragged shapes (row counts that end inside
    a 256-row tile, products with and without a suitable contraction): outputs must equal the plain layout's
    bit for bit, and the oracle's within tolerance."""
    wl = si.scaled_down(si.WORKLOADS["c2_llama3_8b_ffn_rowwise"], M, K, N)
    x, w, dy = wl.x(), wl.w(), wl.dy()
    dx_, dw_, dy_ = dev_bf16(x), dev_bf16(w), dev_bf16(dy)

    def run_all():
        outs = [fp8.fp8_mx_linear_fwd(dx_, dw_)]
        outs += list(fp8.fp8_mx_linear_bwd(dy_, dx_, dw_))
        if M % 128 == 0 and N % 128 == 0 and K % 128 == 0:
            outs.append(fp8.fp8_block_linear_fwd(dx_, dw_))
            outs += list(fp8.fp8_block_linear_bwd(dy_, dx_, dw_))
        return [host_bf16_bits(o) for o in outs]

    with knobs(MX_VARIANT=1, MX_SLAB=1):
        slab = run_all()
    with knobs(MX_VARIANT=1, MX_SLAB=0):
        plain = run_all()
    assert len(slab) == len(plain)
    for a, b in zip(slab, plain):
        assert (a == b).all()
    wy = orc.mx_linear_fwd(x, w)
    wx, ww = orc.mx_linear_bwd(dy, x, w)
    for got, want in zip(slab[:3], (wy, wx, ww)):
        assert orc.rel_frobenius(si.bf16_bits_to_f32(got), si.bf16_bits_to_f32(want.out16)) <= TOL
        assert float((got == want.out16).mean()) > 0.95



# ------------------------------------------------ scale slabs at the public entry points

@pytest.mark.parametrize("rows,cols", [(32, 512), (96, 1024), (288, 1536), (640, 512), (512, 544), (1024, 512)])
@pytest.mark.parametrize("fmt", FMTS)
def test_public_quantizers_write_scale_slabs(rows, cols, fmt):
    """A negative ld_e selects slabs of sixteen blocks, [blocks / 16][rows per slab][16 bytes].  Every quantizer that
    writes E8M0 bytes must produce, in slabs, the bytes (and codes) that it produces in plain rows and that the
    oracle computes; slabs with more rows than the tensor (spare rows at the end of each slab) stay untouched there."""
    x = si.student_t_outlier_bf16((rows, cols), 3.0, 0.01, 100.0, seed=14, stream=rows + cols)
    xd = dev_bf16(x)
    wq, we = orc.mx_quantize(x, fmt)
    wqt, wet = orc.mx_quantize(np.ascontiguousarray(x.T), fmt)
    if rows % 512 == 0:                      # blocks down the columns: rows / 32 of them per scale row
        qt, et = fp8.fp8_mx_quantize_t(xd, fmt, slabs=True)
        assert tuple(et.shape) == (rows // 512, cols, 16)
        assert (host_u8(qt) == wqt).all() and (host_u8(fp8.e8m0_plain_rows(et)) == wet).all()
    if cols % 512 != 0:
        with pytest.raises(fp8.Fp8Error):    # blocks along the rows do not fill whole slabs
            fp8.fp8_mx_quantize(xd, fmt, e8m0=torch.empty((cols // 512 + 1, rows, 16), dtype=torch.uint8, device="cuda"))
        return
    q, e = fp8.fp8_mx_quantize(xd, fmt, slabs=True)
    assert e.dim() == 3 and tuple(e.shape) == (cols // 512, rows, 16)
    assert (host_u8(q) == wq).all() and (host_u8(fp8.e8m0_plain_rows(e)) == we).all()
    # spare rows in every slab: a sentinel there survives
    spare = torch.full((cols // 512, rows + 5, 16), 0xA5, dtype=torch.uint8, device="cuda")
    q2, e2 = fp8.fp8_mx_quantize(xd, fmt, e8m0=spare)
    assert (host_u8(q2) == wq).all()
    assert (host_u8(fp8.e8m0_plain_rows(e2))[:rows] == we).all() and (host_u8(spare)[:, rows:, :] == 0xA5).all()


@pytest.mark.parametrize("rows,cols", [(512, 512), (1024, 640)])
def test_public_row_col_and_block_quantizers_write_scale_slabs(rows, cols):
    """The two-orientation quantizers and the blockwise ones in slabs against their own plain-row output."""
    x = si.student_t_outlier_bf16((rows, cols), 3.0, 0.01, 100.0, seed=15, stream=rows)
    xd = dev_bf16(x)
    fmt = orc.E4M3FN
    for fn in (fp8.fp8_mx_quantize_row_col, fp8.fp8_block_quantize_row_col):
        if fn is fp8.fp8_block_quantize_row_col and (rows % 128 or cols % 128):
            continue
        plain = fn(xd, fmt)
        # slabs only where the blocks of a row fill whole slabs: the row direction needs cols % 512, the column direction rows % 512
        out = (torch.empty_like(plain[0]),
               torch.empty((cols // 512, rows, 16), dtype=torch.uint8, device="cuda") if cols % 512 == 0 else torch.empty_like(plain[1]),
               torch.empty_like(plain[2]),
               torch.empty((rows // 512, cols, 16), dtype=torch.uint8, device="cuda") if rows % 512 == 0 else torch.empty_like(plain[3]))
        got = fn(xd, fmt, out=out)
        for a, b in zip(got, plain):
            assert (host_u8(fp8.e8m0_plain_rows(a)) == host_u8(fp8.e8m0_plain_rows(b))).all()
    for br in (1, 128):
        if cols % 512 == 0 and rows % 128 == 0:
            pq, pe = fp8.fp8_block_quantize(xd, br, fmt)
            sq, se = fp8.fp8_block_quantize(xd, br, fmt, slabs=True)
            assert (host_u8(sq) == host_u8(pq)).all() and (host_u8(fp8.e8m0_plain_rows(se)) == host_u8(pe)).all()
        if rows % 512 == 0:
            pq, pe = fp8.fp8_block_quantize_t(xd, br, fmt)
            sq, se = fp8.fp8_block_quantize_t(xd, br, fmt, slabs=True)
            assert (host_u8(sq) == host_u8(pq)).all() and (host_u8(fp8.e8m0_plain_rows(se)) == host_u8(pe)).all()


@pytest.mark.parametrize("M,N,K", [(256, 512, 512), (200, 300, 1024), (640, 896, 1536), (33, 17, 512)])
def test_public_mx_product_takes_scale_slabs(M, N, K):
    """fp8_mx_scaled_mm with both scale arrays in slabs: the result of the plain-row call on the same kernel bit for
    bit, and the oracle's product within tolerance (exact on these small-integer operands)."""
    rng = np.random.default_rng(M + N + K)
    a = orc.encode_array(rng.integers(-3, 4, (M, K)).astype(np.float32), orc.E4M3FN)
    b = orc.encode_array(rng.integers(-3, 4, (N, K)).astype(np.float32), orc.E4M3FN)
    # (block scales within a factor of 4 and at most 48 blocks: every partial sum fits the significand in any order)
    ea = rng.integers(126, 129, (M, K // 32)).astype(np.uint8)
    eb = rng.integers(126, 129, (N, K // 32)).astype(np.uint8)
    ad, bd = dev_u8(a), dev_u8(b)

    def slabs(e, spare):
        rows, nb = e.shape
        t = torch.full((nb // 16, rows + spare, 16), 0x7F, dtype=torch.uint8, device="cuda")
        t[:, :rows, :] = torch.from_numpy(np.ascontiguousarray(e.reshape(rows, nb // 16, 16).transpose(1, 0, 2))).cuda()
        return t
    want = orc.mx_mm(a, orc.E4M3FN, ea, b, orc.E4M3FN, eb)
    got_slab = fp8.fp8_mx_scaled_mm(ad, fp8.FP8_E4M3FN, slabs(ea, 3), bd, fp8.FP8_E4M3FN, slabs(eb, 0), fp8.FP8_OUT_FP32)
    with knobs(MX_VARIANT=1):
        got_plain = fp8.fp8_mx_scaled_mm(ad, fp8.FP8_E4M3FN, _dev_e(ea), bd, fp8.FP8_E4M3FN, _dev_e(eb), fp8.FP8_OUT_FP32)
    assert torch.equal(got_slab, got_plain)
    assert (host_f32(got_slab) == want.out32).all()
    # one operand in slabs, the other in plain rows: refused
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_mx_scaled_mm(ad, fp8.FP8_E4M3FN, slabs(ea, 0), bd, fp8.FP8_E4M3FN, _dev_e(eb))


def test_public_scale_slabs_full_size_forward():
    """The benchmark's forward product with its scales in slabs, from the public quantizer to the public product:
    bit-identical to the plain-row route on the same kernel."""
    wl = si.WORKLOADS[si.BENCH_WORKLOAD]
    xd, wd = dev_bf16(wl.x()), dev_bf16(wl.w())
    xq, xe = fp8.fp8_mx_quantize(xd, fp8.FP8_E4M3FN)
    wq, we = fp8.fp8_mx_quantize(wd, fp8.FP8_E4M3FN)
    xq2, xe2 = fp8.fp8_mx_quantize(xd, fp8.FP8_E4M3FN, slabs=True)
    wq2, we2 = fp8.fp8_mx_quantize(wd, fp8.FP8_E4M3FN, slabs=True)
    assert torch.equal(xq, xq2) and torch.equal(wq, wq2)
    assert torch.equal(fp8.e8m0_plain_rows(xe2), xe) and torch.equal(fp8.e8m0_plain_rows(we2), we)
    y_plain = fp8.fp8_mx_scaled_mm(xq, fp8.FP8_E4M3FN, xe, wq, fp8.FP8_E4M3FN, we)
    y_slab = fp8.fp8_mx_scaled_mm(xq2, fp8.FP8_E4M3FN, xe2, wq2, fp8.FP8_E4M3FN, we2)
    assert torch.equal(y_plain.view(torch.int16), y_slab.view(torch.int16))
