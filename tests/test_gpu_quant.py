"""GPU parity: amax / scale / cast / fused quantize vs the CPU oracle.
Bytes and scales must match bit for bit (NaN inputs: NaN class only)."""
import numpy as np
import pytest
import torch

import synthetic_inputs as si
from oracle import fp8_oracle as orc
from tests.gpu_util import dev_bf16, dev_f32, host_f32, host_u8, same_codes

pytestmark = pytest.mark.gpu

import paper_2507_16099_amd as fp8  # noqa: E402

FMTS = [orc.E4M3FN, orc.E5M2]


def _bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


# ------------------------------------------------------------------ cast

@pytest.mark.parametrize("fmt", FMTS)
def test_cast_all_bf16_patterns_many_scales(fmt):
    """Every bfloat16 bit pattern times a set of scales: pins rounding,
    subnormals, saturation, signed zeros and denormal inputs of the hardware
    conversion against the oracle."""
    x = si.all_bf16_patterns()
    xd = dev_bf16(x)
    nan = np.isnan(si.bf16_bits_to_f32(x))
    scales = [1.0, 2.0 ** -7, 2.0 ** 9, 2.0 ** -20, 2.0 ** 30, 149.33333, 0.0123, 3.0e-5, 448e12, 5.7e16, 1.0e-30,
              float(np.float32(448.0) / np.float32(3.0)), 57344.0 / 0.37]
    for s in scales:
        sv = np.array([s], np.float32)
        got = host_u8(fp8.fp8_cast(xd, dev_f32(sv), fp8.FP8_TENSOR, fmt))
        want = orc.cast(x, sv, orc.TENSOR, fmt)
        assert same_codes(got, want, nan, fmt == orc.E4M3FN), (fmt, s, np.argwhere(got != want)[:5])


@pytest.mark.parametrize("fmt", FMTS)
def test_cast_row_col_scales_and_transpose_on_all_patterns(fmt):
    x = si.all_bf16_patterns()
    xd = dev_bf16(x)
    nan = np.isnan(si.bf16_bits_to_f32(x))
    rng = np.random.default_rng(7)
    s = np.exp(rng.uniform(-20, 20, 256)).astype(np.float32)
    for gran in (orc.ROW, orc.COL):
        for flags in (0, fp8.FP8_TRANSPOSE_OUT):
            got = host_u8(fp8.fp8_cast(xd, dev_f32(s), gran, fmt, flags))
            want = orc.cast(x, s, gran, fmt, flags)
            m = nan.T if flags else nan
            assert same_codes(got, want, m, fmt == orc.E4M3FN), (fmt, gran, flags)


@pytest.mark.parametrize("shape,ld", [((1, 1), 8), ((7, 13), 16), ((129, 100), 104), ((300, 1000), 1000),
                                      ((257, 4104), 4104), ((130, 260), 512), ((5, 4096), 4096)])
@pytest.mark.parametrize("gran", [orc.TENSOR, orc.ROW, orc.COL])
def test_cast_ragged_shapes_both_layouts(shape, ld, gran):
    x = si.normal_bf16(shape, 1.0, seed=3, stream=shape[0])
    xd = dev_bf16(x, ld)
    for fmt in FMTS:
        s = orc.scale(orc.amax(x, gran), fmt)
        for flags in (0, fp8.FP8_TRANSPOSE_OUT):
            got = host_u8(fp8.fp8_cast(xd, dev_f32(s), gran, fmt, flags))
            want = orc.cast(x, s, gran, fmt, flags)
            assert got.shape == want.shape and (got == want).all(), (shape, gran, fmt, flags)


# ------------------------------------------------------------------ amax

@pytest.mark.parametrize("shape,ld", [((1, 1), 8), ((7, 13), 16), ((129, 100), 104), ((300, 1000), 1000),
                                      ((257, 4104), 4104), ((130, 260), 512), ((3, 40000), 40000),
                                      ((2051, 520), 520), ((1, 100000), 100000)])
def test_amax_all_granularities(shape, ld):
    x = si.normal_bf16(shape, 2.5, seed=4, stream=shape[1])
    xd = dev_bf16(x, ld)
    for gran in (orc.TENSOR, orc.ROW, orc.COL):
        got = host_f32(fp8.fp8_amax(xd, gran))
        want = orc.amax(x, gran)
        assert (_bits(got) == _bits(want)).all(), (shape, gran)


def test_amax_is_dynamic_and_ignores_sign():
    x = si.normal_bf16((64, 512), 1.0, seed=5, stream=0)
    x[17, 300] = 0xC37A  # -250
    xd = dev_bf16(x)
    assert host_f32(fp8.fp8_amax(xd, fp8.FP8_TENSOR))[0] == 250.0
    assert host_f32(fp8.fp8_amax(xd, fp8.FP8_ROW))[17] == 250.0
    assert host_f32(fp8.fp8_amax(xd, fp8.FP8_COL))[300] == 250.0
    zero = torch.zeros((16, 64), dtype=torch.bfloat16, device="cuda")
    for gran in (fp8.FP8_TENSOR, fp8.FP8_ROW, fp8.FP8_COL):
        assert (host_f32(fp8.fp8_amax(zero, gran)) == 0).all()


# ------------------------------------------------------------------ scale

@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("flags", [0, 1])
def test_scale_bit_exact(fmt, flags):
    rng = np.random.default_rng(6)
    bits = rng.integers(0, 0x7F80, size=20000, dtype=np.uint32).astype(np.uint16)
    a = np.concatenate([si.bf16_bits_to_f32(bits),
                        np.array([0.0, 1e-20, 1e-12, 9.999e-13, 1.0001e-12, 1.0, 3.0, 5.25, 448.0, 57344.0, 3.3e38],
                                 np.float32)])
    got = host_f32(fp8.fp8_scale(dev_f32(a), fmt, flags))
    want = orc.scale(a, fmt, flags)
    assert (_bits(got) == _bits(want)).all()


# ------------------------------------------------------- fused quantize

@pytest.mark.parametrize("rows,cols", [(3, 8), (33, 100), (64, 512), (130, 1000), (17, 2048), (16, 4096),
                                       (9, 14336), (5, 28672), (3, 32768), (2, 40000), (1000, 72)])
@pytest.mark.parametrize("fmt", FMTS)
def test_quantize_rowwise_single_pass(rows, cols, fmt):
    x = si.normal_bf16((rows, cols), 0.7, seed=8, stream=cols)
    xd = dev_bf16(x)
    for flags in (0, fp8.FP8_POW2_SCALE):
        q, s = fp8.fp8_quantize(xd, fp8.FP8_ROW, fmt, flags)
        wq, ws = orc.quantize(x, orc.ROW, fmt, flags)
        assert (_bits(host_f32(s)) == _bits(ws)).all(), (rows, cols, fmt, flags)
        assert (host_u8(q) == wq).all(), (rows, cols, fmt, flags)


@pytest.mark.parametrize("shape", [(1, 8), (100, 200), (257, 1032), (512, 384), (130, 4096)])
@pytest.mark.parametrize("gran", [orc.TENSOR, orc.ROW, orc.COL])
@pytest.mark.parametrize("flags", [0, 2, 3])
def test_quantize_all_granularities_and_layouts(shape, gran, flags):
    x = si.normal_bf16(shape, 0.02, seed=9, stream=shape[0])
    xd = dev_bf16(x)
    for fmt in FMTS:
        q, s = fp8.fp8_quantize(xd, gran, fmt, flags)
        wq, ws = orc.quantize(x, gran, fmt, flags)
        assert (_bits(host_f32(s)) == _bits(ws)).all(), (shape, gran, fmt, flags)
        assert (host_u8(q) == wq).all(), (shape, gran, fmt, flags)


def test_quantize_zero_rows_and_outliers():
    x = si.student_t_outlier_bf16((200, 1024), 3.0, 0.004, 100.0, seed=0, stream=0)
    x[7, :] = 0
    x[9, :] = 0x8000
    xd = dev_bf16(x)
    for gran in (orc.TENSOR, orc.ROW, orc.COL):
        q, s = fp8.fp8_quantize(xd, gran, fp8.FP8_E4M3FN, 0)
        wq, ws = orc.quantize(x, gran, orc.E4M3FN, 0)
        assert (_bits(host_f32(s)) == _bits(ws)).all() and (host_u8(q) == wq).all()


@pytest.mark.parametrize("rows,cols,ld", [
    (2048, 512, 512),        # smallest shape of the fused pass: 256 blocks x 8 rows, one vector per thread
    (4100, 1024, 1032),      # ragged row count, padded leading dimension
    (8197, 2048, 2048),      # 1024 blocks, two vectors per thread
    (2500, 4104, 4104),      # partly filled last vector column
    (2050, 14336, 14336),    # benchmark row length (8 vectors per thread)
    (2048, 16392, 16392),    # 16 vectors per thread
    (2047, 512, 512),        # fewer blocks than the device could hold
    (1024, 16384, 16384),    # few long rows: 256 blocks x 4 rows
    (600, 1024, 1024), (256, 2048, 2056), (255, 512, 512),   # down to two rows per block; 255 rows: separate passes
    (100, 200, 200), (3000, 100, 104), (2048, 8, 8), (1000, 512, 512),   # shapes served by the separate passes
])
def test_quantize_row_and_column_in_two_reads(rows, cols, ld):
    """fp8_quantize_row_col == rowwise quantization + per-column transposed
    quantization of the oracle, bytes and scales bit for bit."""
    x = si.normal_bf16((rows, cols), 1e-3, seed=12, stream=rows + cols)
    x[rows // 2, :] = 0                      # an all-zero row ...
    x[:, cols // 3] = 0x8000                 # ... and an all-(negative-)zero column
    x[rows - 1, cols - 1] = 0x4e00           # a large last element (5.4e8): last row, last column
    xd = dev_bf16(x, ld)
    for fmt, flags in ((orc.E5M2, 0), (orc.E4M3FN, fp8.FP8_POW2_SCALE)):
        qr, sr, qc, sc = fp8.fp8_quantize_row_col(xd, fmt, flags)
        wr, wsr = orc.quantize(x, orc.ROW, fmt, flags)
        wc, wsc = orc.quantize(x, orc.COL, fmt, flags | orc.TRANSPOSE_OUT)
        assert (_bits(host_f32(sr)) == _bits(wsr)).all(), (rows, cols, fmt, flags)
        assert (_bits(host_f32(sc)) == _bits(wsc)).all(), (rows, cols, fmt, flags)
        assert (host_u8(qr) == wr).all(), (rows, cols, fmt, flags)
        assert (host_u8(qc) == wc).all(), (rows, cols, fmt, flags)


def test_quantize_row_col_rejects_bad_arguments():
    x = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_quantize_row_col(x, 7)
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_quantize_row_col(x, fp8.FP8_E5M2, fp8.FP8_TRANSPOSE_OUT)
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_quantize_row_col(x, fp8.FP8_E5M2, 0, q_col_t=torch.empty((64, 48), dtype=torch.uint8, device="cuda"))
    e = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    qr, sr, qc, sc = fp8.fp8_quantize_row_col(e, fp8.FP8_E5M2)
    assert qr.shape == (0, 64) and sr.numel() == 0 and (host_f32(sc) == np.float32(57344.0 / 1e-12)).all()


def test_empty_inputs_are_accepted():
    e = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    assert fp8.fp8_amax(e, fp8.FP8_ROW).numel() == 0
    assert (host_f32(fp8.fp8_amax(e, fp8.FP8_COL)) == 0).all()
    q, s = fp8.fp8_quantize(e, fp8.FP8_ROW, fp8.FP8_E4M3FN)
    assert q.shape == (0, 64) and s.numel() == 0
    torch.cuda.synchronize()


# --------------------------------------------- full benchmark-size tensors

def test_quantize_full_size_llama_ffn_operands():
    """The benchmark workload's own tensors: X [16384, 4096] and W [14336, 4096]
    per row (forward), W per column transposed (dX) and X per column
    transposed (dW); bytes and scales bit-exact on the whole tensors."""
    wl = si.WORKLOADS[si.BENCH_WORKLOAD]
    for name, bits in (("x", wl.x()), ("w", wl.w())):
        d = dev_bf16(bits)
        q, s = fp8.fp8_quantize(d, fp8.FP8_ROW, fp8.FP8_E4M3FN)
        wq, ws = orc.quantize(bits, orc.ROW, orc.E4M3FN)
        assert (_bits(host_f32(s)) == _bits(ws)).all(), name
        assert (host_u8(q) == wq).all(), name
        q, s = fp8.fp8_quantize(d, fp8.FP8_COL, fp8.FP8_E4M3FN, fp8.FP8_TRANSPOSE_OUT)
        wq, ws = orc.quantize(bits, orc.COL, orc.E4M3FN, orc.TRANSPOSE_OUT)
        assert (_bits(host_f32(s)) == _bits(ws)).all(), name
        assert (host_u8(q) == wq).all(), name
        q, s = fp8.fp8_quantize(d, fp8.FP8_TENSOR, fp8.FP8_E4M3FN)
        wq, ws = orc.quantize(bits, orc.TENSOR, orc.E4M3FN)
        assert (_bits(host_f32(s)) == _bits(ws)).all() and (host_u8(q) == wq).all(), name
        del d, q, s


def test_quantize_full_size_llama_ffn_gradient_both_axes():
    """dY [16384, 14336] of the benchmark workload through the two-read entry
    point (e5m2): rowwise codes for dX, per-column transposed codes for dW."""
    wl = si.WORKLOADS[si.BENCH_WORKLOAD]
    bits = wl.dy()
    qr, sr, qc, sc = fp8.fp8_quantize_row_col(dev_bf16(bits), fp8.FP8_E5M2)
    wr, wsr = orc.quantize(bits, orc.ROW, orc.E5M2)
    assert (_bits(host_f32(sr)) == _bits(wsr)).all()
    assert (host_u8(qr) == wr).all()
    del wr
    wc, wsc = orc.quantize(bits, orc.COL, orc.E5M2, orc.TRANSPOSE_OUT)
    assert (_bits(host_f32(sc)) == _bits(wsc)).all()
    assert (host_u8(qc) == wc).all()


@pytest.mark.parametrize("rows,cols,pad", [(4096, 1024, 16), (4096, 1024, 0), (3000, 2048, 48), (520, 512, 16)])
def test_transposed_outputs_leave_the_padding_between_rows_alone(rows, cols, pad):
    """A transposed output [cols, rows] handed in as a view of a wider buffer (ld_out = rows + pad): the per-column
    quantization may park its partial column maxima in the output before the cast, but only in bytes that the
    cast rewrites - the bytes between the rows belong to the caller and must keep their sentinel.  Both entry
    points that use the output as scratch; codes and scales still equal the oracle's."""
    x = si.normal_bf16((rows, cols), 1.0, seed=21, stream=rows + pad)
    xd = dev_bf16(x)
    wq, ws = orc.quantize(x, orc.COL, orc.E5M2, orc.TRANSPOSE_OUT)
    ld = (rows + 15) // 16 * 16 + pad
    # fp8_quantize(COL | TRANSPOSE_OUT)
    full = torch.full((cols, ld), 0xAB, dtype=torch.uint8, device="cuda")
    q, s = fp8.fp8_quantize(xd, fp8.FP8_COL, fp8.FP8_E5M2, fp8.FP8_TRANSPOSE_OUT, out=full[:, :rows])
    torch.cuda.synchronize()
    assert (_bits(host_f32(s)) == _bits(ws)).all() and (host_u8(q) == wq).all()
    assert bool((full[:, rows:] == 0xAB).all()), "padding of the transposed output was overwritten"
    # fp8_quantize_row_col: q_col_t is the padded one
    full = torch.full((cols, ld), 0xCD, dtype=torch.uint8, device="cuda")
    q_row, s_row, q_col_t, s_col = fp8.fp8_quantize_row_col(xd, fp8.FP8_E5M2, 0, q_col_t=full[:, :rows])
    torch.cuda.synchronize()
    rq, rs = orc.quantize(x, orc.ROW, orc.E5M2)
    assert (host_u8(q_row) == rq).all() and (_bits(host_f32(s_row)) == _bits(rs)).all()
    assert (host_u8(q_col_t) == wq).all() and (_bits(host_f32(s_col)) == _bits(ws)).all()
    assert bool((full[:, rows:] == 0xCD).all()), "padding of q_col_t was overwritten"
