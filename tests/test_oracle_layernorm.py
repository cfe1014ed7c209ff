"""Pins of the oracle's layer normalisation (the operation in front of the
linear layer in the paper's float8 microbenchmark, appendix "Float8 Training
Microbenchmarks") and of its single-rounding binary64 -> bfloat16 conversion:
closed forms, invariances that hold exactly, and the double-rounding trap."""
import math

import numpy as np
import pytest

import synthetic_inputs as si
from oracle import fp8_oracle as orc


def _bf16(v):
    return si.f32_to_bf16_bits(np.asarray(v, np.float32))


def _f(bits):
    return si.bf16_bits_to_f32(np.asarray(bits, np.uint16))


def test_f64_to_bf16_is_one_rounding():
    # agrees with the binary32 path wherever the value is a binary32 number
    allp = si.all_bf16_patterns().reshape(-1)
    for b in allp[::97]:
        v = float(_f([b])[0])
        if math.isnan(v):
            continue
        assert orc.f64_to_bf16(v) == int(b)
    rng = np.random.default_rng(0)
    f = rng.standard_normal(2000).astype(np.float32) * np.float32(10.0) ** rng.integers(-30, 30, 2000).astype(np.float32)
    want = orc.f32_to_bf16(f)
    assert all(orc.f64_to_bf16(float(v)) == int(w) for v, w in zip(f, want))
    # ties to even, and the double-rounding trap: just above the tie between 1 and 1 + 2^-7; binary32 would
    # first round the 2^-30 away, land on the tie and go to the even side (1.0)
    assert orc.f64_to_bf16(1.0 + 2.0 ** -8) == 0x3F80
    assert orc.f64_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82
    assert orc.f64_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -30) == 0x3F81
    assert orc.f64_to_bf16(-(1.0 + 2.0 ** -8 + 2.0 ** -30)) == 0xBF81
    assert orc.f64_to_bf16(1.0 + 2.0 ** -8 - 2.0 ** -30) == 0x3F80
    # subnormals (quantum 2^-133), overflow, zeros
    assert orc.f64_to_bf16(2.0 ** -133) == 0x0001
    assert orc.f64_to_bf16(2.0 ** -134) == 0x0000           # tie between 0 and the smallest subnormal -> even
    assert orc.f64_to_bf16(1.5 * 2.0 ** -133) == 0x0002     # tie between 1 and 2 quanta -> even
    assert orc.f64_to_bf16(2.0 ** -126) == 0x0080
    assert orc.f64_to_bf16(float(np.finfo(np.float32).max)) == 0x7F80      # above the largest bfloat16 + half ulp
    assert orc.f64_to_bf16(3.3895313892515355e38) == 0x7F7F                # the largest bfloat16 itself
    assert orc.f64_to_bf16(-0.0) == 0x8000 and orc.f64_to_bf16(0.0) == 0x0000


def test_closed_form_row():
    # [1, 2, 3, 4]: mean 2.5, biased variance 1.25 (the unbiased one would be 5/3)
    x = _bf16([[1, 2, 3, 4]])
    one = _bf16([1, 1, 1, 1])
    h, mean, rstd = orc.layernorm(x, one, None, 0.0)
    assert mean[0] == 2.5 and rstd[0] == 1.0 / math.sqrt(1.25)
    want = [orc.f64_to_bf16(v / math.sqrt(1.25)) for v in (-1.5, -0.5, 0.5, 1.5)]
    assert list(h[0]) == want
    assert abs(float(_f(h)[0, 3]) - 1.3416407865) < 2 ** -8
    # eps enters under the root
    h2, _, rstd2 = orc.layernorm(x, one, None, 0.75)
    assert rstd2[0] == 1.0 / math.sqrt(2.0)
    assert list(h2[0]) == [orc.f64_to_bf16(v / math.sqrt(2.0)) for v in (-1.5, -0.5, 0.5, 1.5)]
    # affine part: gamma per column, beta added after
    g, b = _bf16([2, -1, 0.5, 4]), _bf16([10, 20, 30, 40])
    h3, _, _ = orc.layernorm(x, g, b, 0.0)
    assert list(h3[0]) == [orc.f64_to_bf16(v / math.sqrt(1.25) * gg + bb)
                           for v, gg, bb in zip((-1.5, -0.5, 0.5, 1.5), (2, -1, 0.5, 4), (10, 20, 30, 40))]


def test_constant_row_gives_beta():
    x = _bf16(np.full((3, 64), 7.0))
    g, b = _bf16(np.linspace(1, 2, 64)), _bf16(np.linspace(-1, 1, 64))
    h, mean, rstd = orc.layernorm(x, g, b, 1e-5)
    assert (mean == 7.0).all() and np.allclose(rstd, 1.0 / math.sqrt(1e-5), rtol=1e-15)
    assert (h == b[None, :]).all()


def test_exact_invariances():
    rng = np.random.default_rng(1)
    xi = rng.integers(-8, 9, size=(5, 96)).astype(np.float32)
    g, b = _bf16(rng.integers(1, 4, 96)), _bf16(rng.integers(-2, 3, 96))
    h0, m0, r0 = orc.layernorm(_bf16(xi), g, b, 0.0)
    # a shift that stays exactly representable changes nothing: every difference x - mean is the same number
    h1, m1, _ = orc.layernorm(_bf16(xi + 16.0), g, b, 0.0)
    assert (h1 == h0).all() and (m1 == m0 + 16.0).all()
    # scaling by a power of two cancels exactly when eps = 0
    h2, _, r2 = orc.layernorm(_bf16(xi * 4.0), g, b, 0.0)
    assert (h2 == h0).all() and np.array_equal(r2, r0 / 4.0)
    # gamma scaled by two with beta = 0 doubles the output exactly
    hz, _, _ = orc.layernorm(_bf16(xi), g, None, 0.0)
    hd, _, _ = orc.layernorm(_bf16(xi), _bf16(_f(g) * 2.0), None, 0.0)
    assert (_f(hd) == 2.0 * _f(hz)).all()
    # rows are independent and the padding of a wider leading dimension is ignored
    wide = np.full((5, 104), 0x7F00, np.uint16)
    wide[:, :96] = _bf16(xi)
    h3, _, _ = orc.layernorm(wide[:, :96], g, b, 0.0)
    assert (h3 == h0).all()


def test_statistics_of_the_output_and_quantization():
    M, K = 64, 512
    x = si.normal_bf16((M, K), 3.0, seed=3, stream=0)
    one, zero = _bf16(np.ones(K)), _bf16(np.zeros(K))
    h, mean, rstd = orc.layernorm(x, one, zero, 1e-5)
    hf = _f(h).astype(np.float64)
    assert np.abs(hf.mean(axis=1)).max() < 2e-3 and np.abs(hf.var(axis=1) - 1.0).max() < 5e-3
    xf = _f(x).astype(np.float64)
    assert np.allclose(mean, xf.mean(axis=1), rtol=0, atol=1e-12)
    assert np.allclose(rstd, 1.0 / np.sqrt(xf.var(axis=1) + 1e-5), rtol=1e-12)
    # the quantized form is the ordinary rowwise quantization of that bfloat16 tensor
    h2, q, s, _, _ = orc.layernorm_quantize(x, one, zero, 1e-5)
    wq, ws = orc.quantize(h, orc.ROW, orc.E4M3FN)
    assert (h2 == h).all() and (q == wq).all() and (s.view(np.uint32) == ws.view(np.uint32)).all()
    assert (np.abs(_f(h)).max(axis=1) * s <= 448.0 * (1 + 2 ** -23)).all()


def test_sigmoid_closed_forms_and_symmetry():
    # sigmoid(ln 3) = 3/4, sigmoid(ln 7) = 7/8, sigmoid(-ln 3) = 1/4, sigmoid(0) = 1/2: all bfloat16 numbers
    v = np.array([0.0, math.log(3.0), math.log(7.0), -math.log(3.0), 40.0, -200.0], np.float32)
    y = orc.sigmoid_bf16(v)
    assert list(y[:4]) == [0x3F00, 0x3F40, 0x3F60, 0x3E80]
    assert y[4] == 0x3F80 and y[5] == 0x0000                      # saturates to 1 and underflows to 0
    rng = np.random.default_rng(2)
    z = (rng.standard_normal(4096) * 3).astype(np.float32)
    a, b = _f(orc.sigmoid_bf16(z)).astype(np.float64), _f(orc.sigmoid_bf16(-z)).astype(np.float64)
    assert np.abs(a + b - 1.0).max() <= 2.0 ** -8                 # sigmoid(-v) = 1 - sigmoid(v), up to the two roundings
    zs = np.sort(z)
    assert (np.diff(_f(orc.sigmoid_bf16(zs))) >= 0).all()         # monotone
    assert ((a > 0) & (a <= 1)).all()


def test_sigmoid_bwd_closed_forms():
    # y = 1/2: dz = dy / 4 exactly; y = 3/4: dz = 3 dy / 16 exactly; y in {0, 1}: 0
    dy = _bf16([1.0, -2.0, 3.0, 1.0, 5.0, -7.0, 1.0])
    y = _bf16([0.5, 0.5, 0.75, 0.25, 0.0, 1.0, 0.875])
    dz = _f(orc.sigmoid_bwd(dy, y))
    assert list(dz) == [0.25, -0.5, 0.5625, 0.1875, 0.0, -0.0, 0.109375]
    # symmetric in y <-> 1 - y wherever 1 - y is a bfloat16 number, odd in dy
    ys = _bf16(np.arange(1, 128) / 128.0)
    g = _bf16(np.full(127, 1.5))
    a, b = orc.sigmoid_bwd(g, ys), orc.sigmoid_bwd(g, _bf16(1.0 - _f(ys)))
    assert (a == b).all()
    assert (_f(orc.sigmoid_bwd(_bf16(-_f(g)), ys)) == -_f(a)).all()
    # the result is the bfloat16 nearest to the exact product (the binary32 steps lose nothing that matters
    # for numbers of this size): compare with exact rational arithmetic
    from fractions import Fraction
    rng = np.random.default_rng(5)
    gy = _bf16(rng.standard_normal(300))
    yy = _bf16(rng.uniform(0.01, 0.99, 300))
    got = orc.sigmoid_bwd(gy, yy)
    for i in range(300):
        exact = Fraction(float(_f(gy[i:i+1])[0])) * Fraction(float(_f(yy[i:i+1])[0])) * (1 - Fraction(float(_f(yy[i:i+1])[0])))
        lo, hi = sorted((float(_f(got[i:i+1])[0]), float(exact)))
        # within half a bfloat16 step (2^-9 relative) plus the binary32 rounding of the last product
        assert abs(Fraction(float(_f(got[i:i+1])[0])) - exact) <= abs(exact) * Fraction(1, 2 ** 8)
    # peak of y (1 - y) at y = 1/2
    assert _f(orc.sigmoid_bwd(_bf16([1.0] * 3), _bf16([0.4375, 0.5, 0.5625]))).argmax() == 1
