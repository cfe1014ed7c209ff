"""Pins of the oracle's MX (microscaling) block quantization and MX matrix
product against what the OCP Microscaling Formats specification v1.0 fixes
(Section 5: E8M0 scale, value 2^(byte-127); Section 6.3: shared exponent =
floor(log2(max|V|)) - emax_elem, elements = RNE of V/X clamped to the largest
normal): hand-worked blocks, an independent rational-arithmetic conversion
through the search encoder, scale equivariance, error bounds, brute force."""
import math
from fractions import Fraction

import numpy as np
import pytest

import synthetic_inputs as si
from oracle import fp8_oracle as orc

FMTS = [orc.E4M3FN, orc.E5M2]
EMAX = {orc.E4M3FN: 8, orc.E5M2: 15}


def _bf16(vals):
    return si.f32_to_bf16_bits(np.asarray(vals, np.float32))


def test_hand_worked_blocks_e4m3():
    # block 1: max 1.0 -> floor(log2) = 0, shared exponent -8, byte 119, X = 2^-8;
    #          1.0 / X = 256 = 2^8 -> S.1111.000 = 0x78;  0.5 / X = 128 -> 0x70
    # block 2: all zero -> byte 0, codes 0 (sign kept: -0 -> 0x80)
    # block 3: max 448 -> floor(log2 448) = 8, shared exponent 0, byte 127, X = 1;
    #          3.0 -> 1.5 * 2^1 -> 0x44;  -448 -> 0xFE;  0.001 -> nearest of {0, 2^-9}: 2^-9 (0.001 > 2^-10) -> 0x01
    # block 4: max 1.9375 (bf16: 1.1111 b) -> floor(log2) = 0, X = 2^-8; 1.9375 * 256 = 496 -> between 448 and
    #          512: rounds to nearest even 512 which is not finite in E4M3 -> clamped to 448 = 0x7E
    row = [1.0] + [0.5] * 31 + [0.0] * 31 + [-0.0] + [3.0, -448.0] + [0.001] * 30 + [1.9375] + [1.0] * 31
    q, e = orc.mx_quantize(_bf16([row]), orc.E4M3FN)
    assert list(e[0]) == [119, 0, 127, 119]
    assert q[0, 0] == 0x78 and (q[0, 1:32] == 0x70).all()
    assert (q[0, 32:63] == 0).all() and q[0, 63] == 0x80
    assert q[0, 64] == 0x44 and q[0, 65] == 0xFE and (q[0, 66:96] == 0x01).all()
    assert q[0, 96] == 0x7E and (q[0, 97:128] == 0x78).all()


def test_hand_worked_block_e5m2():
    # max 3.0 -> floor(log2) = 1, shared exponent 1 - 15 = -14, byte 113, X = 2^-14
    # 3.0 / X = 1.5 * 2^15 -> S.11110.10 = 0x7A;  1.0 / X = 2^14 -> S.11101.00 = 0x74;  -0.75 / X = -1.5 * 2^13 -> 0xF2
    row = [3.0, 1.0, -0.75] + [0.0] * 29
    q, e = orc.mx_quantize(_bf16([row]), orc.E5M2)
    assert e[0, 0] == 113 and list(q[0, :3]) == [0x7A, 0x74, 0xF2]


def _mx_reference(vals, fmt):
    """Independent conversion in exact rational arithmetic; elements through the
    oracle's nearest-value SEARCH encoder (the definition), not the bit encoder."""
    fr = [Fraction(float(v)) for v in vals]
    amax = max(abs(f) for f in fr)
    if amax == 0:
        byte = 0
    else:
        fl = amax.numerator.bit_length() - amax.denominator.bit_length()
        if Fraction(2) ** fl > amax:
            fl -= 1
        assert Fraction(2) ** fl <= amax < Fraction(2) ** (fl + 1)
        byte = min(max(fl - EMAX[fmt] + 127, 0), 254)
    X = Fraction(2) ** (byte - 127)
    codes = [orc.encode_search(float(f / X), fmt) if f != 0 else (0x80 if math.copysign(1.0, float(v)) < 0 else 0)
             for f, v in zip(fr, vals)]
    return byte, codes


@pytest.mark.parametrize("fmt", FMTS)
def test_against_rational_reference(fmt):
    rng = np.random.default_rng(11 + fmt)
    blocks = []
    for scale in (1.0, 1e-3, 37.0, 2.0 ** -120, 2.0 ** 100, 1e-38, 3e38):
        blocks.append(rng.standard_normal(32) * scale)
    blocks.append(np.r_[np.zeros(31), 2.0 ** -130])                 # subnormal bfloat16 maximum
    blocks.append(np.r_[1.99, rng.uniform(-2, 2, 31)])
    x = _bf16(np.clip(np.array(blocks), -3.3e38, 3.3e38))
    q, e = orc.mx_quantize(x.reshape(1, -1), fmt)
    vals = si.bf16_bits_to_f32(x)
    for b in range(len(blocks)):
        byte, codes = _mx_reference(vals[b], fmt)
        assert e[0, b] == byte, (b, e[0, b], byte)
        assert list(q[0, 32 * b:32 * b + 32]) == codes, b


@pytest.mark.parametrize("fmt", FMTS)
def test_scale_equivariance_and_bounds(fmt):
    """Multiplying a block by 2^k moves only the shared exponent; the largest
    element lands in [2^emax, FMAX]; every element is within half a unit in
    the last place of its code (or saturated)."""
    x = si.normal_bf16((64, 256), 0.37, seed=5, stream=fmt)
    q, e = orc.mx_quantize(x, fmt)
    for k in (-20, 7):
        xs = _bf16(si.bf16_bits_to_f32(x) * np.float32(2.0 ** k))
        qs, es = orc.mx_quantize(xs, fmt)
        assert (qs == q).all() and (es.astype(int) == e.astype(int) + k).all()
    lut = np.array([orc.decode(c, fmt) for c in range(256)], np.float64)
    dec = lut[q].reshape(64, 8, 32)
    X = np.ldexp(1.0, e.astype(int) - 127)[:, :, None]
    v = si.bf16_bits_to_f32(x).astype(np.float64).reshape(64, 8, 32) / X
    top = np.abs(dec).max(axis=2)
    assert (top >= 2.0 ** EMAX[fmt]).all() and (top <= orc.fp8_max(fmt)).all()
    mbits = 3 if fmt == orc.E4M3FN else 2
    emin = -6 if fmt == orc.E4M3FN else -14
    expo = np.maximum(np.floor(np.log2(np.maximum(np.abs(v), 1e-300))), emin)
    half_ulp = np.ldexp(1.0, (expo - mbits - 1).astype(int))
    sat = np.abs(v) > orc.fp8_max(fmt)
    assert (np.abs(v - dec)[~sat] <= half_ulp[~sat] * (1 + 1e-12)).all()
    assert (np.abs(dec)[sat] == orc.fp8_max(fmt)).all()


def test_mx_mm_brute_force_and_exact_integers():
    rng = np.random.default_rng(3)
    M, N, K = 5, 7, 96
    a = rng.integers(0, 0x78, size=(M, K)).astype(np.uint8) | (rng.integers(0, 2, size=(M, K)).astype(np.uint8) << 7)
    b = rng.integers(0, 0x78, size=(N, K)).astype(np.uint8) | (rng.integers(0, 2, size=(N, K)).astype(np.uint8) << 7)
    ea = rng.integers(110, 140, size=(M, K // 32)).astype(np.uint8)
    eb = rng.integers(110, 140, size=(N, K // 32)).astype(np.uint8)
    res = orc.mx_mm(a, orc.E4M3FN, ea, b, orc.E5M2, eb)
    va = np.array([[orc.mx_value(int(a[m, k]), orc.E4M3FN, int(ea[m, k // 32])) for k in range(K)] for m in range(M)])
    vb = np.array([[orc.mx_value(int(b[n, k]), orc.E5M2, int(eb[n, k // 32])) for k in range(K)] for n in range(N)])
    want = va @ vb.T
    assert np.allclose(res.acc64, want, rtol=1e-12, atol=0)
    assert np.allclose(res.out32, want, rtol=1e-5, atol=1e-30)
    assert (res.out16 == orc.f32_to_bf16(res.out32)).all()
    rows = np.array([4, 0], np.int64)
    sub = orc.mx_mm(a, orc.E4M3FN, ea, b, orc.E5M2, eb, rows)
    assert (sub.out32 == res.out32[rows]).all()
    # integers with power-of-two block scales: everything exact
    ai, bi = rng.integers(-3, 4, size=(M, K)), rng.integers(-3, 4, size=(N, K))
    aq = orc.encode_array(ai.astype(np.float32), orc.E4M3FN)
    bq = orc.encode_array(bi.astype(np.float32), orc.E4M3FN)
    ea = rng.integers(120, 131, size=(M, K // 32)).astype(np.uint8)
    eb = rng.integers(120, 131, size=(N, K // 32)).astype(np.uint8)
    exact = sum(np.ldexp(1.0, ea[:, blk].astype(int) - 127)[:, None] * np.ldexp(1.0, eb[:, blk].astype(int) - 127)[None, :]
                * (ai[:, 32 * blk:32 * blk + 32] @ bi[:, 32 * blk:32 * blk + 32].T) for blk in range(K // 32))
    assert (orc.mx_mm(aq, orc.E4M3FN, ea, bq, orc.E4M3FN, eb).out32 == exact.astype(np.float32)).all()


def test_mx_keeps_small_blocks_that_rowwise_scaling_flushes():
    """What block scaling is for: the dynamic range of one row.  A row whose
    first block is ~1e8 times larger than the rest loses the rest entirely
    under one scale per row (everything below half the smallest FP8 subnormal
    becomes zero), while every MX block keeps its own exponent.  The weight
    ignores the large block, so the output depends on the small values only."""
    M, N, K = 16, 24, 256
    xs = si.bf16_bits_to_f32(si.normal_bf16((M, K), 1.0, seed=2, stream=0))
    xs[:, :32] *= 1e4
    xs[:, 32:] *= 1e-4
    x = si.f32_to_bf16_bits(xs)
    ws = si.bf16_bits_to_f32(si.normal_bf16((N, K), 1.0, seed=2, stream=1))
    ws[:, :32] = 0.0
    w = si.f32_to_bf16_bits(ws)
    true = orc.bf16_mm_f64(x, w)
    mx = orc.mx_linear_fwd(x, w)
    row = orc.linear_fwd(x, w, orc.Recipe(gran=orc.ROW))[0]
    e_mx, e_row = orc.rel_frobenius(mx.out32, true), orc.rel_frobenius(row.out32, true)
    assert e_mx < 0.08 and e_row > 0.9, (e_mx, e_row)


def test_mx_linear_bwd_exact_on_integers_and_block_axes():
    """Small integers survive MX quantization unchanged, so both gradients must
    equal the integer products exactly (catches a transposed or swapped operand).
    Scaling every other row of dY (or of W) by 2^-20 then shows which axis the
    blocks run along: a block ALONG such a row keeps it (own exponent), a block
    ACROSS 32 rows loses the small rows (below half the smallest subnormal of
    the shared exponent)."""
    rng = np.random.default_rng(11)
    M, K, N = 64, 96, 32
    dyi, xi, wi = rng.integers(-3, 4, size=(M, N)), rng.integers(-3, 4, size=(M, K)), rng.integers(-3, 4, size=(N, K))
    dyi[0::2][dyi[0::2] == 0] = 3          # every block across rows holds a full-size element
    wi[0::2][wi[0::2] == 0] = 3
    dy, x, w = (_bf16(a.astype(np.float32)) for a in (dyi, xi, wi))
    dx, dw = orc.mx_linear_bwd(dy, x, w)
    assert (dx.out32 == (dyi @ wi).astype(np.float32)).all()
    assert (dw.out32 == (dyi.T @ xi).astype(np.float32)).all()
    assert dx.out32.shape == (M, K) and dw.out32.shape == (N, K)

    small = np.where(np.arange(M) % 2 == 1, 2.0 ** -20, 1.0)[:, None]
    dy_s = _bf16((dyi * small).astype(np.float32))
    dx, dw = orc.mx_linear_bwd(dy_s, x, w)
    assert (dx.out32 == ((dyi * small) @ wi).astype(np.float32)).all()            # blocks along N: rows keep their range
    dy_flushed = np.where(np.arange(M)[:, None] % 2 == 1, 0, dyi)
    assert (dw.out32 == (dy_flushed.T @ xi).astype(np.float32)).all()            # blocks along M: small rows are lost

    small_n = np.where(np.arange(N) % 2 == 1, 2.0 ** -20, 1.0)[:, None]
    w_s = _bf16((wi * small_n).astype(np.float32))
    dx, _ = orc.mx_linear_bwd(dy, x, w_s)
    w_flushed = np.where(np.arange(N)[:, None] % 2 == 1, 0, wi)
    assert (dx.out32 == (dyi @ w_flushed).astype(np.float32)).all()              # W is blocked along N for dX
    assert (orc.mx_linear_fwd(x, w_s).out32 == (xi @ (wi * small_n).T).astype(np.float32)).all()   # and along K forward


def test_mx_linear_bwd_close_to_the_unquantized_gradients():
    M, K, N = 96, 128, 64
    dy = si.normal_bf16((M, N), 1e-3, seed=5, stream=0)
    x = si.normal_bf16((M, K), 1.0, seed=5, stream=1)
    w = si.normal_bf16((N, K), 0.02, seed=5, stream=2)
    dx, dw = orc.mx_linear_bwd(dy, x, w)
    true_dx = orc.bf16_mm_f64(dy, np.ascontiguousarray(w.T))
    true_dw = orc.bf16_mm_f64(np.ascontiguousarray(dy.T), np.ascontiguousarray(x.T))
    assert orc.rel_frobenius(dx.out32, true_dx) < 0.06
    assert orc.rel_frobenius(dw.out32, true_dw) < 0.06
    rows = np.array([5, 63], np.int64)
    sx, sw = orc.mx_linear_bwd(dy, x, w, rows_dx=rows, rows_dw=rows)
    assert (sx.out32 == dx.out32[rows]).all() and (sw.out32 == dw.out32[rows]).all()
