"""Pins for the oracle's amax / scale / cast / scaled matmul / linear fwd+bwd
(no GPU).  Brute force in numpy binary64, exact rational arithmetic, closed
forms and invariants - chosen so that a dropped term, a wrong axis, a
transposed operand or a wrong sign fails at least one of them."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import synthetic_inputs as si
from oracle import fp8_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _f32_rne(q: Fraction) -> np.float32:
    """Correctly rounded binary32 of a positive rational (normal range)."""
    e = math.floor(math.log2(q))
    while Fraction(2) ** e > q:
        e -= 1
    while Fraction(2) ** (e + 1) <= q:
        e += 1
    m = q / Fraction(2) ** (e - 23)          # in [2^23, 2^24)
    fl = m.numerator // m.denominator
    rem = m - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return np.float32(float(Fraction(fl) * Fraction(2) ** (e - 23)))


# -------------------------------------------------------------------- amax

@pytest.mark.parametrize("shape", [(1, 1), (7, 13), (64, 96), (33, 257)])
def test_amax_brute_force_and_magnitude_bits(shape):
    x = si.normal_bf16(shape, 3.0, seed=11, stream=0)
    xf = si.bf16_bits_to_f32(x).astype(np.float64)
    assert orc.amax(x, orc.TENSOR)[0] == np.abs(xf).max()
    assert (orc.amax(x, orc.ROW) == np.abs(xf).max(axis=1)).all()
    assert (orc.amax(x, orc.COL) == np.abs(xf).max(axis=0)).all()
    # |bf16| ordering equals ordering of the 15 magnitude bits
    mag = (x & 0x7FFF)
    assert (orc.amax(x, orc.ROW).view(np.uint32) >> 16 == mag.max(axis=1)).all()
    # permutation invariance
    p = np.random.default_rng(0).permutation(x.size)
    assert orc.amax(x.ravel()[p].reshape(shape), orc.TENSOR)[0] == orc.amax(x, orc.TENSOR)[0]


def test_amax_respects_leading_dimension_and_sign():
    x = si.normal_bf16((8, 32), 1.0, seed=12, stream=0)
    x[3, 20] = 0xC2C8  # -100.0: the maximum is a negative entry outside the view
    view = x[:, :16]
    xf = si.bf16_bits_to_f32(view)
    assert (orc.amax(view, orc.ROW) == np.abs(xf).max(axis=1)).all()
    x[5, 7] = 0xC2C8
    assert orc.amax(x[:, :16], orc.TENSOR)[0] == 100.0
    assert orc.amax(x[:, :16], orc.COL)[7] == 100.0


# ------------------------------------------------------------------- scale

def test_scale_pinned_values():
    pins = {  # (format, amax) -> binary32 bits, worked by hand: FMAX / amax correctly rounded
        (orc.E4M3FN, 1.0): 0x43E00000, (orc.E4M3FN, 3.0): 0x43155555, (orc.E4M3FN, 5.25): 0x42AAAAAB,
        (orc.E4M3FN, 448.0): 0x3F800000, (orc.E4M3FN, 57344.0): 0x3C000000,
        (orc.E5M2, 1.0): 0x47600000, (orc.E5M2, 448.0): 0x43000000, (orc.E5M2, 57344.0): 0x3F800000,
    }
    for (fmt, a), bits in pins.items():
        got = orc.scale(np.array([a], np.float32), fmt)
        assert int(got.view(np.uint32)[0]) == bits, (fmt, a, hex(int(got.view(np.uint32)[0])))


@pytest.mark.parametrize("fmt", [orc.E4M3FN, orc.E5M2])
def test_scale_is_correctly_rounded_quotient(fmt):
    rng = np.random.default_rng(21)
    bits = rng.integers(0x0080, 0x7F00, size=3000, dtype=np.uint32).astype(np.uint16)
    a = si.bf16_bits_to_f32(bits)
    a = a[a > 1e-11]
    got = orc.scale(a, fmt)
    fmax = Fraction(orc.fp8_max(fmt))
    for ai, si_ in zip(a[:600], got[:600]):
        q = fmax / Fraction(float(ai))
        if Fraction(2) ** -126 <= q < Fraction(2) ** 127:
            assert si_ == _f32_rne(q), (ai, si_)
    # invariant: amax * s stays within one binary32 ulp of FMAX
    prod = a.astype(np.float64) * got.astype(np.float64)
    ok = np.isfinite(got) & (got.view(np.uint32) >= 0x00800000)
    assert (prod[ok] <= orc.fp8_max(fmt) * (1 + 2.0 ** -23)).all()
    assert (prod[ok] >= orc.fp8_max(fmt) * (1 - 2.0 ** -23)).all()


@pytest.mark.parametrize("fmt,zero_bits", [(orc.E4M3FN, 0x57CBBA10), (orc.E5M2, 0x5B4BBA10)])
def test_scale_zero_and_tiny_amax_clamp(fmt, zero_bits):
    # FMAX / 1e-12, correctly rounded, by exact arithmetic on the binary64 constant
    want = _f32_rne(Fraction(orc.fp8_max(fmt)) / Fraction(1e-12))
    assert int(want.view(np.uint32)) == zero_bits
    got = orc.scale(np.array([0.0, 1e-20, 1e-12], np.float32), fmt)
    assert (got.view(np.uint32)[:2] == zero_bits).all()
    assert np.isfinite(got).all()


@pytest.mark.parametrize("fmt", [orc.E4M3FN, orc.E5M2])
def test_scale_pow2_rounds_down(fmt):
    a = np.array([3.0, 5.25, 0.09, 1.0, 448.0, 0.75, 1e-3], np.float32)
    s = orc.scale(a, fmt)
    p = orc.scale(a, fmt, orc.POW2_SCALE)
    assert ((p.view(np.uint32) & 0x007FFFFF) == 0).all()           # pure powers of two
    assert (p <= s).all() and (2 * p > s).all()                    # floor, not nearest
    prod = a.astype(np.float64) * p.astype(np.float64)
    fmax = orc.fp8_max(fmt)
    assert ((prod > fmax / 2) & (prod <= fmax)).all()
    if fmt == orc.E4M3FN:
        assert p[0] == 128.0 and p[1] == 64.0 and p[2] == 4096.0   # 149.3 -> 128, 85.3 -> 64, 4977.8 -> 4096


# -------------------------------------------------------------------- cast

@pytest.mark.parametrize("fmt", [orc.E4M3FN, orc.E5M2])
@pytest.mark.parametrize("gran", [orc.TENSOR, orc.ROW, orc.COL])
def test_cast_definition_two_roundings(fmt, gran):
    """q = encode(fp32(x*s)): product rounded to binary32 first (checked with
    numpy float32 multiply), narrowed by the search encoder."""
    x = si.normal_bf16((37, 53), 2.0, seed=31, stream=0)
    s = orc.scale(orc.amax(x, gran), fmt)
    xf = si.bf16_bits_to_f32(x)
    sb = s[0] if gran == orc.TENSOR else (s[:, None] if gran == orc.ROW else s[None, :])
    prod = (xf * sb).astype(np.float32)
    want = orc.encode_array(prod, fmt, use_search=True)
    assert (orc.cast(x, s, gran, fmt) == want).all()
    assert (orc.cast(x, s, gran, fmt, use_search=True) == want).all()
    assert (orc.cast(x, s, gran, fmt, orc.TRANSPOSE_OUT) == want.T).all()


@pytest.mark.parametrize("fmt,sig_bits", [(orc.E4M3FN, 4), (orc.E5M2, 3)])
def test_cast_pow2_scale_is_exact_for_short_significands(fmt, sig_bits):
    rng = np.random.default_rng(32)
    mant = rng.integers(1 << (sig_bits - 1), 1 << sig_bits, size=(16, 64))
    expo = rng.integers(-3, 2, size=(16, 64))   # keeps |x| * 2^k inside the normal range
    sign = rng.choice([-1.0, 1.0], size=(16, 64))
    xf = (sign * mant * 2.0 ** expo).astype(np.float32)
    x = si.f32_to_bf16_bits(xf)
    assert (si.bf16_bits_to_f32(x) == xf).all()
    for k in (-2, 0, 3):
        s = np.array([2.0 ** k], np.float32)
        q = orc.cast(x, s, orc.TENSOR, fmt)
        back = orc.decode_table(fmt)[q] / s[0]
        assert (back == xf).all()


@pytest.mark.parametrize("fmt", [orc.E4M3FN, orc.E5M2])
def test_cast_dynamic_scaling_invariants(fmt):
    x = si.normal_bf16((48, 200), 0.3, seed=33, stream=0)
    xf = si.bf16_bits_to_f32(x)
    am = orc.amax(x, orc.ROW)
    s = orc.scale(am, fmt)
    q = orc.cast(x, s, orc.ROW, fmt)
    mag = q & 0x7F
    maxc = 0x7E if fmt == orc.E4M3FN else 0x7B
    assert (mag <= maxc).all()                       # never NaN / Inf
    # the amax element of every row takes the row's largest code, and that is the top code
    # or the one below it (amax*s is within an ulp of FMAX)
    for r in range(x.shape[0]):
        j = np.abs(xf[r]).argmax()
        assert mag[r, j] == mag[r].max() and mag[r, j] >= maxc - 1
    # sign preserved, including values flushed to zero
    assert ((q >> 7) == (x >> 15)).all()
    # relative error bound for results in the normal range: half an fp8 ulp
    dec = orc.decode_table(fmt)[q].astype(np.float64) / s[:, None].astype(np.float64)
    normal = (mag >> (3 if fmt == orc.E4M3FN else 2)) > 0
    rel = np.abs(dec - xf)[normal] / np.abs(xf[normal])
    assert rel.max() <= (2.0 ** -4 if fmt == orc.E4M3FN else 2.0 ** -3) * (1 + 1e-6)
    st = orc.cast_stats(x, s, orc.ROW, fmt)
    # only an amax element can be counted as saturated under dynamic scaling
    assert st.n_sat <= x.shape[0]
    assert st.n_zero == int(((mag == 0) & (xf != 0)).sum())
    sq = 10 * np.log10((xf.astype(np.float64) ** 2).sum() / ((dec - xf) ** 2).sum())
    assert abs(st.sqnr_db - sq) < 1e-6


def test_cast_all_zero_group_gives_signed_zero_codes():
    x = np.zeros((4, 16), np.uint16)
    x[1, 3] = 0x8000  # -0.0
    q, s = orc.quantize(x, orc.ROW, orc.E4M3FN)
    assert (s.view(np.uint32) == 0x57CBBA10).all()
    assert q[1, 3] == 0x80 and (np.delete(q.ravel(), 1 * 16 + 3) == 0).all()


def test_cast_static_scale_saturates_and_counts():
    xf = np.array([[1.0, -2.0, 500.0, -1e6, 3e-4, 0.0]], np.float32)
    x = si.f32_to_bf16_bits(xf)
    s = np.array([1.0], np.float32)
    q = orc.cast(x, s, orc.TENSOR, orc.E4M3FN)
    assert list(q[0]) == [0x38, 0xC0, 0x7E, 0xFE, 0x00, 0x00]
    st = orc.cast_stats(x, s, orc.TENSOR, orc.E4M3FN)
    assert (st.n_sat, st.n_zero) == (2, 1)


def test_cast_stats_counts_subnormal_codes_hand_worked():
    """n_subnormal = nonzero codes whose exponent field is 0, counted on rows worked by hand with scale 1.
    e4m3: subnormals are m * 2^-9, m = 1..7, the smallest normal is 2^-6.  e5m2: m * 2^-16, m = 1..3, smallest
    normal 2^-14.  Ties go to the even code; half the smallest subnormal goes to zero (counted in n_zero, not here)."""
    one = np.array([1.0], np.float32)
    xf = np.array([[1.0, 2.0 ** -7, 3 * 2.0 ** -9, 2.0 ** -6, 2.0 ** -10, -(2.0 ** -9), 0.0, 7.5 * 2.0 ** -9,
                    1.5 * 2.0 ** -9]], np.float32)
    x = si.f32_to_bf16_bits(xf)
    assert (si.bf16_bits_to_f32(x) == xf).all()           # every value is a bfloat16 number
    q = orc.cast(x, one, orc.TENSOR, orc.E4M3FN)
    assert list(q[0]) == [0x38, 0x04, 0x03, 0x08, 0x00, 0x81, 0x00, 0x08, 0x02]
    st = orc.cast_stats(x, one, orc.TENSOR, orc.E4M3FN)
    assert (st.n_sat, st.n_zero, st.n_subnormal) == (0, 1, 4)
    xf = np.array([[2.0 ** -15, 2.0 ** -14, 3 * 2.0 ** -16, 2.0 ** -17, 1.0, -(2.0 ** -16)]], np.float32)
    x = si.f32_to_bf16_bits(xf)
    q = orc.cast(x, one, orc.TENSOR, orc.E5M2)
    assert list(q[0]) == [0x02, 0x04, 0x03, 0x00, 0x3C, 0x81]
    st = orc.cast_stats(x, one, orc.TENSOR, orc.E5M2)
    assert (st.n_sat, st.n_zero, st.n_subnormal) == (0, 1, 3)
    # a scale moves values across the boundary: x * 2^-3 turns 2^-6 .. 2^-4 into subnormals
    xf = np.array([[2.0 ** -6, 2.0 ** -5, 2.0 ** -4, 2.0 ** -3]], np.float32)
    st = orc.cast_stats(si.f32_to_bf16_bits(xf), np.array([0.125], np.float32), orc.TENSOR, orc.E4M3FN)
    assert st.n_subnormal == 3 and st.n_zero == 0


# --------------------------------------------------------------- scaled mm

def _rand_codes(shape, fmt, rng):
    maxc = 0x7E if fmt == orc.E4M3FN else 0x7B
    c = rng.integers(0, maxc + 1, size=shape, dtype=np.int64).astype(np.uint8)
    return c | (rng.integers(0, 2, size=shape).astype(np.uint8) << 7)


@pytest.mark.parametrize("M,N,K", [(3, 5, 7), (16, 16, 128), (33, 17, 256)])
@pytest.mark.parametrize("fa,fb", [(orc.E4M3FN, orc.E4M3FN), (orc.E5M2, orc.E4M3FN)])
@pytest.mark.parametrize("ga,gb", [(orc.TENSOR, orc.TENSOR), (orc.ROW, orc.ROW), (orc.ROW, orc.TENSOR)])
def test_scaled_mm_brute_force(M, N, K, fa, fb, ga, gb):
    rng = np.random.default_rng(41)
    # moderate magnitudes so that binary32 accumulation stays well conditioned
    a = _rand_codes((M, K), fa, rng) & np.uint8(0xBF if fa == orc.E4M3FN else 0xBF)
    b = _rand_codes((N, K), fb, rng) & np.uint8(0xBF)
    sa = rng.uniform(0.5, 300, 1 if ga == orc.TENSOR else M).astype(np.float32)
    sb = rng.uniform(0.5, 300, 1 if gb == orc.TENSOR else N).astype(np.float32)
    res = orc.scaled_mm(a, fa, sa, ga, b, fb, sb, gb)
    A = orc.decode_table(fa)[a].astype(np.float64)
    B = orc.decode_table(fb)[b].astype(np.float64)
    want = np.zeros((M, N))
    for m in range(M):
        for n in range(N):
            acc = 0.0
            for k in range(K):
                acc += A[m, k] * B[n, k]
            want[m, n] = acc / float(sa[0 if ga == orc.TENSOR else m]) / float(sb[0 if gb == orc.TENSOR else n])
    assert np.allclose(res.acc64, want, rtol=1e-13, atol=0)
    scale_ = np.abs(A) @ np.abs(B).T / np.outer(np.broadcast_to(sa, M), np.broadcast_to(sb, N))
    assert (np.abs(res.out32 - want) <= scale_ * (K + 4) * 2.0 ** -24).all()
    assert (res.out16 == orc.f32_to_bf16(res.out32)).all()
    # a transposed-operand mistake would break this asymmetric identity
    res_t = orc.scaled_mm(b, fb, sb, gb, a, fa, sa, ga)
    assert np.allclose(res_t.acc64, want.T, rtol=1e-13, atol=0)


def test_scaled_mm_exact_integer_case_and_row_sampling():
    rng = np.random.default_rng(42)
    M, N, K = 40, 24, 512
    ai = rng.integers(-2, 3, size=(M, K))
    bi = rng.integers(-2, 3, size=(N, K))
    a = orc.encode_array((ai * 0.5).astype(np.float32), orc.E5M2)
    b = orc.encode_array((bi * 4.0).astype(np.float32), orc.E4M3FN)
    sa = np.array([0.25], np.float32)
    sb = (2.0 ** rng.integers(-3, 4, size=N)).astype(np.float32)
    res = orc.scaled_mm(a, orc.E5M2, sa, orc.TENSOR, b, orc.E4M3FN, sb, orc.ROW)
    want = (ai @ bi.T) * 2.0 / 0.25 / sb[None, :]
    assert (res.out32 == want.astype(np.float32)).all() and (res.acc64 == want).all()
    rows = np.array([0, 7, 39, 12], np.int64)
    sub = orc.scaled_mm(a, orc.E5M2, sa, orc.TENSOR, b, orc.E4M3FN, sb, orc.ROW, rows)
    assert (sub.out32 == res.out32[rows]).all() and (sub.out16 == res.out16[rows]).all()


def test_bf16_mm_f64_brute_force():
    a = si.normal_bf16((5, 33), 1.0, 43, 0)
    b = si.normal_bf16((7, 33), 1.0, 43, 1)
    want = si.bf16_bits_to_f32(a).astype(np.float64) @ si.bf16_bits_to_f32(b).astype(np.float64).T
    assert np.allclose(orc.bf16_mm_f64(a, b), want, rtol=1e-13)


# ---------------------------------------------------------- linear fwd/bwd

def _dense(x):
    return si.bf16_bits_to_f32(x).astype(np.float64)


@pytest.mark.parametrize("gran", [orc.TENSOR, orc.ROW])
@pytest.mark.parametrize("pow2", [False, True])
def test_linear_axes_and_quantization_error_band(gran, pow2):
    M, K, N = 48, 160, 40
    x = si.normal_bf16((M, K), 1.0, 51, 0)
    w = si.normal_bf16((N, K), 0.02, 51, 1)
    dy = si.normal_bf16((M, N), 1e-3, 51, 2)
    r = orc.Recipe(gran=gran, pow2=pow2)
    y, xo, wo = orc.linear_fwd(x, w, r)
    dx, go, wto = orc.linear_bwd_dx(dy, w, r)
    dw, gto, xto = orc.linear_bwd_dw(dy, x, r)
    # shapes say which axis was contracted and which carried the scales
    assert y.out32.shape == (M, N) and dx.out32.shape == (M, K) and dw.out32.shape == (N, K)
    assert wto.q.shape == (K, N) and gto.q.shape == (N, M) and xto.q.shape == (K, M)
    n_s = (lambda n: 1) if gran == orc.TENSOR else (lambda n: n)
    assert [o.s.size for o in (xo, wo, go, wto, gto, xto)] == [n_s(v) for v in (M, N, M, K, N, K)]
    if gran == orc.ROW:
        # every scale comes from the amax over the contraction axis of its GEMM
        flags = orc.POW2_SCALE if pow2 else 0
        assert (xo.s == orc.scale(np.abs(_dense(x)).max(1).astype(np.float32), orc.E4M3FN, flags)).all()
        assert (wto.s == orc.scale(np.abs(_dense(w)).max(0).astype(np.float32), orc.E4M3FN, flags)).all()
        assert (gto.s == orc.scale(np.abs(_dense(dy)).max(0).astype(np.float32), orc.E5M2, flags)).all()
        assert (xto.s == orc.scale(np.abs(_dense(x)).max(0).astype(np.float32), orc.E4M3FN, flags)).all()
    else:
        assert wto.s[0] == wo.s[0] and gto.s[0] == go.s[0] and xto.s[0] == xo.s[0]
        assert (wto.q == wo.q.T).all() and (xto.q == xo.q.T).all() and (gto.q == go.q.T).all()
    # against the unquantized products: right operands, right transposes, errors
    # in the band fp8 quantization gives (e4m3: ~2-4 %, e5m2: ~5-8 % per operand)
    for got, ref, hi in ((y, _dense(x) @ _dense(w).T, 0.08), (dx, _dense(dy) @ _dense(w), 0.12),
                         (dw, _dense(dy).T @ _dense(x), 0.12)):
        err = orc.rel_frobenius(got.acc64, ref)
        assert 1e-3 < err < hi, err
        assert orc.rel_frobenius(got.out32, got.acc64) < 1e-5


def test_linear_exact_on_integer_inputs_with_pow2_scales():
    rng = np.random.default_rng(52)
    M, K, N = 32, 64, 16
    xi, wi, gi = (rng.integers(-3, 4, size=s) for s in ((M, K), (N, K), (M, N)))
    # make every row and column amax a power of two times FMAX's leading bits: pin amax = 4
    xi[:, 0] = 4; xi[0, :] = 4; wi[:, 0] = 4; wi[0, :] = 4; gi[:, 0] = 4; gi[0, :] = 4
    x, w, dy = (si.f32_to_bf16_bits(v.astype(np.float32)) for v in (xi, wi, gi))
    for gran in (orc.TENSOR, orc.ROW):
        r = orc.Recipe(gran=gran, pow2=True)
        assert (orc.linear_fwd(x, w, r)[0].out32 == (xi @ wi.T)).all()
        assert (orc.linear_bwd_dx(dy, w, r)[0].out32 == (gi @ wi)).all()
        assert (orc.linear_bwd_dw(dy, x, r)[0].out32 == (gi.T @ xi)).all()


def test_outliers_hurt_tensorwise_more_than_rowwise():
    """Appendix A of the paper: one outlier sets the scale of a whole tensor under
    tensorwise scaling, so more values underflow to zero; rowwise scaling is
    less sensitive.  Checked on Student-t activations with hot columns."""
    x = si.student_t_outlier_bf16((256, 1024), 3.0, 0.004, 100.0, seed=0, stream=0)
    st_t = orc.cast_stats(x, orc.scale(orc.amax(x, orc.TENSOR), orc.E4M3FN), orc.TENSOR, orc.E4M3FN)
    st_r = orc.cast_stats(x, orc.scale(orc.amax(x, orc.ROW), orc.E4M3FN), orc.ROW, orc.E4M3FN)
    assert st_t.n_zero > 5 * max(1, st_r.n_zero)
    assert st_r.sqnr_db > st_t.sqnr_db


# ------------------------------------- weight gradient in high precision (rowwise_gw_hp)

def test_grad_weight_hp_is_the_plain_transposed_product():
    """Pins of the definition dW[n,k] = sum_m dY[m,n] X[m,k] (Appendix A,
    rowwise_gw_hp): numpy binary64 on the unquantized values (a transposed or
    swapped operand fails it: the shapes are all different), exact small
    integers bit for bit, and the row selection."""
    M, K, N = 37, 24, 40
    dy = si.normal_bf16((M, N), 1e-3, 51, 0)
    x = si.normal_bf16((M, K), 1.0, 51, 1)
    want = si.bf16_bits_to_f32(dy).astype(np.float64).T @ si.bf16_bits_to_f32(x).astype(np.float64)
    out32, out16 = orc.linear_bwd_dw_hp(dy, x)
    assert out32.shape == (N, K) and np.allclose(out32, want, rtol=1e-6, atol=0)
    assert (out16 == orc.f32_to_bf16(want.astype(np.float32))).all()
    rows = np.array([3, 39, 0], np.int64)
    s32, s16 = orc.linear_bwd_dw_hp(dy, x, rows)
    assert (s32 == out32[rows]).all() and (s16 == out16[rows]).all()
    rng = np.random.default_rng(2)
    gi, xi = rng.integers(-4, 5, size=(M, N)), rng.integers(-4, 5, size=(M, K))
    e32, e16 = orc.linear_bwd_dw_hp(si.f32_to_bf16_bits(gi.astype(np.float32)), si.f32_to_bf16_bits(xi.astype(np.float32)))
    assert (e32 == (gi.T @ xi).astype(np.float32)).all()
    assert (si.bf16_bits_to_f32(e16) == si.bf16_bits_to_f32(orc.f32_to_bf16((gi.T @ xi).astype(np.float32)))).all()


def test_grad_weight_hp_is_closer_to_the_true_gradient_than_the_fp8_one():
    """What the recipe is for (Appendix A): on the same inputs the bfloat16
    weight gradient has a far smaller error against the binary64 product than
    the rowwise FP8 one."""
    M, K, N = 256, 64, 48
    dy = si.normal_bf16((M, N), 1e-3, 52, 0)
    x = si.normal_bf16((M, K), 1.0, 52, 1)
    true = si.bf16_bits_to_f32(dy).astype(np.float64).T @ si.bf16_bits_to_f32(x).astype(np.float64)
    hp32, _ = orc.linear_bwd_dw_hp(dy, x)
    lp = orc.linear_bwd_dw(dy, x, orc.Recipe(gran=orc.ROW))[0]
    e_hp, e_lp = orc.rel_frobenius(hp32, true), orc.rel_frobenius(lp.out32, true)
    assert e_hp < 1e-6 and 5e-3 < e_lp < 0.2, (e_hp, e_lp)
