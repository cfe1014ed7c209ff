"""Pins for the oracle's fp8 decode / encode / bfloat16 rounding (no GPU).

Each check is something other than the oracle itself: the format's printed
values (tests/golden), closed forms, an exhaustive round trip, two encoders
written independently of each other, exact rational arithmetic, numpy's
float16 (E5M2 is the high byte of IEEE binary16) and PyTorch's CPU fp8 dtypes.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import fp8_oracle as orc

FMTS = {"e4m3fn": orc.E4M3FN, "e5m2": orc.E5M2}
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                yield line.split()


def _val(expr):
    return float(eval(expr, {"inf": math.inf, "nan": math.nan}))


# ------------------------------------------------------------------ decode

def test_decode_golden_values():
    for fmt, code, expr in _rows("ofp8_format_values.txt"):
        want = _val(expr)
        got = orc.decode(int(code, 16), FMTS[fmt])
        if math.isnan(want):
            assert math.isnan(got), (fmt, code)
        else:
            assert got == want and math.copysign(1, got) == math.copysign(1, want), (fmt, code, got, want)


@pytest.mark.parametrize("fmt,mb,bias,maxc", [(orc.E4M3FN, 3, 7, 0x7E), (orc.E5M2, 2, 15, 0x7B)])
def test_decode_closed_form_and_monotone(fmt, mb, bias, maxc):
    prev = -1.0
    for c in range(maxc + 1):
        e, m = c >> mb, c & ((1 << mb) - 1)
        want = Fraction(m, 1 << mb) * Fraction(2) ** (1 - bias) if e == 0 else \
            (1 + Fraction(m, 1 << mb)) * Fraction(2) ** (e - bias)
        got = orc.decode(c, fmt)
        assert Fraction(got) == want
        assert got > prev
        prev = got
        assert orc.decode(c | 0x80, fmt) == -got
    assert prev == orc.fp8_max(fmt)


def test_e5m2_is_high_byte_of_binary16():
    codes = np.arange(256, dtype=np.uint16)
    half = (codes << np.uint16(8)).view(np.float16).astype(np.float32)
    tab = orc.decode_table(orc.E5M2)
    nan = np.isnan(half)
    assert (np.isnan(tab) == nan).all()
    assert (tab[~nan].view(np.uint32) == half[~nan].view(np.uint32)).all()


def test_decode_matches_torch_cpu_dtypes():
    torch = pytest.importorskip("torch")
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    for fmt, dt in ((orc.E4M3FN, torch.float8_e4m3fn), (orc.E5M2, torch.float8_e5m2)):
        ref = codes.view(dt).to(torch.float32).numpy()
        tab = orc.decode_table(fmt)
        nan = np.isnan(ref)
        assert (np.isnan(tab) == nan).all()
        assert (tab[~nan].view(np.uint32) == ref[~nan].view(np.uint32)).all()


# ------------------------------------------------------------------ encode

def test_encode_golden_pins():
    for fmt, expr, code in _rows("encode_pins.txt"):
        v = _val(expr)
        for enc in (orc.encode_search, orc.encode_bits):
            assert enc(v, FMTS[fmt]) == int(code, 16), (fmt, expr, enc.__name__, hex(enc(v, FMTS[fmt])))


@pytest.mark.parametrize("fmt", [orc.E4M3FN, orc.E5M2])
def test_encode_round_trip_all_codes(fmt):
    for c in range(256):
        v = orc.decode(c, fmt)
        for enc in (orc.encode_search, orc.encode_bits):
            got = enc(v, fmt)
            if math.isnan(v):
                assert math.isnan(orc.decode(got, fmt))
            elif math.isinf(v):  # E5M2 infinities saturate
                assert got == ((c & 0x80) | 0x7B)
            else:
                assert got == c, (hex(c), hex(got))


@pytest.mark.parametrize("fmt", [orc.E4M3FN, orc.E5M2])
def test_encoders_agree_on_all_bf16_and_random_f32(fmt):
    bf = (np.arange(65536, dtype=np.uint32) << np.uint32(16)).view(np.float32)
    a, b = orc.encode_array(bf, fmt, True), orc.encode_array(bf, fmt, False)
    nan = np.isnan(bf)
    assert (a[~nan] == b[~nan]).all()
    assert np.isnan(orc.decode_table(fmt)[b[nan]]).all()
    rng = np.random.default_rng(1)
    # random bit patterns (all exponents) and values concentrated in fp8 range
    u = rng.integers(0, 2 ** 32, size=1 << 21, dtype=np.uint64).astype(np.uint32).view(np.float32)
    g = (rng.standard_normal(1 << 21) * np.exp(rng.uniform(-14, 12, 1 << 21))).astype(np.float32)
    for v in (u[~np.isnan(u)], g):
        assert (orc.encode_array(v, fmt, True) == orc.encode_array(v, fmt, False)).all()


@pytest.mark.parametrize("fmt", [orc.E4M3FN, orc.E5M2])
def test_encode_midpoints_neighbours_and_monotone(fmt):
    maxc = 0x7E if fmt == orc.E4M3FN else 0x7B
    vals = [orc.decode(c, fmt) for c in range(maxc + 1)]
    for c in range(maxc):
        lo, hi = np.float32(vals[c]), np.float32(vals[c + 1])
        mid = np.float32((float(lo) + float(hi)) / 2)          # exact in binary32
        assert Fraction(float(mid)) == (Fraction(float(lo)) + Fraction(float(hi))) / 2
        even = c if c % 2 == 0 else c + 1
        below = np.nextafter(mid, np.float32(0))
        above = np.nextafter(mid, np.float32(np.inf))
        for enc in (orc.encode_search, orc.encode_bits):
            assert enc(mid, fmt) == even
            assert enc(below, fmt) == c
            assert enc(above, fmt) == c + 1
            assert enc(-mid, fmt) == (even | 0x80)
    # monotone non-decreasing over a dense sweep of non-negative binary32 values
    sweep = np.sort(np.abs(np.random.default_rng(2).standard_normal(1 << 18).astype(np.float32))
                    * np.float32(orc.fp8_max(fmt) / 2))
    codes = orc.encode_array(sweep, fmt, False)
    assert (np.diff(codes.astype(np.int32)) >= 0).all()


@pytest.mark.parametrize("fmt", [orc.E4M3FN, orc.E5M2])
def test_encode_is_nearest_value_by_exact_arithmetic(fmt):
    """Definition check in rational arithmetic on random inputs: no finite code
    is strictly nearer than the chosen one, and ties chose the even code."""
    maxc = 0x7E if fmt == orc.E4M3FN else 0x7B
    grid = [Fraction(orc.decode(c, fmt)) for c in range(maxc + 1)]
    rng = np.random.default_rng(3)
    xs = (rng.standard_normal(400) * np.exp(rng.uniform(-12, 7 if fmt == orc.E4M3FN else 11, 400))).astype(np.float32)
    for x in xs:
        a = min(abs(Fraction(float(x))), grid[-1])
        code = orc.encode_bits(float(x), fmt)
        assert (code >> 7) == (1 if math.copysign(1, x) < 0 else 0)
        c = code & 0x7F
        d = abs(grid[c] - a)
        best = min(abs(g - a) for g in grid)
        assert d == best
        ties = [i for i, g in enumerate(grid) if abs(g - a) == best]
        if len(ties) > 1:
            assert c % 2 == 0


def test_encode_matches_torch_cpu_cast_on_clamped_inputs():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(4)
    for fmt, dt in ((orc.E4M3FN, torch.float8_e4m3fn), (orc.E5M2, torch.float8_e5m2)):
        fmax = orc.fp8_max(fmt)
        v = (rng.standard_normal(1 << 20) * np.exp(rng.uniform(-14, 11, 1 << 20))).astype(np.float32)
        v = np.clip(v, -fmax, fmax)
        ref = torch.from_numpy(v).to(dt).view(torch.uint8).numpy()
        got = orc.encode_array(v, fmt, False)
        assert (ref == got).all()


# -------------------------------------------------------------- bf16 round

def test_bf16_rounding_matches_closed_form_and_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(5)
    v = (rng.standard_normal(1 << 18) * np.exp(rng.uniform(-20, 20, 1 << 18))).astype(np.float32)
    # ties: values exactly between two bfloat16 neighbours
    base = (rng.integers(0x0080, 0x7F00, size=4096, dtype=np.uint32) << np.uint32(16)) | np.uint32(0x8000)
    v = np.concatenate([v, base.view(np.float32), -base.view(np.float32)])
    got = orc.f32_to_bf16(v)
    ref = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (got == ref).all()
    # widening is the inverse on representable values
    allb = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    wide = orc.bf16_to_f32(allb)
    ok = ~np.isnan(wide)
    assert (orc.f32_to_bf16(wide[ok]) == allb[ok]).all()
