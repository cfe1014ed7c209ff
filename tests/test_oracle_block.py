"""Pins of the oracle's blockwise FP8 quantization (blocks of 1 x 128 for
activations, 128 x 128 for weights, power-of-two scales stored as E8M0 bytes;
the recipe the paper's list of prototype features attributes to DeepSeek):
hand-worked blocks, the invariants that the scale rule fixes (the block maximum
lands in (FMAX/2, FMAX], nothing saturates), exact rational arithmetic through
the search encoder, the special cases that reduce to the rowwise / tensorwise
power-of-two quantization, locality and replication of the scale bytes, and a
brute-force product."""
from fractions import Fraction

import numpy as np
import pytest

import synthetic_inputs as si
from oracle import fp8_oracle as orc

FMTS = [orc.E4M3FN, orc.E5M2]
FMAX = {orc.E4M3FN: 448.0, orc.E5M2: 57344.0}


def _bf16(vals):
    return si.f32_to_bf16_bits(np.asarray(vals, np.float32))


def test_hand_worked_blocks():
    # one row, four tiles of 1 x 128
    # tile 0: max 448 -> s = 448/448 = 1 -> byte 127; 448 -> 0x7E, 3 -> 0x44
    # tile 1: max 1.0 -> 448/1 = 448 -> rounded down to 256 = 2^8 -> byte 127 - 8 = 119; 1.0 * 256 = 2^8 -> 0x78
    # tile 2: max 450 (bf16: 1.1100001 b * 2^8) -> 448/450 < 1 -> s = 1/2 -> byte 128; 450/2 = 225 -> nearest of
    #         {224, 240} -> 224 = 1.75 * 2^7 -> 0x76
    # tile 3: all zero -> amax clamps to 1e-12 -> s = fp32(448e12) rounded down = 2^48 -> byte 79; codes +-0
    row = [448.0, 3.0] + [0.0] * 126 + [1.0] * 128 + [450.0] + [-1.0] * 127 + [0.0] * 127 + [-0.0]
    q, e = orc.block_quantize(_bf16([row]), 1, 128, orc.E4M3FN)
    assert list(e[0]) == [127] * 4 + [119] * 4 + [128] * 4 + [79] * 4
    assert q[0, 0] == 0x7E and q[0, 1] == 0x44 and (q[0, 2:128] == 0).all()
    assert (q[0, 128:256] == 0x78).all()
    assert q[0, 256] == 0x76 and (q[0, 257:384] == 0xB0).all()          # -1 * 0.5 = -0.5 = -(1.0 * 2^-1) -> S.0110.000
    assert (q[0, 384:511] == 0).all() and q[0, 511] == 0x80
    # e5m2: max 57344 -> byte 127; max 1 -> 57344 -> 2^15 -> byte 112
    q5, e5 = orc.block_quantize(_bf16([[57344.0] + [1.0] * 127 + [1.0] * 128]), 1, 128, orc.E5M2)
    assert list(e5[0]) == [127] * 4 + [112] * 4 and q5[0, 0] == 0x7B and q5[0, 128] == 0x78   # 2^15 = S.11110.00


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("br,bc", [(1, 128), (128, 128)])
def test_block_maximum_lands_in_the_top_binade_and_nothing_saturates(fmt, br, bc):
    rng = np.random.default_rng(5)
    x = _bf16(rng.standard_normal((300, 512)) * np.exp(rng.uniform(-20, 20, (300, 1))))
    q, e = orc.block_quantize(x, br, bc, fmt)
    xf = si.bf16_bits_to_f32(x).astype(np.float64)
    fmax = FMAX[fmt]
    for rb in range(0, 300, br):
        for cb in range(0, 512, bc):
            blk = xf[rb:rb + br, cb:cb + bc]
            by = e[rb:rb + br, cb // 32:(cb + bc) // 32]
            assert (by == by.flat[0]).all()                                    # one byte per block, replicated
            s = 2.0 ** (127 - int(by.flat[0]))
            top = np.abs(blk).max() * s
            assert fmax / 2 < top <= fmax, (rb, cb, top)
    dec = orc.decode_table(fmt).astype(np.float64)
    deq = dec[q] * 2.0 ** (e.astype(np.float64).repeat(32, axis=1) - 127)
    assert np.isfinite(deq).all()
    # relative error of a value in the normal range of the format: half a unit in the last place
    ulp = 2.0 ** -(3 if fmt == orc.E4M3FN else 2)
    scaled = np.abs(xf) * 2.0 ** (127 - e.astype(np.float64).repeat(32, axis=1))
    normal = scaled >= (2.0 ** -6 if fmt == orc.E4M3FN else 2.0 ** -14)
    assert (np.abs(deq - xf)[normal] <= ulp / 2 * np.abs(xf)[normal] * (1 + 1e-12)).all()


@pytest.mark.parametrize("fmt", FMTS)
def test_codes_equal_exact_rational_rounding(fmt):
    """q = RNE(x * 2^(127 - byte)) recomputed with exact fractions and the search encoder."""
    rng = np.random.default_rng(6)
    x = _bf16(rng.standard_normal((3, 256)) * 37.0)
    q, e = orc.block_quantize(x, 1, 128, fmt)
    xf = si.bf16_bits_to_f32(x)
    for r in range(3):
        for c in range(256):
            exact = Fraction(float(xf[r, c])) * Fraction(2) ** (127 - int(e[r, c // 32]))
            assert q[r, c] == orc.encode_search(float(exact), fmt), (r, c)     # exact: a power-of-two multiple


@pytest.mark.parametrize("fmt", FMTS)
def test_reduces_to_rowwise_and_tensorwise_power_of_two_quantization(fmt):
    rng = np.random.default_rng(7)
    x = _bf16(rng.standard_normal((128, 128)) * 0.3)
    # one tile per row == the rowwise recipe with power-of-two scales
    q, e = orc.block_quantize(x, 1, 128, fmt)
    wq, ws = orc.quantize(x, orc.ROW, fmt, orc.POW2_SCALE)
    assert (q == wq).all()
    assert (2.0 ** (e[:, 0].astype(np.float64) - 127) == 1.0 / ws.astype(np.float64)).all()
    # one block for the matrix == the tensorwise recipe with a power-of-two scale
    q, e = orc.block_quantize(x, 128, 128, fmt)
    wq, ws = orc.quantize(x, orc.TENSOR, fmt, orc.POW2_SCALE)
    assert (q == wq).all() and (e == e[0, 0]).all()
    assert 2.0 ** (float(e[0, 0]) - 127) == 1.0 / float(np.asarray(ws).reshape(-1)[0])


def test_blocks_are_independent_and_partial_bottom_blocks_work():
    rng = np.random.default_rng(8)
    x = _bf16(rng.standard_normal((200, 256)))            # second row of blocks has 72 rows
    q0, e0 = orc.block_quantize(x, 128, 128, orc.E4M3FN)
    y = x.copy()
    y[150, 200] = _bf16([1000.0])[0]                       # inside block (1, 1) only
    q1, e1 = orc.block_quantize(y, 128, 128, orc.E4M3FN)
    same = np.ones((200, 256), bool)
    same[128:, 128:] = False
    assert (q0[same] == q1[same]).all() and (e0[:128] == e1[:128]).all() and (e0[128:, :4] == e1[128:, :4]).all()
    assert (e1[128:, 4:] != e0[128:, 4:]).all()
    # the partial block equals the full-block quantization of the same rows padded with zeros
    pad = np.zeros((256, 256), np.uint16)
    pad[:200] = x
    qp, ep = orc.block_quantize(pad, 128, 128, orc.E4M3FN)
    assert (qp[:200] == q0).all() and (ep[:200] == e0).all()


def test_blockwise_linear_equals_the_brute_force_sum_of_dequantized_products():
    rng = np.random.default_rng(9)
    M, K, N = 5, 256, 130
    x = _bf16(rng.standard_normal((M, K)))
    w = _bf16(rng.standard_normal((N, K)) * 0.02)
    res = orc.block_linear_fwd(x, w)
    xq, xe = orc.block_quantize(x, 1, 128, orc.E4M3FN)
    wq, we = orc.block_quantize(w, 128, 128, orc.E4M3FN)
    dec = orc.decode_table(orc.E4M3FN).astype(np.float64)
    xd = dec[xq] * 2.0 ** (xe.astype(np.float64).repeat(32, axis=1) - 127)
    wd = dec[wq] * 2.0 ** (we.astype(np.float64).repeat(32, axis=1) - 127)
    want = xd @ wd.T
    assert np.allclose(res.acc64, want, rtol=1e-12, atol=0)
    assert np.allclose(res.out32, want, rtol=K * 2.0 ** -23, atol=1e-30)
    # and it approximates the unquantized product to the accuracy of two e4m3 operands
    ref = si.bf16_bits_to_f32(x).astype(np.float64) @ si.bf16_bits_to_f32(w).astype(np.float64).T
    assert np.linalg.norm(want - ref) <= 0.06 * np.linalg.norm(ref)


def test_blockwise_backward_equals_brute_force_and_square_blocks_transpose():
    rng = np.random.default_rng(11)
    M, K, N = 128, 256, 256
    x = _bf16(rng.standard_normal((M, K)))
    w = _bf16(rng.standard_normal((N, K)) * 0.02)
    dy = _bf16(rng.standard_normal((M, N)) * 1e-3)
    dx, dw = orc.block_linear_bwd(dy, x, w)
    dec = orc.decode_table(orc.E4M3FN).astype(np.float64)

    def deq(t, br):
        q, e = orc.block_quantize(t, br, 128, orc.E4M3FN)
        return dec[q] * 2.0 ** (e.astype(np.float64).repeat(32, axis=1) - 127)
    # dX = deq(dY tiles along N) . deq(W^T blocks)^T ;  dW = deq(dY^T tiles along M) . deq(X^T tiles along M)^T
    want_dx = deq(dy, 1) @ deq(np.ascontiguousarray(w.T), 128).T
    want_dw = deq(np.ascontiguousarray(dy.T), 1) @ deq(np.ascontiguousarray(x.T), 1).T
    assert np.allclose(dx.acc64, want_dx, rtol=1e-12, atol=0) and np.allclose(dw.acc64, want_dw, rtol=1e-12, atol=0)
    # square blocks: the blockwise quantization of W^T is the transpose of that of W (codes and scale bytes)
    q, e = orc.block_quantize(w, 128, 128, orc.E4M3FN)
    qt, et = orc.block_quantize(np.ascontiguousarray(w.T), 128, 128, orc.E4M3FN)
    assert (qt == q.T).all()
    assert (et[::128, ::4] == e[::128, ::4].T).all()
    # and both gradients approximate the unquantized ones to the accuracy of two e4m3 operands
    f = lambda t: si.bf16_bits_to_f32(t).astype(np.float64)
    assert np.linalg.norm(want_dx - f(dy) @ f(w)) <= 0.06 * np.linalg.norm(f(dy) @ f(w))
    assert np.linalg.norm(want_dw - f(dy).T @ f(x)) <= 0.06 * np.linalg.norm(f(dy).T @ f(x))
