"""GPU parity: layer normalisation with the fused rowwise float8 quantization
(fp8_layernorm_quantize) vs the CPU oracle.  The normalised bfloat16 tensor, the
scales and the fp8 codes bit for bit (both sides decide them from binary64
statistics rounded once); mean and rstd to binary32 round-off."""
import numpy as np
import pytest
import torch

import synthetic_inputs as si
from oracle import fp8_oracle as orc
from tests.gpu_util import dev_bf16, host_bf16_bits, host_u8

pytestmark = pytest.mark.gpu

import paper_2507_16099_amd as fp8  # noqa: E402


def _vec(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def _check(x, g, b, eps, fmt, pow2, ld=None):
    h, q, s, mean, rstd = fp8.fp8_layernorm_quantize(dev_bf16(x, ld), _vec(g), None if b is None else _vec(b), eps, fmt,
                                                     fp8.FP8_POW2_SCALE if pow2 else 0)
    wh, wq, ws, wmean, wrstd = orc.layernorm_quantize(x, g, b, eps, fmt, pow2)
    gh = host_bf16_bits(h)
    assert (gh == wh).all(), (np.argwhere(gh != wh)[:4], gh[gh != wh][:4], wh[gh != wh][:4])
    assert (s.cpu().numpy().view(np.uint32) == ws.view(np.uint32)).all()
    assert (host_u8(q) == wq).all()
    assert np.allclose(mean.cpu().numpy(), wmean, rtol=1e-6, atol=1e-30)
    assert np.allclose(rstd.cpu().numpy(), wrstd, rtol=1e-6, atol=0)


@pytest.mark.parametrize("rows,cols,ld", [(1, 8, 8), (5, 24, 32), (7, 512, 512), (33, 520, 520), (64, 1024, 1032),
                                          (300, 4096, 4096), (17, 8192, 8192), (9, 14336, 14336), (3, 16384, 16384)])
@pytest.mark.parametrize("fmt", [orc.E4M3FN, orc.E5M2])
def test_layernorm_quantize_shapes(rows, cols, ld, fmt):
    x = si.normal_bf16((rows, cols), 2.0, seed=11, stream=rows)
    xf = si.bf16_bits_to_f32(x)
    xf += 3.0                                                         # a mean well away from zero
    x = si.f32_to_bf16_bits(xf)
    rng = np.random.default_rng(cols)
    g = si.f32_to_bf16_bits(rng.uniform(0.5, 1.5, cols).astype(np.float32))
    b = si.f32_to_bf16_bits(rng.uniform(-0.5, 0.5, cols).astype(np.float32))
    _check(x, g, b, 1e-5, fmt, pow2=False, ld=ld)


def test_layernorm_quantize_outliers_constant_rows_and_options():
    rows, cols = 40, 4096
    x = si.student_t_outlier_bf16((rows, cols), 3.0, 0.001, 100.0, seed=4, stream=1)
    x[3, :] = si.f32_to_bf16_bits(np.full(cols, -2.5, np.float32))   # zero variance: h = beta
    x[4, :] = 0
    g = si.f32_to_bf16_bits(np.ones(cols, np.float32))
    b = si.f32_to_bf16_bits(np.linspace(-1, 1, cols).astype(np.float32))
    _check(x, g, b, 1e-5, orc.E4M3FN, pow2=True)
    _check(x, g, None, 1e-6, orc.E4M3FN, pow2=False)
    # optional outputs skipped: same codes
    xd = dev_bf16(x)
    h, q, s, mean, rstd = fp8.fp8_layernorm_quantize(xd, _vec(g), _vec(b), 1e-5)
    h2, q2, s2, mean2, rstd2 = fp8.fp8_layernorm_quantize(xd, _vec(g), _vec(b), 1e-5, want_h=False, want_stats=False)
    assert h2 is None and mean2 is None and rstd2 is None
    assert torch.equal(q, q2) and torch.equal(s, s2)
    # the fused result equals the library's own rowwise quantization of h
    q3, s3 = fp8.fp8_quantize(h, fp8.FP8_ROW, fp8.FP8_E4M3FN)
    assert torch.equal(q, q3) and torch.equal(s, s3)
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_layernorm_quantize(dev_bf16(x[:, :4092]), _vec(g[:4092]), None, 1e-5)     # cols % 8


def test_layernorm_quantize_full_size_activations():
    """X [16384, 4096] of the benchmark workload, whole tensor bit for bit."""
    wl = si.WORKLOADS[si.BENCH_WORKLOAD]
    x = wl.x()
    rng = np.random.default_rng(0)
    g = si.f32_to_bf16_bits(rng.uniform(0.5, 1.5, wl.K).astype(np.float32))
    b = si.f32_to_bf16_bits(rng.uniform(-0.5, 0.5, wl.K).astype(np.float32))
    _check(x, g, b, 1e-5, orc.E4M3FN, pow2=False)
