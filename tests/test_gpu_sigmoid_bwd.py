"""GPU parity: backward through Sigmoid + Linear (fp8_linear_bwd_sigmoid) vs the
CPU oracle.  dz = dy * y * (1 - y) is an exactly specified bfloat16 tensor, so the
entry point must give, bit for bit, what fp8_linear_bwd gives on the oracle's dz
(same codes, same scales, same GEMM kernels), whether dz is formed inside the
quantization passes (rowwise, M >= 1024, 512 <= N <= 32768) or written out first;
dX and dW are also compared with the oracle's backward of that dz."""
import numpy as np
import pytest
import torch

import synthetic_inputs as si
from oracle import fp8_oracle as orc
from tests.gpu_util import dev_bf16, host_bf16_bits

pytestmark = pytest.mark.gpu

import paper_2507_16099_amd as fp8  # noqa: E402


def _inputs(M, K, N, base="c2_llama3_8b_ffn_rowwise"):
    wl = si.scaled_down(si.WORKLOADS[base], M, K, N)
    x, w, dy = wl.x(), wl.w(), wl.dy()
    z = si.normal_bf16((M, N), 2.0, seed=23, stream=M + N)          # pre-activations: y spans (0, 1), some saturate
    y = orc.sigmoid_bf16(si.bf16_bits_to_f32(z))
    return x, w, dy, y


def _close(got_t, want, min_identical=0.97):
    """bfloat16 result against the oracle's bfloat16 result: relative Frobenius error and share of identical bits"""
    got = host_bf16_bits(got_t)
    assert orc.rel_frobenius(si.bf16_bits_to_f32(got), si.bf16_bits_to_f32(want.out16)) <= 1e-3
    assert (got == want.out16).mean() >= min_identical


FUSED = [(1024, 384, 512), (1040, 176, 528), (2048, 256, 4096), (1024, 128, 8208)]
WRITTEN = [(208, 176, 272), (512, 1024, 768), (1024, 256, 384), (1024, 128, 496)]


@pytest.mark.parametrize("M,K,N", FUSED + WRITTEN)
@pytest.mark.parametrize("recipe", ["rowwise", "rowwise_pow2", "rowwise_saved", "tensorwise", "rowwise_gw_hp"])
def test_sigmoid_backward_equals_backward_of_the_oracle_dz(M, K, N, recipe):
    x, w, dy, y = _inputs(M, K, N)
    dz = orc.sigmoid_bwd(dy, y)
    xd, wd, dyd, yd, dzd = dev_bf16(x), dev_bf16(w), dev_bf16(dy), dev_bf16(y), dev_bf16(dz)
    gran = fp8.FP8_TENSOR if recipe == "tensorwise" else fp8.FP8_ROW
    fl = (fp8.FP8_POW2_SCALE if recipe.endswith("pow2") else 0) | (fp8.FP8_GRAD_WEIGHT_HP if recipe.endswith("gw_hp") else 0)
    plain = fp8.Recipe(gran=gran, flags=fl)
    dx0, dw0 = fp8.fp8_linear_bwd(dzd, xd, wd, plain)
    if recipe.endswith("saved"):
        r = fp8.Recipe(gran=gran, flags=fl | fp8.FP8_SAVE_FOR_BWD)
        nbytes = fp8.fp8_linear_bwd_sigmoid_workspace_bytes(M, K, N, r)
        assert nbytes >= fp8.fp8_linear_workspace_bytes(M, K, N, r, True)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        fp8.fp8_linear_fwd(xd, wd, r, workspace=ws)
        dx1, dw1 = fp8.fp8_linear_bwd_sigmoid(dyd, yd, (M, K), (N, K), r, workspace=ws)
    else:
        r = plain
        dx1, dw1 = fp8.fp8_linear_bwd_sigmoid(dyd, yd, xd, wd, r)
    assert torch.equal(dx0.view(torch.int16), dx1.view(torch.int16))
    assert torch.equal(dw0.view(torch.int16), dw1.view(torch.int16))
    o = orc.Recipe(gran=orc.TENSOR if gran == fp8.FP8_TENSOR else orc.ROW, pow2=recipe.endswith("pow2"))
    _close(dx1, orc.linear_bwd_dx(dz, w, o)[0])
    if not recipe.endswith("gw_hp"):
        _close(dw1, orc.linear_bwd_dw(dz, x, o)[0])
    # one output only
    a, none = fp8.fp8_linear_bwd_sigmoid(dyd, yd, xd, wd, plain, need_dw=False)
    assert none is None and torch.equal(a.view(torch.int16), dx0.view(torch.int16))
    none, b = fp8.fp8_linear_bwd_sigmoid(dyd, yd, xd, wd, plain, need_dx=False)
    assert none is None and torch.equal(b.view(torch.int16), dw0.view(torch.int16))


def test_sigmoid_backward_special_values():
    """y = 0 and y = 1 (saturated sigmoid) give dz = +-0 whatever dy; rows of zeros get the
    floor of the amax; e5m2 gradients."""
    M, K, N = 1024, 128, 512
    x, w, dy, y = _inputs(M, K, N)
    y[5, :] = 0
    y[6, :] = 0x3F80                       # 1.0
    y[:, 9] = 0x3F80
    dy[7, :] = 0
    dz = orc.sigmoid_bwd(dy, y)
    assert not (dz[5] & 0x7FFF).any() and not (dz[:, 9] & 0x7FFF).any()
    xd, wd = dev_bf16(x), dev_bf16(w)
    for fmt in (fp8.FP8_E4M3FN, fp8.FP8_E5M2):
        r = fp8.Recipe(gran=fp8.FP8_ROW, fmt_dy=fmt)
        dx0, dw0 = fp8.fp8_linear_bwd(dev_bf16(dz), xd, wd, r)
        dx1, dw1 = fp8.fp8_linear_bwd_sigmoid(dev_bf16(dy), dev_bf16(y), xd, wd, r)
        assert torch.equal(dx0.view(torch.int16), dx1.view(torch.int16))
        assert torch.equal(dw0.view(torch.int16), dw1.view(torch.int16))


def test_sigmoid_backward_rejects_bad_arguments():
    M, K, N = 1024, 128, 512
    x, w, dy, y = _inputs(M, K, N)
    r = fp8.Recipe(gran=fp8.FP8_ROW)
    small = torch.empty(fp8.fp8_linear_bwd_sigmoid_workspace_bytes(M, K, N, r) - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(fp8.Fp8Error):
        fp8.fp8_linear_bwd_sigmoid(dev_bf16(dy), dev_bf16(y), dev_bf16(x), dev_bf16(w), r, workspace=small)
    # the written-out form needs room for dz behind the ordinary backward's workspace
    t = fp8.Recipe(gran=fp8.FP8_TENSOR)
    assert fp8.fp8_linear_bwd_sigmoid_workspace_bytes(M, K, N, t) >= fp8.fp8_linear_workspace_bytes(M, K, N, t, True) + 2 * M * N


def test_sigmoid_backward_full_size_block_shape():
    """dY, Y [16384, 14336] of the benchmark workload: bit-identical to the backward of a
    dz written by the oracle, both outputs."""
    wl = si.WORKLOADS[si.BENCH_WORKLOAD]
    M, K, N = wl.M, wl.K, wl.N
    dy = wl.dy()
    z = si.normal_bf16((M, N), 2.0, seed=23, stream=1)
    y = orc.sigmoid_bf16(si.bf16_bits_to_f32(z))
    dz = orc.sigmoid_bwd(dy, y)
    xd, wd = dev_bf16(wl.x()), dev_bf16(wl.w())
    r = fp8.Recipe(gran=fp8.FP8_ROW)
    dx0, dw0 = fp8.fp8_linear_bwd(dev_bf16(dz), xd, wd, r)
    dx1, dw1 = fp8.fp8_linear_bwd_sigmoid(dev_bf16(dy), dev_bf16(y), xd, wd, r)
    assert torch.equal(dx0.view(torch.int16), dx1.view(torch.int16))
    assert torch.equal(dw0.view(torch.int16), dw1.view(torch.int16))
