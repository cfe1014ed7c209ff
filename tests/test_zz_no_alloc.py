"""fp8_linear_fwd_prequantized_static: the entry point that allocates nothing (its scratch is a static device
array inside the library).  Its output must equal that of fp8_linear_fwd_prequantized bit for bit - same kernels,
same codes - also on a second call with a smaller input, which finds the first call's contents in the buffer."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2507_16099_amd as fp8
import synthetic_inputs as si
from tests.gpu_util import dev_bf16, host_bf16_bits

pytestmark = pytest.mark.gpu


def _case(M, K, N, gran_x, gran_w, seed):
    x = dev_bf16(si.normal_bf16((M, K), 1.0, seed, 0))
    w = dev_bf16(si.normal_bf16((N, K), 0.02, seed, 1))
    wq, sw = fp8.fp8_quantize(w, gran_w, fp8.FP8_E4M3FN)
    want = fp8.fp8_linear_fwd_prequantized(x, wq, fp8.FP8_E4M3FN, sw, gran_w, fp8.FP8_E4M3FN, gran_x)
    got = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    fp8.fp8_linear_fwd_prequantized_static(x, wq, fp8.FP8_E4M3FN, sw, gran_w, got, fp8.FP8_E4M3FN, gran_x)
    torch.cuda.synchronize()
    return host_bf16_bits(got), host_bf16_bits(want)


def test_static_scratch_entry_point_matches_the_workspace_one():
    # two calls in a row through the same static buffer, the second with a smaller input; then a tiled
    # (many-row) shape and the tensorwise path, which leaves an amax and a scale in the buffer
    for M, K, N, gx, gw in ((24, 4096, 1024, fp8.FP8_ROW, fp8.FP8_ROW),
                            (12, 512, 264, fp8.FP8_ROW, fp8.FP8_ROW),
                            (300, 1024, 520, fp8.FP8_TENSOR, fp8.FP8_TENSOR),
                            (16, 256, 64, fp8.FP8_ROW, fp8.FP8_TENSOR),
                            (1, 1024, 520, fp8.FP8_ROW, fp8.FP8_ROW)):      # one token: quantized inside the product, the buffer stays untouched
        print(f"static scratch case M={M} K={K} N={N} gran_x={gx} gran_w={gw}", flush=True)
        got, want = _case(M, K, N, gx, gw, seed=M)
        assert np.array_equal(got, want), (M, K, N)


def test_static_scratch_rejects_what_does_not_fit():
    L = fp8.load_library()
    x = torch.zeros((16, 64), dtype=torch.bfloat16, device="cuda")
    p = x.data_ptr()
    # 4096 x 4096 activation codes are 16 MiB: more than the 8 MiB buffer -> FP8_ERR_WORKSPACE, nothing launched
    rc = L.fp8_linear_fwd_prequantized_static(p, 4096, 4096, 0, 1, 0, p, 4096, 0, p, 1, 64, p, 64, None)
    assert rc == -5 and "static buffer" in fp8.fp8_last_error()
    assert fp8.FP8_STATIC_SCRATCH_BYTES == 8 << 20
