"""The entry points only enqueue kernels on the caller's stream (no allocation,
no memset nodes, no host synchronisation), so a whole training step can be
recorded into a HIP graph.  Each replay, with new inputs written into the same
buffers and eager work in between, must reproduce the eager result bit for bit."""
import numpy as np
import pytest
import torch

import synthetic_inputs as si
from tests.gpu_util import dev_bf16

pytestmark = pytest.mark.gpu

import paper_2507_16099_amd as fp8  # noqa: E402


def _bits(t):
    return t.view(torch.int16).clone()


@pytest.mark.parametrize("recipe", ["rowwise", "rowwise_saved", "tensorwise", "tensorwise_saved", "rowwise_gw_hp", "mx",
                                    "rowwise_sigmoid", "block"])
def test_step_replays_from_a_hip_graph(recipe):
    M, K, N = 1024, 512, 768
    wl = si.scaled_down(si.WORKLOADS["c2_llama3_8b_ffn_rowwise"], M, K, N)
    inputs = []
    for seed in range(3):
        w2 = si.Workload(wl.name, M, K, N, wl.recipe, wl.pow2, wl.x_dist, wl.w_dist, wl.dy_dist, wl.backward, seed)
        inputs.append((dev_bf16(w2.x()), dev_bf16(w2.w()), dev_bf16(w2.dy())))
    x, w, dy = (torch.empty_like(t) for t in inputs[0])
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    dx = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    dw = torch.empty((N, K), dtype=torch.bfloat16, device="cuda")
    if recipe == "block":
        ws_f = torch.empty(fp8.fp8_block_linear_workspace_bytes(M, K, N), dtype=torch.uint8, device="cuda")
        ws_b = torch.empty(fp8.fp8_block_linear_bwd_workspace_bytes(M, K, N), dtype=torch.uint8, device="cuda")

        def step():
            fp8.fp8_block_linear_fwd(x, w, y=y, workspace=ws_f)
            fp8.fp8_block_linear_bwd(dy, x, w, dx=dx, dw=dw, workspace=ws_b)
    elif recipe == "mx":
        ws_f = torch.empty(fp8.fp8_mx_linear_workspace_bytes(M, K, N), dtype=torch.uint8, device="cuda")
        ws_b = torch.empty(fp8.fp8_mx_linear_bwd_workspace_bytes(M, K, N), dtype=torch.uint8, device="cuda")

        def step():
            fp8.fp8_mx_linear_fwd(x, w, y=y, workspace=ws_f)
            fp8.fp8_mx_linear_bwd(dy, x, w, dx=dx, dw=dw, workspace=ws_b)
    elif recipe == "rowwise_sigmoid":
        # sigmoid inside the forward GEMM's epilogue, its gradient inside the backward's quantization
        r = fp8.Recipe(gran=fp8.FP8_ROW)
        ws_f = torch.empty(fp8.fp8_linear_workspace_bytes(M, K, N, r, False), dtype=torch.uint8, device="cuda")
        ws_b = torch.empty(fp8.fp8_linear_bwd_sigmoid_workspace_bytes(M, K, N, r), dtype=torch.uint8, device="cuda")
        xq = torch.empty((M, K), dtype=torch.uint8, device="cuda")
        wq = torch.empty((N, K), dtype=torch.uint8, device="cuda")
        sx = torch.empty(M, dtype=torch.float32, device="cuda")
        sw = torch.empty(N, dtype=torch.float32, device="cuda")

        def step():
            fp8.fp8_quantize(x, fp8.FP8_ROW, fp8.FP8_E4M3FN, out=xq, scale_out=sx)
            fp8.fp8_quantize(w, fp8.FP8_ROW, fp8.FP8_E4M3FN, out=wq, scale_out=sw)
            fp8.fp8_scaled_mm(xq, fp8.FP8_E4M3FN, sx, fp8.FP8_ROW, wq, fp8.FP8_E4M3FN, sw, fp8.FP8_ROW,
                              fp8.FP8_EPILOGUE_SIGMOID, out=y)
            fp8.fp8_linear_bwd_sigmoid(dy, y, x, w, r, dx=dx, dw=dw, workspace=ws_b)
    else:
        r = {"rowwise": fp8.Recipe(gran=fp8.FP8_ROW), "tensorwise": fp8.Recipe(gran=fp8.FP8_TENSOR),
             "tensorwise_saved": fp8.Recipe(gran=fp8.FP8_TENSOR, flags=fp8.FP8_SAVE_FOR_BWD),
             "rowwise_saved": fp8.Recipe(gran=fp8.FP8_ROW, flags=fp8.FP8_SAVE_FOR_BWD),
             "rowwise_gw_hp": fp8.Recipe(gran=fp8.FP8_ROW, flags=fp8.FP8_GRAD_WEIGHT_HP)}[recipe]
        ws_b = torch.empty(fp8.fp8_linear_workspace_bytes(M, K, N, r, True), dtype=torch.uint8, device="cuda")
        ws_f = ws_b if recipe.endswith("_saved") else torch.empty(fp8.fp8_linear_workspace_bytes(M, K, N, r, False),
                                                                     dtype=torch.uint8, device="cuda")

        def step():
            fp8.fp8_linear_fwd(x, w, r, y=y, workspace=ws_f)
            fp8.fp8_linear_bwd(dy, x, w, r, dx=dx, dw=dw, workspace=ws_b)

    def load(i):
        for dst, src in zip((x, w, dy), inputs[i]):
            dst.copy_(src)

    # eager results for every input set (the first call also does the one-time kernel attribute set-up)
    eager = []
    for i in range(3):
        load(i)
        step()
        torch.cuda.synchronize()
        eager.append((_bits(y), _bits(dx), _bits(dw)))

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    load(0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for i in (1, 2, 0, 2):
        load(i)
        for t in (y, dx, dw, ws_f, ws_b):
            t.zero_()                              # eager work between the replays; stale results cannot pass
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want, name in zip((y, dx, dw), eager[i], ("y", "dx", "dw")):
            assert torch.equal(got.view(torch.int16), want), (recipe, i, name)


@pytest.mark.parametrize("M", [1, 4, 12])
def test_decode_linear_replays_from_a_hip_graph(M):
    """The decode linear with a weight quantized once - one launch for a few tokens, two launches beyond -
    recorded once and replayed with new activations in the same buffer."""
    K, N = 2048, 1000
    w = dev_bf16(si.normal_bf16((N, K), 0.02, 11, 0))
    wq, sw = fp8.fp8_quantize(w, fp8.FP8_ROW, fp8.FP8_E4M3FN)
    inputs = [dev_bf16(si.f32_to_bf16_bits(si.bf16_bits_to_f32(si.normal_bf16((M, K), 1.0, 11, 1 + s)) * np.float32(0.5 + 3 * s)))
              for s in range(3)]
    x = torch.empty_like(inputs[0])
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(fp8.fp8_linear_prequantized_workspace_bytes(M, K), dtype=torch.uint8, device="cuda")

    def step():
        fp8.fp8_linear_fwd_prequantized(x, wq, fp8.FP8_E4M3FN, sw, fp8.FP8_ROW, fp8.FP8_E4M3FN, fp8.FP8_ROW, 0, y=y, workspace=ws)

    eager = []
    for i in range(3):
        x.copy_(inputs[i])
        step()
        torch.cuda.synchronize()
        eager.append(_bits(y))
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    x.copy_(inputs[0])
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for i in (1, 2, 0, 2):
        x.copy_(inputs[i])
        y.zero_()
        ws.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), eager[i]), (M, i)
