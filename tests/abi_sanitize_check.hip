// Sanitizer driver for the HOST side of the C ABI (test infrastructure).
//
// Built by tests/test_sanitizers.py from this file, api.hip and tuning.hip with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host code only.  The kernel launchers are replaced by the stubs below
// (they record that they were called and touch nothing), so every entry point can be driven through its
// argument validation AND its workspace planning on a machine without a GPU: the pointers handed in are
// never dereferenced by host code.  Any out-of-bounds access, overflow or misuse inside the ABI layer
// aborts the run.
#include "../include/fp8mi355.h"
#include "../paper_2507_16099_amd/csrc/launchers.hpp"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

static int g_launches = 0;
#define STUB { ++g_launches; return hipSuccess; }
namespace fp8k {
hipError_t launch_fill_u32(uint32_t*, int64_t, uint32_t, hipStream_t) STUB
hipError_t launch_amax(const void*, int64_t, int64_t, int64_t, int, float*, hipStream_t) STUB
hipError_t launch_col_scales_two_level(const void*, int64_t, int64_t, int64_t, int, int, float*, void*, size_t, hipStream_t) { ++g_launches; return hipErrorNotSupported; }
hipError_t launch_quant_tensor(const void*, int64_t, int64_t, int, int, int, uint8_t*, int64_t, uint8_t*, int64_t, float*, float*, hipStream_t) STUB
hipError_t launch_block_quant(const void*, int64_t, int64_t, int64_t, int, int, uint8_t*, int64_t, uint8_t*, int64_t, hipStream_t) STUB
hipError_t launch_block_quant_t(const void*, int64_t, int64_t, int64_t, int, int, uint8_t*, int64_t, uint8_t*, int64_t, hipStream_t, uint8_t*, int64_t, uint8_t*, int64_t) STUB
hipError_t launch_scale(const float*, int64_t, int, int, float*, hipStream_t) STUB
hipError_t launch_cast(const void*, int64_t, int64_t, int64_t, const float*, int, int, int, uint8_t*, int64_t, uint8_t*, int64_t, hipStream_t) STUB
hipError_t launch_quant_row(const void*, int64_t, int64_t, int64_t, int, int, uint8_t*, int64_t, float*, hipStream_t) STUB
hipError_t launch_gemm_fp8(const uint8_t*, int64_t, int, const float*, int, const uint8_t*, int64_t, int, const float*, int, int64_t, int64_t, int64_t, void*, int64_t, int, hipStream_t) STUB
hipError_t launch_quant_row_colmax(const void*, int64_t, int64_t, int64_t, int, int, uint8_t*, int64_t, float*, float*, void*, size_t, hipStream_t) { ++g_launches; return hipErrorNotSupported; }
bool gemm_fp8_snake_fits(int64_t lda, int64_t ldb) { return lda < (1 << 23) && ldb < (1 << 23); }
hipError_t launch_gemm_fp8_snake(const uint8_t*, int64_t, int, const float*, int, const uint8_t*, int64_t, int, const float*, int, int64_t, int64_t, int64_t, void*, int64_t, int, hipStream_t, int) STUB
hipError_t launch_gemm_fp8_skinny(const uint8_t*, int64_t, int, const float*, int, const uint8_t*, int64_t, int, const float*, int, int64_t, int64_t, int64_t, void*, int64_t, int, hipStream_t) STUB
hipError_t launch_gemm_bf16_at_b(const void*, int64_t, const void*, int64_t, int64_t, int64_t, int64_t, void*, int64_t, hipStream_t) STUB
bool gemm_bf16_at_b_snake_fits(int64_t, int64_t, int64_t, int64_t, int64_t) { return true; }
hipError_t launch_gemm_bf16_at_b_snake(const void*, int64_t, const void*, int64_t, int64_t, int64_t, int64_t, void*, int64_t, hipStream_t) STUB
hipError_t launch_quant_row_col_sigmoid_bwd(const void*, const void*, int64_t, int64_t, int64_t, int, int, uint8_t*, int64_t, float*, uint8_t*, int64_t, float*, hipStream_t) STUB
// the paired launches decline every other call, so that both the paired path and the one-by-one path behind it run
#define STUB_ALTERNATING { return (++g_launches & 1) ? hipSuccess : hipErrorNotSupported; }
hipError_t launch_quant_tensor_pair(const TensorOperand&, const TensorOperand&, int64_t, int, int, int, hipStream_t) STUB_ALTERNATING
hipError_t launch_quant_row_pair(const void*, int64_t, int64_t, uint8_t*, int64_t, float*, const void*, int64_t, int64_t, uint8_t*, int64_t, float*, int64_t, int, int, hipStream_t) STUB_ALTERNATING
hipError_t launch_quant_row_col_pair(const RowColOperand&, const RowColOperand*, int64_t, int, int, hipStream_t) STUB_ALTERNATING
int64_t quant_fold_bytes(int64_t rows, int64_t cols) { return rows >= 256 && rows <= 2048 && cols >= 8 && cols % 8 == 0 && rows * cols <= ((int64_t)4 << 20) ? FOLD_ROWS * ((cols + 7) / 8 * 8) * 2 : 0; }
hipError_t launch_linear_skinny_fused(const void*, int64_t, int, int, int, const uint8_t*, int64_t, int, const float*, int, int64_t, int64_t, int64_t, void*, int64_t, hipStream_t) STUB_ALTERNATING
hipError_t launch_quant_col_t_pair(const ColOperand&, const ColOperand&, int64_t, int, int, hipStream_t) STUB_ALTERNATING
hipError_t launch_quant_bwd_rowwise(const RowColOperand&, int64_t, int, const ColOperand&, const ColOperand&, int64_t, int, int, hipStream_t) STUB_ALTERNATING
hipError_t launch_gemm_fp8_pair(const GemmOperands&, const GemmOperands&, int, int, int, int, hipStream_t) STUB_ALTERNATING
hipError_t launch_sigmoid_bwd(const void*, const void*, int64_t, void*, hipStream_t) STUB
hipError_t launch_layernorm_quant_row(const void*, int64_t, int64_t, int64_t, const void*, const void*, double, int, int, void*, int64_t, uint8_t*, int64_t, float*, float*, float*, hipStream_t) STUB
hipError_t launch_mx_quant(const void*, int64_t, int64_t, int64_t, int, uint8_t*, int64_t, uint8_t*, int64_t, hipStream_t) STUB
hipError_t launch_mx_quant_t(const void*, int64_t, int64_t, int64_t, int, uint8_t*, int64_t, uint8_t*, int64_t, uint8_t*, int64_t, uint8_t*, int64_t, hipStream_t) STUB
bool gemm_mxfp8_takes_slab_scales(int64_t, int64_t, int64_t M, int64_t N, int64_t K) { return K % 512 == 0 && M * N > 65536; }
hipError_t launch_gemm_mxfp8(const uint8_t*, int64_t, int, const uint8_t*, int64_t, const uint8_t*, int64_t, int, const uint8_t*, int64_t, int64_t, int64_t, int64_t, void*, int64_t, int, hipStream_t) STUB
hipError_t launch_gemm_mxfp8_snake(const uint8_t*, int64_t, int, const uint8_t*, int64_t, const uint8_t*, int64_t, int, const uint8_t*, int64_t, int64_t, int64_t, int64_t, void*, int64_t, int, hipStream_t) STUB
}  // namespace fp8k

extern "C" int fp8_internal_set_knob(const char* name, int value);

#define EXPECT(call, want)                                                                                  \
    do {                                                                                                    \
        const int got__ = (call);                                                                           \
        if (got__ != (want)) {                                                                              \
            std::fprintf(stderr, "%s:%d: %s returned %d, expected %d (%s)\n", __FILE__, __LINE__, #call, got__, (want), fp8_last_error()); \
            std::exit(1);                                                                                   \
        }                                                                                                   \
    } while (0)

int main() {
    // never dereferenced by host code: a fake, suitably aligned "device" address
    void* p = reinterpret_cast<void*>(uintptr_t(1) << 32);
    uint8_t* q = static_cast<uint8_t*>(p);
    float* f = static_cast<float*>(p);
    const int64_t shapes[][3] = {{0, 0, 0}, {16, 16, 16}, {48, 64, 80}, {4096, 4096, 11008}, {16384, 4096, 14336},
                                 {8192, 28672, 8192}, {2147483647, 16, 8}, {1 << 20, 1 << 16, 1 << 12}, {1000, 64, 48},
                                 {2147483647 - 15, 16, 16}, {2147483647 - 20, 16, 16}, {3, 16, 16}, {96, 128, 160}, {1056, 384, 672}};
    for (const auto& s : shapes) {
        const int64_t M = s[0], K = s[1], N = s[2];
        for (int gran = FP8_TENSOR; gran <= FP8_ROW; ++gran)
            for (int flags : {0, int(FP8_POW2_SCALE), int(FP8_SAVE_FOR_BWD), int(FP8_GRAD_WEIGHT_HP | FP8_SAVE_FOR_BWD)}) {
                const fp8_recipe r{gran, FP8_E4M3FN, FP8_E4M3FN, FP8_E5M2, flags};
                const size_t wf = fp8_linear_workspace_bytes(M, K, N, &r, 0), wb = fp8_linear_workspace_bytes(M, K, N, &r, 1);
                const bool bwd_ok = N % 16 == 0 && M <= 2147483647 - 15;
                if (wf == 0 && !(flags & FP8_SAVE_FOR_BWD && !bwd_ok)) { std::fprintf(stderr, "workspace 0 for %lld %lld %lld\n", (long long)M, (long long)K, (long long)N); return 1; }
                if (wf) EXPECT(fp8_linear_fwd(p, p, M, K, N, &r, p, p, wf, nullptr), FP8_OK);
                if (wf > 256) EXPECT(fp8_linear_fwd(p, p, M, K, N, &r, p, p, wf - 1, nullptr), M && N ? FP8_ERR_WORKSPACE : FP8_OK);
                if (wb && bwd_ok) {
                    EXPECT(fp8_linear_bwd(p, p, p, M, K, N, &r, p, p, p, wb, nullptr), FP8_OK);
                    EXPECT(fp8_linear_bwd(p, p, p, M, K, N, &r, p, nullptr, p, wb, nullptr), FP8_OK);
                    EXPECT(fp8_linear_bwd(p, p, p, M, K, N, &r, nullptr, p, p, wb, nullptr), FP8_OK);
                    const size_t wsg = fp8_linear_bwd_sigmoid_workspace_bytes(M, K, N, &r);
                    if (wsg) EXPECT(fp8_linear_bwd_sigmoid(p, p, p, p, M, K, N, &r, p, p, p, wsg, nullptr), FP8_OK);
                }
            }
        if (M <= (1 << 20) && K % 128 == 0) {
            const size_t wm = fp8_mx_linear_workspace_bytes(M, K, N);
            if (wm) {
                EXPECT(fp8_mx_linear_fwd(p, p, M, K, N, 0, 0, p, p, wm, nullptr), FP8_OK);
                EXPECT(fp8_block_linear_fwd(p, p, M, K, N, 0, 0, p, p, wm, nullptr), FP8_OK);
            }
            if (M % 32 == 0 && N % 32 == 0) {
                const size_t wmx = fp8_mx_linear_bwd_workspace_bytes(M, K, N);
                EXPECT(fp8_mx_linear_bwd(p, p, p, M, K, N, 1, 0, 0, p, p, p, wmx, nullptr), FP8_OK);
                if (wmx > 256) EXPECT(fp8_mx_linear_bwd(p, p, p, M, K, N, 1, 0, 0, p, p, p, wmx - 1, nullptr), M && N && K ? FP8_ERR_WORKSPACE : FP8_OK);
            }
            if (M % 128 == 0 && N % 128 == 0) {
                const size_t wmb = fp8_block_linear_bwd_workspace_bytes(M, K, N);
                EXPECT(fp8_block_linear_bwd(p, p, p, M, K, N, 1, 0, 0, p, p, p, wmb, nullptr), FP8_OK);
            }
        }
        const size_t wp = fp8_linear_prequantized_workspace_bytes(M, K);
        EXPECT(fp8_linear_fwd_prequantized(p, M, K, 0, 1, 0, q, K, 0, f, 1, N, p, N, p, wp, nullptr), FP8_OK);
        EXPECT(fp8_grad_weight_hp(p, p, M, K, N, p, nullptr), FP8_OK);
    }
    // fine-grained entry points on ragged shapes and padded leading dimensions
    for (int gran = FP8_TENSOR; gran <= FP8_COL; ++gran)
        for (int flags : {0, int(FP8_TRANSPOSE_OUT), int(FP8_POW2_SCALE | FP8_TRANSPOSE_OUT)}) {
            EXPECT(fp8_amax(p, 33, 40, 48, gran, f, nullptr), FP8_OK);
            EXPECT(fp8_cast(p, 33, 40, 48, f, gran, 1, flags & FP8_TRANSPOSE_OUT, q, 64, nullptr), FP8_OK);
            EXPECT(fp8_quantize(p, 33, 40, 48, gran, 0, flags, q, 64, f, nullptr), FP8_OK);
            EXPECT(fp8_quantize(p, 3000, 1024, 1024, gran, 0, flags, q, (flags & FP8_TRANSPOSE_OUT) ? 3008 : 1024, f, nullptr), FP8_OK);
        }
    EXPECT(fp8_quantize_row_col(p, 3000, 1024, 1024, 1, 0, q, 1024, f, q, 3008, f, nullptr), FP8_OK);
    EXPECT(fp8_scale(f, 1000, 1, FP8_POW2_SCALE, f, nullptr), FP8_OK);
    EXPECT(fp8_scaled_mm(q, 128, 0, f, 1, q, 144, 1, f, 0, 77, 99, 112, p, 104, FP8_OUT_FP32, nullptr), FP8_OK);
    EXPECT(fp8_scaled_mm(q, 128, 0, f, 1, q, 144, 1, f, 0, 77, 99, 112, p, 104, FP8_EPILOGUE_SIGMOID, nullptr), FP8_OK);
    EXPECT(fp8_layernorm_quantize(p, 77, 4096, 4096, p, nullptr, 1e-5, 0, 0, nullptr, 0, q, 4096, f, nullptr, nullptr, nullptr), FP8_OK);
    EXPECT(fp8_mx_quantize(p, 77, 96, 96, 0, q, 96, q, 4, nullptr), FP8_OK);
    EXPECT(fp8_mx_quantize_t(p, 96, 77 * 8, 77 * 8, 0, q, 96, q, 4, nullptr), FP8_OK);
    EXPECT(fp8_mx_quantize_row_col(p, 96, 64, 64, 0, q, 64, q, 4, q, 96, q, 4, nullptr), FP8_OK);
    EXPECT(fp8_mx_scaled_mm(q, 256, 0, q, 8, q, 256, 0, q, 8, 77, 99, 256, p, 104, 0, nullptr), FP8_OK);
    EXPECT(fp8_block_quantize(p, 77, 256, 256, 128, 0, q, 256, q, 8, nullptr), FP8_OK);
    EXPECT(fp8_block_quantize_t(p, 256, 80, 80, 1, 0, q, 256, q, 8, nullptr), FP8_OK);
    EXPECT(fp8_block_quantize_row_col(p, 256, 128, 128, 0, q, 128, q, 4, q, 256, q, 8, nullptr), FP8_OK);
    // error paths
    EXPECT(fp8_amax(nullptr, 4, 8, 8, 0, f, nullptr), FP8_ERR_NULL);
    EXPECT(fp8_amax(p, 4, 8, 8, 9, f, nullptr), FP8_ERR_ENUM);
    EXPECT(fp8_amax(p, 4, 16, 8, 0, f, nullptr), FP8_ERR_SHAPE);
    EXPECT(fp8_amax(static_cast<uint8_t*>(p) + 2, 4, 8, 8, 0, f, nullptr), FP8_ERR_ALIGN);
    EXPECT(fp8_scaled_mm(q, 16, 0, f, 0, q, 16, 0, f, 0, 4, 4, 8, p, 8, 0, nullptr), FP8_ERR_SHAPE);
    EXPECT(fp8_linear_fwd_prequantized_static(p, 4096, 4096, 0, 1, 0, q, 4096, 0, f, 1, 64, p, 64, nullptr), FP8_ERR_WORKSPACE);
    EXPECT(fp8_internal_set_knob("NO_SUCH_SWITCH", 1), FP8_ERR_ENUM);
    EXPECT(fp8_internal_set_knob("MX_SLAB", 0), FP8_OK);
    if (std::strlen(fp8_last_error()) > 255) return 1;
    std::printf("abi_sanitize_check ok (%d stubbed launches, %s)\n", g_launches, fp8_version());
    return 0;
}
