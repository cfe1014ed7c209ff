// C ABI of libfp8mi355.so: argument validation, workspace planning and the
// composition of the linear forward / backward out of the kernels.
// Every entry point validates on the host, then only enqueues work.
#include "../../include/fp8mi355.h"
#include "launchers.hpp"

#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

// Scratch of fp8_linear_fwd_prequantized_static, the entry point for callers that cannot allocate: every GPU the
// library runs on holds its own copy of this array until the process ends.  In host code the name is only a handle
// for hipGetSymbolAddress; kernels and copies get the per-device address that call returns.
static __device__ __align__(256) unsigned char scratch[FP8_STATIC_SCRATCH_BYTES];

namespace {

thread_local char g_err[256] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(hipError_t e, const char* what) {
    return fail(FP8_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
bool fmt_ok(int f) { return f == FP8_E4M3FN || f == FP8_E5M2; }
bool gran_ok(int g) { return g == FP8_TENSOR || g == FP8_ROW || g == FP8_COL; }
constexpr int64_t kMaxDim = 0x7FFFFFFF;

#define FP8_TRY(expr)                               \
    do {                                            \
        hipError_t e__ = (expr);                    \
        if (e__ != hipSuccess) return hip_fail(e__, #expr); \
    } while (0)

// common checks of a bfloat16 input matrix
int check_bf16(const char* fn, const void* x, int64_t rows, int64_t cols, int64_t ld) {
    if (rows < 0 || cols < 0 || rows > kMaxDim || cols > kMaxDim)
        return fail(FP8_ERR_SHAPE, "%s: rows=%lld cols=%lld out of range", fn, (long long)rows, (long long)cols);
    if (ld < cols) return fail(FP8_ERR_SHAPE, "%s: ld=%lld < cols=%lld", fn, (long long)ld, (long long)cols);
    if (rows > 0 && cols > 0) {
        if (!x) return fail(FP8_ERR_NULL, "%s: input pointer is NULL", fn);
        if (!aligned(x, 16)) return fail(FP8_ERR_ALIGN, "%s: input pointer not 16-byte aligned", fn);
        if (ld % 8 != 0) return fail(FP8_ERR_ALIGN, "%s: ld=%lld not a multiple of 8", fn, (long long)ld);
    }
    return FP8_OK;
}

int64_t n_groups(int gran, int64_t rows, int64_t cols) {
    return gran == FP8_TENSOR ? 1 : (gran == FP8_ROW ? rows : cols);
}

// bytes at the start of an fp8 output [out_rows, out_cols] (leading dimension ld_out) that may hold scratch data
// before the cast writes its codes: every byte of a dense matrix, else only the first row (the bytes between the
// rows of a padded output belong to the caller and are never written)
size_t output_scratch_bytes(int64_t out_rows, int64_t out_cols, int64_t ld_out) {
    return ld_out == out_cols ? (size_t)out_rows * (size_t)out_cols : (size_t)out_cols;
}

// amax -> scale -> cast of one operand; amax_tmp has n_groups floats
int quantize_impl(const void* x, int64_t rows, int64_t cols, int64_t ld, int gran, int format, int flags,
                  uint8_t* q, int64_t ld_out, uint8_t* q_plain, int64_t ld_plain, float* scale_out,
                  hipStream_t st, float* part = nullptr) {
    const int transpose = (flags & FP8_TRANSPOSE_OUT) ? 1 : 0;
    const int pow2 = flags & FP8_POW2_SCALE;
    // dense tensor, one scale, scratch for the per-block maxima at hand: two launches instead of four
    if (gran == FP8_TENSOR && part != nullptr && ld == cols) {
        FP8_TRY(fp8k::launch_quant_tensor(x, rows, cols, format, pow2, transpose, q, ld_out, q_plain, ld_plain, scale_out,
                                          part, st));
        return FP8_OK;
    }
    if (gran == FP8_ROW && !transpose) {
        hipError_t e = fp8k::launch_quant_row(x, rows, cols, ld, format, pow2, q, ld_out, scale_out, st);
        if (e == hipSuccess) return FP8_OK;
        if (e != hipErrorNotSupported) return hip_fail(e, "quant_row");
    }
    // scale_out doubles as the amax buffer: fp8_scale may run in place.  For a
    // per-column quantization with transposed output, the output buffer itself
    // (overwritten by the cast afterwards) serves as the scratch matrix of the
    // two-level column amax - only the bytes that the cast will rewrite: all of a
    // dense output, the first row of one whose rows are padded (ld_out > rows).
    hipError_t ea = hipErrorNotSupported;
    if (gran == FP8_COL && transpose && q_plain == nullptr && rows > 0 && cols > 0)
        ea = fp8k::launch_col_scales_two_level(x, rows, cols, ld, format, pow2, scale_out, q,
                                               output_scratch_bytes(cols, rows, ld_out), st);
    if (ea == hipErrorNotSupported) {
        ea = fp8k::launch_amax(x, rows, cols, ld, gran, scale_out, st);
        if (ea != hipSuccess) return hip_fail(ea, "amax");
        FP8_TRY(fp8k::launch_scale(scale_out, n_groups(gran, rows, cols), format, pow2, scale_out, st));
    } else if (ea != hipSuccess) {
        return hip_fail(ea, "column scales");
    }
    FP8_TRY(fp8k::launch_cast(x, rows, cols, ld, scale_out, gran, format, transpose, q, ld_out, q_plain, ld_plain, st));
    return FP8_OK;
}

// rowwise codes and per-column transposed codes of one tensor, the column
// maxima gathered while the rowwise codes are written (q_col_t holds the
// first-level maxima until the cast overwrites it)
int quantize_row_col_impl(const void* x, int64_t rows, int64_t cols, int64_t ld, int format, int flags,
                          uint8_t* q_row, int64_t ld_row, float* scale_row, uint8_t* q_col_t, int64_t ld_col_t,
                          float* scale_col, hipStream_t st) {
    const int pow2 = flags & FP8_POW2_SCALE;
    hipError_t e = hipErrorNotSupported;
    if (rows > 0 && cols > 0)
        e = fp8k::launch_quant_row_colmax(x, rows, cols, ld, format, pow2, q_row, ld_row, scale_row, scale_col, q_col_t,
                                          output_scratch_bytes(cols, rows, ld_col_t), st);
    if (e == hipSuccess) {
        FP8_TRY(fp8k::launch_cast(x, rows, cols, ld, scale_col, FP8_COL, format, 1, q_col_t, ld_col_t, nullptr, 0, st));
        return FP8_OK;
    }
    if (e != hipErrorNotSupported) return hip_fail(e, "quant_row_colmax");
    if (int rc = quantize_impl(x, rows, cols, ld, FP8_ROW, format, pow2, q_row, ld_row, nullptr, 0, scale_row, st)) return rc;
    return quantize_impl(x, rows, cols, ld, FP8_COL, format, pow2 | FP8_TRANSPOSE_OUT, q_col_t, ld_col_t, nullptr, 0,
                         scale_col, st);
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
// Leading dimension of the operands whose contraction axis is the token axis M (dY^T [N, M] and X^T [K, M] of the
// weight gradient): rows of 16-byte multiples for the products' loads.  The pad columns hold zero codes (the buffers
// are cleared before the transposing casts write the valid part), so the product may contract over the padded length.
int64_t pad16(int64_t v) { return (v + 15) / 16 * 16; }

// part: per-block maxima of the tensorwise amax pass, room for two tensors (a pair shares its launches; otherwise one
// tensor at a time: the casts consume them in stream order)
// fold_*: side storage for first-level column maxima of small tensors (rowwise recipe; may be empty)
struct FwdPlan {
    size_t xq, wq, sx, sw, part, fold_x, fold_w, total;
};
struct BwdPlan {
    size_t gq, gqt, wt, xt, sg, sgt, swt, sxt, part, fold_g, fold_w, fold_x, total;
};

FwdPlan plan_fwd(int64_t M, int64_t K, int64_t N, int gran) {
    FwdPlan p{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    p.xq = take((size_t)M * K);
    p.wq = take((size_t)N * K);
    p.sx = take(sizeof(float) * (gran == FP8_ROW ? (size_t)M : 1));
    p.sw = take(sizeof(float) * (gran == FP8_ROW ? (size_t)N : 1));
    p.part = take(2 * sizeof(float) * fp8k::TENSOR_PARTIALS);
    p.fold_x = take(gran == FP8_ROW ? (size_t)fp8k::quant_fold_bytes(M, K) : 0);
    p.fold_w = take(gran == FP8_ROW ? (size_t)fp8k::quant_fold_bytes(N, K) : 0);
    p.total = o;
    return p;
}

BwdPlan plan_bwd(int64_t M, int64_t K, int64_t N, int gran) {
    BwdPlan p{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    const bool row = gran == FP8_ROW;
    p.gq = take((size_t)M * N);   // dY codes, [M, N]
    p.gqt = take((size_t)pad16(M) * N);  // dY codes, [N, M] (rows padded to multiples of 16 bytes)
    p.wt = take((size_t)K * N);   // W codes,  [K, N]
    p.xt = take((size_t)K * pad16(M));   // X codes,  [K, M] (rows padded likewise)
    p.sg = take(sizeof(float) * (row ? (size_t)M : 1));
    p.sgt = take(sizeof(float) * (row ? (size_t)N : 1));
    p.swt = take(sizeof(float) * (row ? (size_t)K : 1));
    p.sxt = take(sizeof(float) * (row ? (size_t)K : 1));
    p.part = take(2 * sizeof(float) * fp8k::TENSOR_PARTIALS);
    p.fold_g = take(row ? (size_t)fp8k::quant_fold_bytes(M, N) : 0);
    p.fold_w = take(row ? (size_t)fp8k::quant_fold_bytes(N, K) : 0);
    p.fold_x = take(row ? (size_t)fp8k::quant_fold_bytes(M, K) : 0);
    p.total = o;
    return p;
}

// The two products of a backward step from quantized operands: dX[M, K] = dY W (contraction over N) and
// dW[N, K] = dY^T X (contraction over M).  sg / sgt: scales of dY for the first / second product (the same
// pointer for tensorwise scaling).  Small products share one launch.  Mp: padded token count, the leading dimension
// of gqt and xt and the contraction length of the second product.
int grad_gemms(const fp8_recipe* r, int row, const uint8_t* gq, const float* sg, const uint8_t* wt, const float* swt,
               const uint8_t* gqt, const float* sgt, const uint8_t* xt, const float* sxt, int64_t M, int64_t Mp, int64_t K,
               int64_t N, void* dx, void* dw, hipStream_t st) {
    if (dx && dw && r->fmt_w == r->fmt_x) {
        const fp8k::GemmOperands g1{gq, N, sg, wt, N, swt, M, K, N, dx, K}, g2{gqt, Mp, sgt, xt, Mp, sxt, N, K, Mp, dw, K};
        const hipError_t e = fp8k::launch_gemm_fp8_pair(g1, g2, r->fmt_dy, r->fmt_w, row, row, st);
        if (e == hipSuccess) return FP8_OK;
        if (e != hipErrorNotSupported) return hip_fail(e, "gemm_fp8_pair");
    }
    if (dx) FP8_TRY(fp8k::launch_gemm_fp8(gq, N, r->fmt_dy, sg, row, wt, N, r->fmt_w, swt, row, M, K, N, dx, K, 0, st));
    if (dw) FP8_TRY(fp8k::launch_gemm_fp8(gqt, Mp, r->fmt_dy, sgt, row, xt, Mp, r->fmt_x, sxt, row, N, K, Mp, dw, K, 0, st));
    return FP8_OK;
}

int check_recipe(const char* fn, const fp8_recipe* r) {
    if (!r) return fail(FP8_ERR_NULL, "%s: recipe is NULL", fn);
    if (r->gran != FP8_TENSOR && r->gran != FP8_ROW)
        return fail(FP8_ERR_ENUM, "%s: recipe.gran=%d must be FP8_TENSOR or FP8_ROW", fn, r->gran);
    if (!fmt_ok(r->fmt_x) || !fmt_ok(r->fmt_w) || !fmt_ok(r->fmt_dy))
        return fail(FP8_ERR_ENUM, "%s: unknown fp8 format in recipe", fn);
    if (r->flags & ~(FP8_POW2_SCALE | FP8_GRAD_WEIGHT_HP | FP8_SAVE_FOR_BWD))
        return fail(FP8_ERR_ENUM, "%s: recipe.flags=%d has unknown bits", fn, r->flags);
    return FP8_OK;
}

int check_linear_dims(const char* fn, int64_t M, int64_t K, int64_t N, bool bwd) {
    if (M < 0 || K < 0 || N < 0 || M > kMaxDim || K > kMaxDim || N > kMaxDim)
        return fail(FP8_ERR_SHAPE, "%s: M=%lld K=%lld N=%lld out of range", fn, (long long)M, (long long)K, (long long)N);
    if (K % 16 != 0) return fail(FP8_ERR_SHAPE, "%s: K=%lld must be a multiple of 16", fn, (long long)K);
    if (N % 8 != 0) return fail(FP8_ERR_SHAPE, "%s: N=%lld must be a multiple of 8 (dense bfloat16 rows)", fn, (long long)N);
    if (bwd && N % 16 != 0)
        return fail(FP8_ERR_SHAPE, "%s: the backward contracts over N: N=%lld must be a multiple of 16", fn, (long long)N);
    if (bwd && M > kMaxDim - 15)
        return fail(FP8_ERR_SHAPE, "%s: M=%lld, padded to a multiple of 16, is out of range", fn, (long long)M);
    return FP8_OK;
}

}  // namespace

extern "C" {

const char* fp8_last_error(void) { return g_err; }

const char* fp8_version(void) { return "fp8mi355 0.2 (gfx950)"; }

int fp8_amax(const void* x, int64_t rows, int64_t cols, int64_t ld, int gran, float* amax_out, void* stream) {
    g_err[0] = 0;
    if (!gran_ok(gran)) return fail(FP8_ERR_ENUM, "fp8_amax: unknown granularity %d", gran);
    if (int rc = check_bf16("fp8_amax", x, rows, cols, ld)) return rc;
    if (n_groups(gran, rows, cols) > 0 && !amax_out) return fail(FP8_ERR_NULL, "fp8_amax: amax_out is NULL");
    if (!aligned(amax_out, 4)) return fail(FP8_ERR_ALIGN, "fp8_amax: amax_out not 4-byte aligned");
    FP8_TRY(fp8k::launch_amax(x, rows, cols, ld, gran, amax_out, static_cast<hipStream_t>(stream)));
    return FP8_OK;
}

int fp8_scale(const float* amax, int64_t n, int format, int flags, float* scale_out, void* stream) {
    g_err[0] = 0;
    if (!fmt_ok(format)) return fail(FP8_ERR_ENUM, "fp8_scale: unknown format %d", format);
    if (flags & ~FP8_POW2_SCALE) return fail(FP8_ERR_ENUM, "fp8_scale: flags=%d has unknown bits", flags);
    if (n < 0) return fail(FP8_ERR_SHAPE, "fp8_scale: n=%lld is negative", (long long)n);
    if (n > 0 && (!amax || !scale_out)) return fail(FP8_ERR_NULL, "fp8_scale: NULL pointer");
    if (!aligned(amax, 4) || !aligned(scale_out, 4)) return fail(FP8_ERR_ALIGN, "fp8_scale: pointer not 4-byte aligned");
    FP8_TRY(fp8k::launch_scale(amax, n, format, flags, scale_out, static_cast<hipStream_t>(stream)));
    return FP8_OK;
}

static int check_q_out(const char* fn, const uint8_t* q, int64_t rows, int64_t cols, int64_t ld_out, int transpose) {
    const int64_t out_cols = transpose ? rows : cols;
    if (ld_out < out_cols) return fail(FP8_ERR_SHAPE, "%s: ld_out=%lld < %lld", fn, (long long)ld_out, (long long)out_cols);
    if (rows > 0 && cols > 0) {
        if (!q) return fail(FP8_ERR_NULL, "%s: q_out is NULL", fn);
        if (!aligned(q, 16)) return fail(FP8_ERR_ALIGN, "%s: q_out not 16-byte aligned", fn);
        if (ld_out % 16 != 0) return fail(FP8_ERR_ALIGN, "%s: ld_out=%lld not a multiple of 16", fn, (long long)ld_out);
        if (transpose && (cols + 127) / 128 > 65535) return fail(FP8_ERR_SHAPE, "%s: too many columns for a transposed cast", fn);
    }
    return FP8_OK;
}

int fp8_cast(const void* x, int64_t rows, int64_t cols, int64_t ld, const float* scale, int gran, int format,
             int flags, uint8_t* q_out, int64_t ld_out, void* stream) {
    g_err[0] = 0;
    if (!gran_ok(gran)) return fail(FP8_ERR_ENUM, "fp8_cast: unknown granularity %d", gran);
    if (!fmt_ok(format)) return fail(FP8_ERR_ENUM, "fp8_cast: unknown format %d", format);
    if (flags & ~FP8_TRANSPOSE_OUT) return fail(FP8_ERR_ENUM, "fp8_cast: flags=%d has unknown bits", flags);
    if (int rc = check_bf16("fp8_cast", x, rows, cols, ld)) return rc;
    const int transpose = (flags & FP8_TRANSPOSE_OUT) ? 1 : 0;
    if (int rc = check_q_out("fp8_cast", q_out, rows, cols, ld_out, transpose)) return rc;
    if (rows > 0 && cols > 0 && !scale) return fail(FP8_ERR_NULL, "fp8_cast: scale is NULL");
    if (!aligned(scale, 4)) return fail(FP8_ERR_ALIGN, "fp8_cast: scale not 4-byte aligned");
    FP8_TRY(fp8k::launch_cast(x, rows, cols, ld, scale, gran, format, transpose, q_out, ld_out, nullptr, 0,
                              static_cast<hipStream_t>(stream)));
    return FP8_OK;
}

int fp8_quantize(const void* x, int64_t rows, int64_t cols, int64_t ld, int gran, int format, int flags,
                 uint8_t* q_out, int64_t ld_out, float* scale_out, void* stream) {
    g_err[0] = 0;
    if (!gran_ok(gran)) return fail(FP8_ERR_ENUM, "fp8_quantize: unknown granularity %d", gran);
    if (!fmt_ok(format)) return fail(FP8_ERR_ENUM, "fp8_quantize: unknown format %d", format);
    if (flags & ~(FP8_TRANSPOSE_OUT | FP8_POW2_SCALE)) return fail(FP8_ERR_ENUM, "fp8_quantize: flags=%d has unknown bits", flags);
    if (int rc = check_bf16("fp8_quantize", x, rows, cols, ld)) return rc;
    const int transpose = (flags & FP8_TRANSPOSE_OUT) ? 1 : 0;
    if (int rc = check_q_out("fp8_quantize", q_out, rows, cols, ld_out, transpose)) return rc;
    if (n_groups(gran, rows, cols) > 0 && !scale_out) return fail(FP8_ERR_NULL, "fp8_quantize: scale_out is NULL");
    if (!aligned(scale_out, 4)) return fail(FP8_ERR_ALIGN, "fp8_quantize: scale_out not 4-byte aligned");
    return quantize_impl(x, rows, cols, ld, gran, format, flags, q_out, ld_out, nullptr, 0, scale_out,
                         static_cast<hipStream_t>(stream));
}

int fp8_quantize_row_col(const void* x, int64_t rows, int64_t cols, int64_t ld, int format, int flags,
                         uint8_t* q_row, int64_t ld_row, float* scale_row, uint8_t* q_col_t, int64_t ld_col_t,
                         float* scale_col, void* stream) {
    g_err[0] = 0;
    if (!fmt_ok(format)) return fail(FP8_ERR_ENUM, "fp8_quantize_row_col: unknown format %d", format);
    if (flags & ~FP8_POW2_SCALE) return fail(FP8_ERR_ENUM, "fp8_quantize_row_col: flags=%d has unknown bits", flags);
    if (int rc = check_bf16("fp8_quantize_row_col", x, rows, cols, ld)) return rc;
    if (int rc = check_q_out("fp8_quantize_row_col(q_row)", q_row, rows, cols, ld_row, 0)) return rc;
    if (int rc = check_q_out("fp8_quantize_row_col(q_col_t)", q_col_t, rows, cols, ld_col_t, 1)) return rc;
    if ((rows > 0 && !scale_row) || (cols > 0 && !scale_col)) return fail(FP8_ERR_NULL, "fp8_quantize_row_col: scale output is NULL");
    if (!aligned(scale_row, 4) || !aligned(scale_col, 4)) return fail(FP8_ERR_ALIGN, "fp8_quantize_row_col: scales not 4-byte aligned");
    return quantize_row_col_impl(x, rows, cols, ld, format, flags, q_row, ld_row, scale_row, q_col_t, ld_col_t, scale_col,
                                 static_cast<hipStream_t>(stream));
}

int fp8_scaled_mm(const uint8_t* a, int64_t lda, int fmt_a, const float* scale_a, int gran_a, const uint8_t* b,
                  int64_t ldb, int fmt_b, const float* scale_b, int gran_b, int64_t M, int64_t N, int64_t K,
                  void* out, int64_t ld_out, int flags, void* stream) {
    g_err[0] = 0;
    if (!fmt_ok(fmt_a) || !fmt_ok(fmt_b)) return fail(FP8_ERR_ENUM, "fp8_scaled_mm: unknown format");
    if ((gran_a != FP8_TENSOR && gran_a != FP8_ROW) || (gran_b != FP8_TENSOR && gran_b != FP8_ROW))
        return fail(FP8_ERR_ENUM, "fp8_scaled_mm: granularity must be FP8_TENSOR or FP8_ROW");
    if (flags & ~(FP8_OUT_FP32 | FP8_EPILOGUE_SIGMOID)) return fail(FP8_ERR_ENUM, "fp8_scaled_mm: flags=%d has unknown bits", flags);
    if ((flags & FP8_EPILOGUE_SIGMOID) && (flags & FP8_OUT_FP32))
        return fail(FP8_ERR_ENUM, "fp8_scaled_mm: the sigmoid epilogue writes bfloat16 (not with FP8_OUT_FP32)");
    if (M < 0 || N < 0 || K < 0 || M > kMaxDim || N > kMaxDim || K > kMaxDim)
        return fail(FP8_ERR_SHAPE, "fp8_scaled_mm: M=%lld N=%lld K=%lld out of range", (long long)M, (long long)N, (long long)K);
    if (K % 16 != 0) return fail(FP8_ERR_SHAPE, "fp8_scaled_mm: K=%lld must be a multiple of 16", (long long)K);
    if (lda < K || ldb < K || ld_out < N) return fail(FP8_ERR_SHAPE, "fp8_scaled_mm: leading dimension too small");
    if (M > 0 && N > 0) {
        if (!out || !scale_a || !scale_b || (K > 0 && (!a || !b))) return fail(FP8_ERR_NULL, "fp8_scaled_mm: NULL pointer");
        if (!aligned(a, 16) || !aligned(b, 16) || !aligned(out, 16))
            return fail(FP8_ERR_ALIGN, "fp8_scaled_mm: a, b and out must be 16-byte aligned");
        if (lda % 16 != 0 || ldb % 16 != 0) return fail(FP8_ERR_ALIGN, "fp8_scaled_mm: lda and ldb must be multiples of 16");
        const int64_t out_align = (flags & FP8_OUT_FP32) ? 4 : 8;
        if (ld_out % out_align != 0)
            return fail(FP8_ERR_ALIGN, "fp8_scaled_mm: ld_out=%lld must be a multiple of %lld", (long long)ld_out, (long long)out_align);
        if (!aligned(scale_a, 4) || !aligned(scale_b, 4)) return fail(FP8_ERR_ALIGN, "fp8_scaled_mm: scales not 4-byte aligned");
    }
    if (flags & FP8_EPILOGUE_SIGMOID) {
        // the fused activation lives in the LDS-DMA kernel's epilogue, which handles every shape
        if (!fp8k::gemm_fp8_snake_fits(lda, ldb))
            return fail(FP8_ERR_SHAPE, "fp8_scaled_mm: the sigmoid epilogue needs lda, ldb below 2^23");
        FP8_TRY(fp8k::launch_gemm_fp8_snake(a, lda, fmt_a, scale_a, gran_a == FP8_ROW, b, ldb, fmt_b, scale_b, gran_b == FP8_ROW,
                                            M, N, K, out, ld_out, 0, static_cast<hipStream_t>(stream), 1));
        return FP8_OK;
    }
    FP8_TRY(fp8k::launch_gemm_fp8(a, lda, fmt_a, scale_a, gran_a == FP8_ROW, b, ldb, fmt_b, scale_b, gran_b == FP8_ROW,
                                  M, N, K, out, ld_out, (flags & FP8_OUT_FP32) ? 1 : 0, static_cast<hipStream_t>(stream)));
    return FP8_OK;
}

size_t fp8_linear_workspace_bytes(int64_t M, int64_t K, int64_t N, const fp8_recipe* recipe, int bwd) {
    g_err[0] = 0;
    if (check_recipe("fp8_linear_workspace_bytes", recipe)) return 0;
    if (check_linear_dims("fp8_linear_workspace_bytes", M, K, N, bwd != 0)) return 0;
    size_t t = bwd ? plan_bwd(M, K, N, recipe->gran).total : plan_fwd(M, K, N, recipe->gran).total;
    // shared workspace: the backward's layout (it holds the saved copies), then the forward's own buffers
    if (recipe->flags & FP8_SAVE_FOR_BWD) {
        if (check_linear_dims("fp8_linear_workspace_bytes", M, K, N, true)) return 0;
        t = plan_bwd(M, K, N, recipe->gran).total + plan_fwd(M, K, N, recipe->gran).total;
    }
    return t ? t : 256;
}

int fp8_linear_fwd(const void* x, const void* w, int64_t M, int64_t K, int64_t N, const fp8_recipe* recipe, void* y,
                   void* workspace, size_t workspace_bytes, void* stream) {
    g_err[0] = 0;
    if (int rc = check_recipe("fp8_linear_fwd", recipe)) return rc;
    if (int rc = check_linear_dims("fp8_linear_fwd", M, K, N, false)) return rc;
    if (int rc = check_bf16("fp8_linear_fwd(x)", x, M, K, K)) return rc;
    if (int rc = check_bf16("fp8_linear_fwd(w)", w, N, K, K)) return rc;
    if (M == 0 || N == 0) return FP8_OK;
    if (!y || !workspace) return fail(FP8_ERR_NULL, "fp8_linear_fwd: y or workspace is NULL");
    if (!aligned(y, 16) || !aligned(workspace, 256)) return fail(FP8_ERR_ALIGN, "fp8_linear_fwd: y (16) / workspace (256) misaligned");
    const FwdPlan p = plan_fwd(M, K, N, recipe->gran);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (recipe->flags & FP8_SAVE_FOR_BWD) {
        // The copies of X and W that the backward needs do not depend on the gradient, so they are made
        // here, from the same read as the forward's: the transposed codes and their scales go where the
        // backward's plan expects them.  Tensorwise: one conversion into both layouts.  Rowwise: the
        // rowwise codes for this GEMM plus the per-column (transposed) ones for dX / dW.
        if (int rc = check_linear_dims("fp8_linear_fwd", M, K, N, true)) return rc;
        const BwdPlan b = plan_bwd(M, K, N, recipe->gran);
        if (workspace_bytes < b.total + p.total)
            return fail(FP8_ERR_WORKSPACE, "fp8_linear_fwd: workspace %zu < %zu bytes", workspace_bytes, b.total + p.total);
        if ((K + 127) / 128 > 65535) return fail(FP8_ERR_SHAPE, "fp8_linear_fwd: K too large");
        uint8_t* wsb = static_cast<uint8_t*>(workspace);
        uint8_t* wsf = wsb + b.total;
        const int fl = recipe->flags & FP8_POW2_SCALE;
        float *sxt = reinterpret_cast<float*>(wsb + b.sxt), *swt = reinterpret_cast<float*>(wsb + b.swt);
        const int64_t Mp = pad16(M);
        if (Mp != M) FP8_TRY(fp8k::launch_fill_u32(reinterpret_cast<uint32_t*>(wsb + b.xt), K * Mp / 4, 0u, st));   // zero codes in the pad columns of X^T
        if (recipe->gran == FP8_TENSOR) {
            float* part = reinterpret_cast<float*>(wsf + p.part);
            bool pair_done = false;
            if (recipe->fmt_x == recipe->fmt_w && K > 0) {   // both tensors in two launches
                const fp8k::TensorOperand ox{x, M, wsb + b.xt, Mp, wsf + p.xq, K, sxt, part};
                const fp8k::TensorOperand ow{w, N, wsb + b.wt, N, wsf + p.wq, K, swt, part + fp8k::TENSOR_PARTIALS};
                const hipError_t e = fp8k::launch_quant_tensor_pair(ox, ow, K, recipe->fmt_x, fl, 1, st);
                if (e == hipSuccess) pair_done = true;
                else if (e != hipErrorNotSupported) return hip_fail(e, "quant_tensor_pair");
            }
            if (!pair_done) {
                if (int rc = quantize_impl(x, M, K, K, FP8_TENSOR, recipe->fmt_x, fl | FP8_TRANSPOSE_OUT, wsb + b.xt, Mp, wsf + p.xq, K, sxt, st, part)) return rc;
                if (int rc = quantize_impl(w, N, K, K, FP8_TENSOR, recipe->fmt_w, fl | FP8_TRANSPOSE_OUT, wsb + b.wt, N, wsf + p.wq, K, swt, st, part)) return rc;
            }
            FP8_TRY(fp8k::launch_gemm_fp8(wsf + p.xq, K, recipe->fmt_x, sxt, 0, wsf + p.wq, K, recipe->fmt_w, swt, 0, M, N, K, y, N, 0, st));
            return FP8_OK;
        }
        float *sx = reinterpret_cast<float*>(wsf + p.sx), *sw = reinterpret_cast<float*>(wsf + p.sw);
        bool done = false;
        if (!(recipe->flags & FP8_GRAD_WEIGHT_HP) && recipe->fmt_x == recipe->fmt_w) {
            // X and W the same way: twin launches, three (small tensors: two) instead of six
            const fp8k::RowColOperand ox{x, M, K, wsf + p.xq, K, sx, wsb + b.xt, Mp, sxt, wsf + p.fold_x};
            const fp8k::RowColOperand ow{w, N, K, wsf + p.wq, K, sw, wsb + b.wt, N, swt, wsf + p.fold_w};
            const hipError_t e = fp8k::launch_quant_row_col_pair(ox, &ow, K, recipe->fmt_x, fl, st);
            if (e == hipSuccess) done = true;
            else if (e != hipErrorNotSupported) return hip_fail(e, "quant_row_col_pair");
        }
        if (!done) {
            if (recipe->flags & FP8_GRAD_WEIGHT_HP) {   // dW will come from the bfloat16 X: no fp8 copy of X to keep
                if (int rc = quantize_impl(x, M, K, K, FP8_ROW, recipe->fmt_x, fl, wsf + p.xq, K, nullptr, 0, sx, st)) return rc;
            } else {
                if (int rc = quantize_row_col_impl(x, M, K, K, recipe->fmt_x, fl, wsf + p.xq, K, sx, wsb + b.xt, Mp, sxt, st)) return rc;
            }
            if (int rc = quantize_row_col_impl(w, N, K, K, recipe->fmt_w, fl, wsf + p.wq, K, sw, wsb + b.wt, N, swt, st)) return rc;
        }
        FP8_TRY(fp8k::launch_gemm_fp8(wsf + p.xq, K, recipe->fmt_x, sx, 1, wsf + p.wq, K, recipe->fmt_w, sw, 1, M, N, K, y, N, 0, st));
        return FP8_OK;
    }
    if (workspace_bytes < p.total)
        return fail(FP8_ERR_WORKSPACE, "fp8_linear_fwd: workspace %zu < %zu bytes", workspace_bytes, p.total);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    uint8_t *xq = ws + p.xq, *wq = ws + p.wq;
    float *sx = reinterpret_cast<float*>(ws + p.sx), *sw = reinterpret_cast<float*>(ws + p.sw);
    const int g = recipe->gran, fl = recipe->flags & FP8_POW2_SCALE;
    float* part = reinterpret_cast<float*>(ws + p.part);
    bool pair_done = false;
    if (g == FP8_ROW && recipe->fmt_x == recipe->fmt_w && K > 0) {   // X and W in one launch
        const hipError_t e = fp8k::launch_quant_row_pair(x, M, K, xq, K, sx, w, N, K, wq, K, sw, K, recipe->fmt_x, fl, st);
        if (e == hipSuccess) pair_done = true;
        else if (e != hipErrorNotSupported) return hip_fail(e, "quant_row_pair");
    }
    if (g == FP8_TENSOR && recipe->fmt_x == recipe->fmt_w && K > 0) {
        const fp8k::TensorOperand ox{x, M, xq, K, nullptr, 0, sx, part}, ow{w, N, wq, K, nullptr, 0, sw, part + fp8k::TENSOR_PARTIALS};
        const hipError_t e = fp8k::launch_quant_tensor_pair(ox, ow, K, recipe->fmt_x, fl, 0, st);
        if (e == hipSuccess) pair_done = true;
        else if (e != hipErrorNotSupported) return hip_fail(e, "quant_tensor_pair");
    }
    if (!pair_done) {
        if (int rc = quantize_impl(x, M, K, K, g, recipe->fmt_x, fl, xq, K, nullptr, 0, sx, st, part)) return rc;
        if (int rc = quantize_impl(w, N, K, K, g, recipe->fmt_w, fl, wq, K, nullptr, 0, sw, st, part)) return rc;
    }
    FP8_TRY(fp8k::launch_gemm_fp8(xq, K, recipe->fmt_x, sx, g == FP8_ROW, wq, K, recipe->fmt_w, sw, g == FP8_ROW, M, N, K,
                                  y, N, 0, st));
    return FP8_OK;
}

int fp8_linear_bwd(const void* dy, const void* x, const void* w, int64_t M, int64_t K, int64_t N,
                   const fp8_recipe* recipe, void* dx, void* dw, void* workspace, size_t workspace_bytes,
                   void* stream) {
    g_err[0] = 0;
    if (int rc = check_recipe("fp8_linear_bwd", recipe)) return rc;
    if (int rc = check_linear_dims("fp8_linear_bwd", M, K, N, true)) return rc;
    if (int rc = check_bf16("fp8_linear_bwd(dy)", dy, M, N, N)) return rc;
    const bool saved = (recipe->flags & FP8_SAVE_FOR_BWD) != 0;   // codes of X and W left by the forward
    if (dw && (!saved || (recipe->flags & FP8_GRAD_WEIGHT_HP))) if (int rc = check_bf16("fp8_linear_bwd(x)", x, M, K, K)) return rc;
    if (dx && !saved) if (int rc = check_bf16("fp8_linear_bwd(w)", w, N, K, K)) return rc;
    if (M == 0 || N == 0 || K == 0 || (!dx && !dw)) return FP8_OK;
    if (!workspace) return fail(FP8_ERR_NULL, "fp8_linear_bwd: workspace is NULL");
    if (!aligned(dx, 16) || !aligned(dw, 16) || !aligned(workspace, 256))
        return fail(FP8_ERR_ALIGN, "fp8_linear_bwd: dx, dw (16) / workspace (256) misaligned");
    if ((K + 127) / 128 > 65535 || (N + 127) / 128 > 65535) return fail(FP8_ERR_SHAPE, "fp8_linear_bwd: K or N too large");
    const BwdPlan p = plan_bwd(M, K, N, recipe->gran);
    if (workspace_bytes < p.total + (saved ? plan_fwd(M, K, N, recipe->gran).total : 0))
        return fail(FP8_ERR_WORKSPACE, "fp8_linear_bwd: workspace %zu < %zu bytes", workspace_bytes,
                    p.total + (saved ? plan_fwd(M, K, N, recipe->gran).total : 0));
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    uint8_t *gq = ws + p.gq, *gqt = ws + p.gqt, *wt = ws + p.wt, *xt = ws + p.xt;
    float *sg = reinterpret_cast<float*>(ws + p.sg), *sgt = reinterpret_cast<float*>(ws + p.sgt);
    float *swt = reinterpret_cast<float*>(ws + p.swt), *sxt = reinterpret_cast<float*>(ws + p.sxt);
    const int fl = recipe->flags & FP8_POW2_SCALE;
    const int T = FP8_TRANSPOSE_OUT;

    if (dw && (recipe->flags & FP8_GRAD_WEIGHT_HP)) {
        // dW from the unquantized tensors on the bfloat16 matrix cores; the FP8 part below then
        // only has dX left to do (and quantizes dY along N only)
        FP8_TRY(fp8k::launch_gemm_bf16_at_b(dy, N, x, K, N, K, M, dw, K, st));
        dw = nullptr;
        if (!dx) return FP8_OK;
    }
    const int64_t Mp = pad16(M);
    if (dw && Mp != M) {   // zero codes in the pad columns of dY^T and (unless the forward left it) X^T
        FP8_TRY(fp8k::launch_fill_u32(reinterpret_cast<uint32_t*>(gqt), N * Mp / 4, 0u, st));
        if (!saved) FP8_TRY(fp8k::launch_fill_u32(reinterpret_cast<uint32_t*>(xt), K * Mp / 4, 0u, st));
    }

    if (recipe->gran == FP8_TENSOR) {
        // one scale per tensor; dY is converted once into both layouts
        float* part = reinterpret_cast<float*>(ws + p.part);
        uint8_t* plain = dx ? gq : nullptr;
        if (dw) {
            if (int rc = quantize_impl(dy, M, N, N, FP8_TENSOR, recipe->fmt_dy, fl | T, gqt, Mp, plain, N, sg, st, part)) return rc;
        } else {
            if (int rc = quantize_impl(dy, M, N, N, FP8_TENSOR, recipe->fmt_dy, fl, gq, N, nullptr, 0, sg, st, part)) return rc;
        }
        bool pair_done = false;
        if (dx && dw && !saved && recipe->fmt_w == recipe->fmt_x) {   // W and X in two launches
            const fp8k::TensorOperand ow{w, N, wt, N, nullptr, 0, swt, part}, ox{x, M, xt, Mp, nullptr, 0, sxt, part + fp8k::TENSOR_PARTIALS};
            const hipError_t e = fp8k::launch_quant_tensor_pair(ow, ox, K, recipe->fmt_w, fl, 1, st);
            if (e == hipSuccess) pair_done = true;
            else if (e != hipErrorNotSupported) return hip_fail(e, "quant_tensor_pair");
        }
        if (dx && !saved && !pair_done)
            if (int rc = quantize_impl(w, N, K, K, FP8_TENSOR, recipe->fmt_w, fl | T, wt, N, nullptr, 0, swt, st, part)) return rc;
        if (dw && !saved && !pair_done)
            if (int rc = quantize_impl(x, M, K, K, FP8_TENSOR, recipe->fmt_x, fl | T, xt, Mp, nullptr, 0, sxt, st, part)) return rc;
        return grad_gemms(recipe, 0, gq, sg, wt, swt, gqt, sg, xt, sxt, M, Mp, K, N, dx, dw, st);
    }
    // rowwise: every operand re-quantized along the contraction axis of its GEMM
    // (dX = dY W contracts over N, dW = dY^T X over M).  All quantizations first,
    // then the GEMMs back to back.
    const bool both = dx && dw;
    if (both && !saved && recipe->fmt_w == recipe->fmt_x) {
        // all three tensors in five launches: dY's rowwise pass (which also gathers its column maxima), the column
        // maxima of W and X together, one launch for every column scale, two for the transposing casts
        const fp8k::RowColOperand og{dy, M, N, gq, N, sg, gqt, Mp, sgt, ws + p.fold_g};
        const fp8k::ColOperand ow{w, N, K, wt, N, swt, ws + p.fold_w}, ox{x, M, K, xt, Mp, sxt, ws + p.fold_x};
        const hipError_t e = fp8k::launch_quant_bwd_rowwise(og, N, recipe->fmt_dy, ow, ox, K, recipe->fmt_w, fl, st);
        if (e == hipSuccess) return grad_gemms(recipe, 1, gq, sg, wt, swt, gqt, sgt, xt, sxt, M, Mp, K, N, dx, dw, st);
        if (e != hipErrorNotSupported) return hip_fail(e, "quant_bwd_rowwise");
    }
    if (both) {   // dY along N (rows) and along M (columns, transposed) from two reads instead of three
        const fp8k::RowColOperand og{dy, M, N, gq, N, sg, gqt, Mp, sgt, ws + p.fold_g};
        const hipError_t e = fp8k::launch_quant_row_col_pair(og, nullptr, N, recipe->fmt_dy, fl, st);
        if (e == hipErrorNotSupported) {
            if (int rc = quantize_row_col_impl(dy, M, N, N, recipe->fmt_dy, fl, gq, N, sg, gqt, Mp, sgt, st)) return rc;
        } else if (e != hipSuccess) {
            return hip_fail(e, "quant_row_col");
        }
    } else if (dx) {
        if (int rc = quantize_impl(dy, M, N, N, FP8_ROW, recipe->fmt_dy, fl, gq, N, nullptr, 0, sg, st)) return rc;
    } else {
        if (int rc = quantize_impl(dy, M, N, N, FP8_COL, recipe->fmt_dy, fl | T, gqt, Mp, nullptr, 0, sgt, st)) return rc;
    }
    if (dx && !saved)
        if (int rc = quantize_impl(w, N, K, K, FP8_COL, recipe->fmt_w, fl | T, wt, N, nullptr, 0, swt, st)) return rc;
    if (dw && !saved)
        if (int rc = quantize_impl(x, M, K, K, FP8_COL, recipe->fmt_x, fl | T, xt, Mp, nullptr, 0, sxt, st)) return rc;
    return grad_gemms(recipe, 1, gq, sg, wt, swt, gqt, sgt, xt, sxt, M, Mp, K, N, dx, dw, st);
}

namespace {
// shapes and recipes for which the gradient through the sigmoid is quantized without being materialised
bool sigmoid_bwd_fused(int64_t M, int64_t N, const fp8_recipe* r) {
    return r->gran == FP8_ROW && !(r->flags & FP8_GRAD_WEIGHT_HP) && N % 8 == 0 && N / 8 >= 64 && N / 8 <= 4096 && M >= 1024 &&
           M % 16 == 0;   // (a token count off the 16-byte grid takes the padded buffers of fp8_linear_bwd)
}
}  // namespace

size_t fp8_linear_bwd_sigmoid_workspace_bytes(int64_t M, int64_t K, int64_t N, const fp8_recipe* recipe) {
    const size_t base = fp8_linear_workspace_bytes(M, K, N, recipe, 1);
    if (base == 0) return 0;
    return sigmoid_bwd_fused(M, N, recipe) ? base : align_up(base, 256) + align_up((size_t)M * (size_t)N * 2, 256);
}

int fp8_linear_bwd_sigmoid(const void* dy, const void* y, const void* x, const void* w, int64_t M, int64_t K, int64_t N,
                           const fp8_recipe* recipe, void* dx, void* dw, void* workspace, size_t workspace_bytes,
                           void* stream) {
    g_err[0] = 0;
    const char* fn = "fp8_linear_bwd_sigmoid";
    if (int rc = check_recipe(fn, recipe)) return rc;
    if (int rc = check_linear_dims(fn, M, K, N, true)) return rc;
    if (int rc = check_bf16("fp8_linear_bwd_sigmoid(dy)", dy, M, N, N)) return rc;
    if (int rc = check_bf16("fp8_linear_bwd_sigmoid(y)", y, M, N, N)) return rc;
    if (M == 0 || N == 0 || K == 0 || (!dx && !dw)) return FP8_OK;
    if (!workspace) return fail(FP8_ERR_NULL, "%s: workspace is NULL", fn);
    if (!aligned(workspace, 256)) return fail(FP8_ERR_ALIGN, "%s: workspace not 256-byte aligned", fn);
    const size_t need = fp8_linear_bwd_sigmoid_workspace_bytes(M, K, N, recipe);
    if (need == 0) return FP8_ERR_SHAPE;
    if (workspace_bytes < need) return fail(FP8_ERR_WORKSPACE, "%s: workspace %zu < %zu bytes", fn, workspace_bytes, need);
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    const size_t base = fp8_linear_workspace_bytes(M, K, N, recipe, 1);
    if (!sigmoid_bwd_fused(M, N, recipe)) {
        // small or unusual shapes, other recipes: dz = dy * y * (1 - y) is written out once and the ordinary
        // backward runs on it
        uint8_t* dz = ws + align_up(base, 256);
        FP8_TRY(fp8k::launch_sigmoid_bwd(dy, y, M * N, dz, st));
        return fp8_linear_bwd(dz, x, w, M, K, N, recipe, dx, dw, workspace, base, stream);
    }
    // rowwise: dz is formed inside the two quantization passes (never stored), then the usual products
    const bool saved = (recipe->flags & FP8_SAVE_FOR_BWD) != 0;
    if (dw && !saved) if (int rc = check_bf16("fp8_linear_bwd_sigmoid(x)", x, M, K, K)) return rc;
    if (dx && !saved) if (int rc = check_bf16("fp8_linear_bwd_sigmoid(w)", w, N, K, K)) return rc;
    if (!aligned(dx, 16) || !aligned(dw, 16)) return fail(FP8_ERR_ALIGN, "%s: dx, dw not 16-byte aligned", fn);
    if ((K + 127) / 128 > 65535 || (N + 127) / 128 > 65535) return fail(FP8_ERR_SHAPE, "%s: K or N too large", fn);
    const BwdPlan p = plan_bwd(M, K, N, recipe->gran);
    uint8_t *gq = ws + p.gq, *gqt = ws + p.gqt, *wt = ws + p.wt, *xt = ws + p.xt;
    float *sg = reinterpret_cast<float*>(ws + p.sg), *sgt = reinterpret_cast<float*>(ws + p.sgt);
    float *swt = reinterpret_cast<float*>(ws + p.swt), *sxt = reinterpret_cast<float*>(ws + p.sxt);
    const int fl = recipe->flags & FP8_POW2_SCALE;
    const int T = FP8_TRANSPOSE_OUT;
    hipError_t e = fp8k::launch_quant_row_col_sigmoid_bwd(dy, y, M, N, N, recipe->fmt_dy, fl, gq, N, sg, gqt, M, sgt, st);
    if (e == hipErrorNotSupported) return fail(FP8_ERR_SHAPE, "%s: shape not supported by the fused gradient quantization", fn);
    if (e != hipSuccess) return hip_fail(e, "quant_row_col_sigmoid_bwd");
    if (dx && !saved)
        if (int rc = quantize_impl(w, N, K, K, FP8_COL, recipe->fmt_w, fl | T, wt, N, nullptr, 0, swt, st)) return rc;
    if (dw && !saved)
        if (int rc = quantize_impl(x, M, K, K, FP8_COL, recipe->fmt_x, fl | T, xt, M, nullptr, 0, sxt, st)) return rc;
    return grad_gemms(recipe, 1, gq, sg, wt, swt, gqt, sgt, xt, sxt, M, M, K, N, dx, dw, st);
}

int fp8_grad_weight_hp(const void* dy, const void* x, int64_t M, int64_t K, int64_t N, void* dw, void* stream) {
    g_err[0] = 0;
    const char* fn = "fp8_grad_weight_hp";
    if (M < 0 || K < 0 || N < 0 || M > kMaxDim || K > kMaxDim || N > kMaxDim)
        return fail(FP8_ERR_SHAPE, "%s: M=%lld K=%lld N=%lld out of range", fn, (long long)M, (long long)K, (long long)N);
    if (K % 8 != 0 || N % 8 != 0) return fail(FP8_ERR_SHAPE, "%s: K=%lld and N=%lld must be multiples of 8", fn, (long long)K, (long long)N);
    if (int rc = check_bf16("fp8_grad_weight_hp(dy)", dy, M, N, N)) return rc;
    if (int rc = check_bf16("fp8_grad_weight_hp(x)", x, M, K, K)) return rc;
    if (N == 0 || K == 0) return FP8_OK;
    if (!dw) return fail(FP8_ERR_NULL, "%s: dw is NULL", fn);
    if (!aligned(dw, 16)) return fail(FP8_ERR_ALIGN, "%s: dw not 16-byte aligned", fn);
    FP8_TRY(fp8k::launch_gemm_bf16_at_b(dy, N, x, K, N, K, M, dw, K, static_cast<hipStream_t>(stream)));
    return FP8_OK;
}

size_t fp8_linear_prequantized_workspace_bytes(int64_t M, int64_t K) {
    g_err[0] = 0;
    if (M < 0 || K < 0 || M > kMaxDim || K > kMaxDim) {
        fail(FP8_ERR_SHAPE, "fp8_linear_prequantized_workspace_bytes: M=%lld K=%lld out of range", (long long)M, (long long)K);
        return 0;
    }
    return align_up((size_t)M * (size_t)K, 256) + align_up(sizeof(float) * (size_t)(M > 0 ? M : 1), 256) + 256;
}

namespace {
// validation and composition shared by fp8_linear_fwd_prequantized and its variant without a workspace argument
int linear_fwd_prequantized_impl(const char* fn, const void* x, int64_t M, int64_t K, int fmt_x, int gran_x, int flags,
                                 const uint8_t* wq, int64_t ldw, int fmt_w, const float* scale_w, int gran_w, int64_t N,
                                 void* y, int64_t ld_y, void* (*workspace_of)(size_t need, void* ctx, int* rc), void* ctx,
                                 void* stream) {
    if (!fmt_ok(fmt_x) || !fmt_ok(fmt_w)) return fail(FP8_ERR_ENUM, "%s: unknown fp8 format", fn);
    if ((gran_x != FP8_TENSOR && gran_x != FP8_ROW) || (gran_w != FP8_TENSOR && gran_w != FP8_ROW))
        return fail(FP8_ERR_ENUM, "%s: granularity must be FP8_TENSOR or FP8_ROW", fn);
    if (flags & ~FP8_POW2_SCALE) return fail(FP8_ERR_ENUM, "%s: flags=%d has unknown bits", fn, flags);
    if (M < 0 || K < 0 || N < 0 || M > kMaxDim || K > kMaxDim || N > kMaxDim)
        return fail(FP8_ERR_SHAPE, "%s: M=%lld K=%lld N=%lld out of range", fn, (long long)M, (long long)K, (long long)N);
    if (K % 16 != 0) return fail(FP8_ERR_SHAPE, "%s: K=%lld must be a multiple of 16", fn, (long long)K);
    if (ldw < K || ld_y < N) return fail(FP8_ERR_SHAPE, "%s: leading dimension too small", fn);
    if (int rc = check_bf16(fn, x, M, K, K)) return rc;
    if (M == 0 || N == 0) return FP8_OK;
    if (!y || !scale_w || (K > 0 && !wq)) return fail(FP8_ERR_NULL, "%s: NULL pointer", fn);
    if (!aligned(y, 16) || !aligned(wq, 16) || !aligned(scale_w, 4))
        return fail(FP8_ERR_ALIGN, "%s: y, wq (16) / scale_w (4) misaligned", fn);
    if (ldw % 16 != 0 || ld_y % 8 != 0) return fail(FP8_ERR_ALIGN, "%s: ldw %% 16 and ld_y %% 8 must be 0", fn);
    const size_t need = fp8_linear_prequantized_workspace_bytes(M, K);
    int rc = FP8_OK;
    void* workspace = workspace_of(need, ctx, &rc);
    if (rc != FP8_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t* xq = static_cast<uint8_t*>(workspace);
    float* sx = reinterpret_cast<float*>(xq + align_up((size_t)M * (size_t)K, 256));
    // a few tokens: scales and codes of x are formed inside the product's launch (the workspace stays unused)
    const hipError_t fused = fp8k::launch_linear_skinny_fused(x, K, fmt_x, gran_x == FP8_ROW, flags & FP8_POW2_SCALE, wq, ldw, fmt_w,
                                                              scale_w, gran_w == FP8_ROW, M, N, K, y, ld_y, st);
    if (fused == hipSuccess) return FP8_OK;
    if (fused != hipErrorNotSupported) return hip_fail(fused, "launch_linear_skinny_fused");
    if (int rq = quantize_impl(x, M, K, K, gran_x, fmt_x, flags, xq, K, nullptr, 0, sx, st)) return rq;
    FP8_TRY(fp8k::launch_gemm_fp8(xq, K, fmt_x, sx, gran_x == FP8_ROW, wq, ldw, fmt_w, scale_w, gran_w == FP8_ROW, M, N, K, y,
                                  ld_y, 0, st));
    return FP8_OK;
}

struct CallerWorkspace { void* p; size_t bytes; };
void* caller_workspace(size_t need, void* ctx, int* rc) {
    const CallerWorkspace* w = static_cast<const CallerWorkspace*>(ctx);
    if (!w->p) { *rc = fail(FP8_ERR_NULL, "fp8_linear_fwd_prequantized: workspace is NULL"); return nullptr; }
    if (!aligned(w->p, 256)) { *rc = fail(FP8_ERR_ALIGN, "fp8_linear_fwd_prequantized: workspace not 256-byte aligned"); return nullptr; }
    if (w->bytes < need) { *rc = fail(FP8_ERR_WORKSPACE, "fp8_linear_fwd_prequantized: workspace %zu < %zu bytes", w->bytes, need); return nullptr; }
    return w->p;
}
}  // namespace

int fp8_linear_fwd_prequantized(const void* x, int64_t M, int64_t K, int fmt_x, int gran_x, int flags, const uint8_t* wq,
                                int64_t ldw, int fmt_w, const float* scale_w, int gran_w, int64_t N, void* y,
                                int64_t ld_y, void* workspace, size_t workspace_bytes, void* stream) {
    g_err[0] = 0;
    CallerWorkspace w{workspace, workspace_bytes};
    return linear_fwd_prequantized_impl("fp8_linear_fwd_prequantized", x, M, K, fmt_x, gran_x, flags, wq, ldw, fmt_w, scale_w,
                                        gran_w, N, y, ld_y, caller_workspace, &w, stream);
}

namespace {
// per device: the address of that device's copy of `scratch` (resolved once, with the device current)
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mu;

void* static_workspace(size_t need, void*, int* rc) {
    const char* fn = "fp8_linear_fwd_prequantized_static";
    if (need > (size_t)FP8_STATIC_SCRATCH_BYTES) {
        *rc = fail(FP8_ERR_WORKSPACE, "%s: M x K needs %zu bytes of scratch, the static buffer holds %zu", fn, need,
                   (size_t)FP8_STATIC_SCRATCH_BYTES);
        return nullptr;
    }
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { *rc = hip_fail(e, "hipGetDevice"); return nullptr; }
    if (dev < 0 || dev >= kMaxDevices) { *rc = fail(FP8_ERR_HIP, "%s: device index %d out of range", fn, dev); return nullptr; }
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lock(g_scratch_mu);
        p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
        if (!p) {
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !p) { *rc = hip_fail(e, "hipGetSymbolAddress(scratch)"); return nullptr; }
            g_scratch_ptr[dev].store(p, std::memory_order_release);
        }
    }
    return p;
}
}  // namespace

int fp8_linear_fwd_prequantized_static(const void* x, int64_t M, int64_t K, int fmt_x, int gran_x, int flags,
                                       const uint8_t* wq, int64_t ldw, int fmt_w, const float* scale_w, int gran_w,
                                       int64_t N, void* y, int64_t ld_y, void* stream) {
    g_err[0] = 0;
    return linear_fwd_prequantized_impl("fp8_linear_fwd_prequantized_static", x, M, K, fmt_x, gran_x, flags, wq, ldw, fmt_w,
                                        scale_w, gran_w, N, y, ld_y, static_workspace, nullptr, stream);
}

int fp8_layernorm_quantize(const void* x, int64_t rows, int64_t cols, int64_t ld, const void* gamma, const void* beta,
                           double eps, int format, int flags, void* h_out, int64_t ld_h, uint8_t* q_out, int64_t ld_q,
                           float* scale_out, float* mean_out, float* rstd_out, void* stream) {
    g_err[0] = 0;
    const char* fn = "fp8_layernorm_quantize";
    if (!fmt_ok(format)) return fail(FP8_ERR_ENUM, "%s: unknown format %d", fn, format);
    if (flags & ~FP8_POW2_SCALE) return fail(FP8_ERR_ENUM, "%s: flags=%d has unknown bits", fn, flags);
    if (int rc = check_bf16(fn, x, rows, cols, ld)) return rc;
    if (cols % 8 != 0 || cols > 16384)
        return fail(FP8_ERR_SHAPE, "%s: cols=%lld must be a multiple of 8 and at most 16384", fn, (long long)cols);
    if (!(eps >= 0.0)) return fail(FP8_ERR_SHAPE, "%s: eps must be non-negative", fn);
    if (int rc = check_q_out(fn, q_out, rows, cols, ld_q, 0)) return rc;
    if (rows > 0 && cols > 0) {
        if (!gamma || !scale_out) return fail(FP8_ERR_NULL, "%s: gamma or scale_out is NULL", fn);
        if (!aligned(gamma, 16) || !aligned(beta, 16) || !aligned(h_out, 16))
            return fail(FP8_ERR_ALIGN, "%s: gamma, beta and h_out must be 16-byte aligned", fn);
        if (h_out && (ld_h < cols || ld_h % 8 != 0)) return fail(FP8_ERR_SHAPE, "%s: ld_h=%lld must be >= cols and a multiple of 8", fn, (long long)ld_h);
        if (!aligned(scale_out, 4) || !aligned(mean_out, 4) || !aligned(rstd_out, 4))
            return fail(FP8_ERR_ALIGN, "%s: scale_out, mean_out, rstd_out not 4-byte aligned", fn);
    }
    FP8_TRY(fp8k::launch_layernorm_quant_row(x, rows, cols, ld, gamma, beta, eps, format, flags & FP8_POW2_SCALE, h_out, ld_h,
                                             q_out, ld_q, scale_out, mean_out, rstd_out, static_cast<hipStream_t>(stream)));
    return FP8_OK;
}

namespace {
// An array of E8M0 scale bytes, one per block of 32: `rows` scale rows of `blocks` bytes.  ld_e >= 0: plain rows of
// ld_e bytes (a multiple of 4, 4-byte aligned).  ld_e < 0: slabs of sixteen blocks, [blocks / 16][-ld_e][16 bytes]
// (blocks a multiple of 16, -ld_e >= rows, 16-byte aligned): the layout that the 256 x 256 product kernel reads as
// whole 16-byte pieces.
int check_e8m0(const char* fn, const void* e, int64_t rows, int64_t blocks, int64_t ld_e) {
    if (ld_e < 0) {
        if (blocks % 16 != 0)
            return fail(FP8_ERR_SHAPE, "%s: scale slabs (negative ld_e) need a multiple of 512 elements along the blocks, got %lld blocks", fn, (long long)blocks);
        if (-ld_e < rows) return fail(FP8_ERR_SHAPE, "%s: scale slabs of %lld rows for %lld rows of scales", fn, (long long)-ld_e, (long long)rows);
        if (-ld_e > kMaxDim || -ld_e * blocks >= ((int64_t)1 << 31))
            return fail(FP8_ERR_SHAPE, "%s: scale slabs of %lld rows x %lld blocks exceed 2^31 bytes", fn, (long long)-ld_e, (long long)blocks);
        if (rows > 0 && blocks > 0 && !e) return fail(FP8_ERR_NULL, "%s: scale array is NULL", fn);
        if (!aligned(e, 16)) return fail(FP8_ERR_ALIGN, "%s: scale slabs not 16-byte aligned", fn);
        return FP8_OK;
    }
    if (ld_e < blocks || ld_e % 4 != 0)
        return fail(FP8_ERR_SHAPE, "%s: ld_e=%lld must be >= %lld (one byte per block of 32) and a multiple of 4", fn, (long long)ld_e, (long long)blocks);
    if (rows > 0 && blocks > 0 && !e) return fail(FP8_ERR_NULL, "%s: scale array is NULL", fn);
    if (!aligned(e, 4)) return fail(FP8_ERR_ALIGN, "%s: scale array not 4-byte aligned", fn);
    return FP8_OK;
}
}  // namespace

int fp8_mx_quantize(const void* x, int64_t rows, int64_t cols, int64_t ld, int format, uint8_t* q_out, int64_t ld_q,
                    uint8_t* e8m0_out, int64_t ld_e, void* stream) {
    g_err[0] = 0;
    const char* fn = "fp8_mx_quantize";
    if (!fmt_ok(format)) return fail(FP8_ERR_ENUM, "%s: unknown format %d", fn, format);
    if (int rc = check_bf16(fn, x, rows, cols, ld)) return rc;
    if (cols % 32 != 0) return fail(FP8_ERR_SHAPE, "%s: cols=%lld must be a multiple of the block size 32", fn, (long long)cols);
    if (int rc = check_q_out(fn, q_out, rows, cols, ld_q, 0)) return rc;
    if (int rc = check_e8m0(fn, e8m0_out, rows, cols / 32, ld_e)) return rc;
    FP8_TRY(fp8k::launch_mx_quant(x, rows, cols, ld, format, q_out, ld_q, e8m0_out, ld_e, static_cast<hipStream_t>(stream)));
    return FP8_OK;
}

int fp8_mx_quantize_t(const void* x, int64_t rows, int64_t cols, int64_t ld, int format, uint8_t* qt_out, int64_t ld_q,
                      uint8_t* e8m0_t_out, int64_t ld_e, void* stream) {
    g_err[0] = 0;
    const char* fn = "fp8_mx_quantize_t";
    if (!fmt_ok(format)) return fail(FP8_ERR_ENUM, "%s: unknown format %d", fn, format);
    if (int rc = check_bf16(fn, x, rows, cols, ld)) return rc;
    if (rows % 32 != 0) return fail(FP8_ERR_SHAPE, "%s: rows=%lld must be a multiple of the block size 32", fn, (long long)rows);
    if (int rc = check_q_out(fn, qt_out, cols, rows, ld_q, 0)) return rc;
    if (int rc = check_e8m0(fn, e8m0_t_out, cols, rows / 32, ld_e)) return rc;
    FP8_TRY(fp8k::launch_mx_quant_t(x, rows, cols, ld, format, qt_out, ld_q, e8m0_t_out, ld_e, nullptr, 0, nullptr, 0,
                                    static_cast<hipStream_t>(stream)));
    return FP8_OK;
}

int fp8_mx_quantize_row_col(const void* x, int64_t rows, int64_t cols, int64_t ld, int format, uint8_t* q_row,
                            int64_t ld_row, uint8_t* e_row, int64_t ld_er, uint8_t* q_col_t, int64_t ld_col_t,
                            uint8_t* e_col_t, int64_t ld_ec, void* stream) {
    g_err[0] = 0;
    const char* fn = "fp8_mx_quantize_row_col";
    if (!fmt_ok(format)) return fail(FP8_ERR_ENUM, "%s: unknown format %d", fn, format);
    if (int rc = check_bf16(fn, x, rows, cols, ld)) return rc;
    if (rows % 32 != 0 || cols % 32 != 0)
        return fail(FP8_ERR_SHAPE, "%s: rows=%lld and cols=%lld must be multiples of the block size 32", fn, (long long)rows, (long long)cols);
    if (int rc = check_q_out("fp8_mx_quantize_row_col(q_row)", q_row, rows, cols, ld_row, 0)) return rc;
    if (int rc = check_q_out("fp8_mx_quantize_row_col(q_col_t)", q_col_t, cols, rows, ld_col_t, 0)) return rc;
    if (int rc = check_e8m0("fp8_mx_quantize_row_col(e_row)", e_row, rows, cols / 32, ld_er)) return rc;
    if (int rc = check_e8m0("fp8_mx_quantize_row_col(e_col_t)", e_col_t, cols, rows / 32, ld_ec)) return rc;
    FP8_TRY(fp8k::launch_mx_quant_t(x, rows, cols, ld, format, q_col_t, ld_col_t, e_col_t, ld_ec, q_row, ld_row, e_row, ld_er,
                                    static_cast<hipStream_t>(stream)));
    return FP8_OK;
}

int fp8_mx_scaled_mm(const uint8_t* a, int64_t lda, int fmt_a, const uint8_t* ea, int64_t ld_ea, const uint8_t* b,
                     int64_t ldb, int fmt_b, const uint8_t* eb, int64_t ld_eb, int64_t M, int64_t N, int64_t K, void* out,
                     int64_t ld_out, int flags, void* stream) {
    g_err[0] = 0;
    const char* fn = "fp8_mx_scaled_mm";
    if (!fmt_ok(fmt_a) || !fmt_ok(fmt_b)) return fail(FP8_ERR_ENUM, "%s: unknown format", fn);
    if (flags & ~FP8_OUT_FP32) return fail(FP8_ERR_ENUM, "%s: flags=%d has unknown bits", fn, flags);
    if (M < 0 || N < 0 || K < 0 || M > kMaxDim || N > kMaxDim || K > kMaxDim)
        return fail(FP8_ERR_SHAPE, "%s: M=%lld N=%lld K=%lld out of range", fn, (long long)M, (long long)N, (long long)K);
    if (K % 128 != 0) return fail(FP8_ERR_SHAPE, "%s: K=%lld must be a multiple of 128", fn, (long long)K);
    if (lda < K || ldb < K || ld_out < N) return fail(FP8_ERR_SHAPE, "%s: leading dimension too small", fn);
    if ((ld_ea < 0) != (ld_eb < 0)) return fail(FP8_ERR_SHAPE, "%s: scale slabs (negative ld_ea, ld_eb) for both operands or for neither", fn);
    if (ld_ea < 0 && !fp8k::gemm_fp8_snake_fits(lda, ldb))
        return fail(FP8_ERR_SHAPE, "%s: scale slabs need lda, ldb below 2^23", fn);
    if (M > 0 && N > 0) {
        if (int rc = check_e8m0("fp8_mx_scaled_mm(ea)", ea, K > 0 ? M : 0, K / 32, ld_ea)) return rc;
        if (int rc = check_e8m0("fp8_mx_scaled_mm(eb)", eb, K > 0 ? N : 0, K / 32, ld_eb)) return rc;
        if (!out || (K > 0 && (!a || !b))) return fail(FP8_ERR_NULL, "%s: NULL pointer", fn);
        if (!aligned(a, 16) || !aligned(b, 16) || !aligned(out, 16))
            return fail(FP8_ERR_ALIGN, "%s: a, b, out not 16-byte aligned", fn);
        if (lda % 16 != 0 || ldb % 16 != 0)
            return fail(FP8_ERR_ALIGN, "%s: lda, ldb must be multiples of 16", fn);
        const int64_t out_align = (flags & FP8_OUT_FP32) ? 4 : 8;
        if (ld_out % out_align != 0) return fail(FP8_ERR_ALIGN, "%s: ld_out=%lld must be a multiple of %lld", fn, (long long)ld_out, (long long)out_align);
    }
    FP8_TRY(fp8k::launch_gemm_mxfp8(a, lda, fmt_a, ea, ld_ea, b, ldb, fmt_b, eb, ld_eb, M, N, K, out, ld_out,
                                    (flags & FP8_OUT_FP32) ? 1 : 0, static_cast<hipStream_t>(stream)));
    return FP8_OK;
}

namespace {
struct MxPlan { size_t xq, wq, xe, we, total; };
MxPlan plan_mx(int64_t M, int64_t K, int64_t N) {
    MxPlan p{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    p.xq = take((size_t)M * K);
    p.wq = take((size_t)N * K);
    p.xe = take((size_t)M * (K / 32));
    p.we = take((size_t)N * (K / 32));
    p.total = o;
    return p;
}
}  // namespace

size_t fp8_mx_linear_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    g_err[0] = 0;
    if (M < 0 || K < 0 || N < 0 || M > kMaxDim || K > kMaxDim || N > kMaxDim || K % 128 != 0) {
        fail(FP8_ERR_SHAPE, "fp8_mx_linear_workspace_bytes: M=%lld K=%lld N=%lld (K must be a multiple of 128)", (long long)M, (long long)K, (long long)N);
        return 0;
    }
    const size_t t = plan_mx(M, K, N).total;
    return t ? t : 256;
}

int fp8_mx_linear_fwd(const void* x, const void* w, int64_t M, int64_t K, int64_t N, int fmt_x, int fmt_w, void* y,
                      void* workspace, size_t workspace_bytes, void* stream) {
    g_err[0] = 0;
    const char* fn = "fp8_mx_linear_fwd";
    if (!fmt_ok(fmt_x) || !fmt_ok(fmt_w)) return fail(FP8_ERR_ENUM, "%s: unknown fp8 format", fn);
    if (int rc = check_linear_dims(fn, M, K, N, false)) return rc;
    if (K % 128 != 0) return fail(FP8_ERR_SHAPE, "%s: K=%lld must be a multiple of 128", fn, (long long)K);
    if (int rc = check_bf16("fp8_mx_linear_fwd(x)", x, M, K, K)) return rc;
    if (int rc = check_bf16("fp8_mx_linear_fwd(w)", w, N, K, K)) return rc;
    if (M == 0 || N == 0) return FP8_OK;
    if (!y || !workspace) return fail(FP8_ERR_NULL, "%s: y or workspace is NULL", fn);
    if (!aligned(y, 16) || !aligned(workspace, 256)) return fail(FP8_ERR_ALIGN, "%s: y (16) / workspace (256) misaligned", fn);
    const MxPlan p = plan_mx(M, K, N);
    if (workspace_bytes < p.total) return fail(FP8_ERR_WORKSPACE, "%s: workspace %zu < %zu bytes", fn, workspace_bytes, p.total);
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    // scales between the quantizers and the GEMM: in slabs of sixteen blocks (negative leading dimension) where the GEMM takes them
    const bool slab = fp8k::gemm_mxfp8_takes_slab_scales(K, K, M, N, K);
    const int64_t ld_xe = slab ? -M : K / 32, ld_we = slab ? -N : K / 32;
    FP8_TRY(fp8k::launch_mx_quant(x, M, K, K, fmt_x, ws + p.xq, K, ws + p.xe, ld_xe, st));
    FP8_TRY(fp8k::launch_mx_quant(w, N, K, K, fmt_w, ws + p.wq, K, ws + p.we, ld_we, st));
    FP8_TRY(fp8k::launch_gemm_mxfp8(ws + p.xq, K, fmt_x, ws + p.xe, ld_xe, ws + p.wq, K, fmt_w, ws + p.we, ld_we, M, N, K, y,
                                    N, 0, st));
    return FP8_OK;
}

int fp8_block_quantize(const void* x, int64_t rows, int64_t cols, int64_t ld, int block_rows, int format, uint8_t* q_out,
                       int64_t ld_q, uint8_t* e8m0_out, int64_t ld_e, void* stream) {
    g_err[0] = 0;
    const char* fn = "fp8_block_quantize";
    if (!fmt_ok(format)) return fail(FP8_ERR_ENUM, "%s: unknown format %d", fn, format);
    if (block_rows != 1 && block_rows != 128) return fail(FP8_ERR_ENUM, "%s: block_rows=%d must be 1 or 128", fn, block_rows);
    if (int rc = check_bf16(fn, x, rows, cols, ld)) return rc;
    if (cols % 128 != 0) return fail(FP8_ERR_SHAPE, "%s: cols=%lld must be a multiple of the block width 128", fn, (long long)cols);
    if (block_rows == 128 && rows > (int64_t)65535 * 128) return fail(FP8_ERR_SHAPE, "%s: rows=%lld too large", fn, (long long)rows);
    if (int rc = check_q_out(fn, q_out, rows, cols, ld_q, 0)) return rc;
    if (int rc = check_e8m0(fn, e8m0_out, rows, cols / 32, ld_e)) return rc;
    FP8_TRY(fp8k::launch_block_quant(x, rows, cols, ld, block_rows, format, q_out, ld_q, e8m0_out, ld_e, static_cast<hipStream_t>(stream)));
    return FP8_OK;
}

size_t fp8_block_linear_workspace_bytes(int64_t M, int64_t K, int64_t N) { return fp8_mx_linear_workspace_bytes(M, K, N); }

int fp8_block_linear_fwd(const void* x, const void* w, int64_t M, int64_t K, int64_t N, int fmt_x, int fmt_w, void* y,
                         void* workspace, size_t workspace_bytes, void* stream) {
    g_err[0] = 0;
    const char* fn = "fp8_block_linear_fwd";
    if (!fmt_ok(fmt_x) || !fmt_ok(fmt_w)) return fail(FP8_ERR_ENUM, "%s: unknown fp8 format", fn);
    if (int rc = check_linear_dims(fn, M, K, N, false)) return rc;
    if (K % 128 != 0) return fail(FP8_ERR_SHAPE, "%s: K=%lld must be a multiple of 128", fn, (long long)K);
    if (N > (int64_t)65535 * 128) return fail(FP8_ERR_SHAPE, "%s: N=%lld too large", fn, (long long)N);
    if (int rc = check_bf16("fp8_block_linear_fwd(x)", x, M, K, K)) return rc;
    if (int rc = check_bf16("fp8_block_linear_fwd(w)", w, N, K, K)) return rc;
    if (M == 0 || N == 0) return FP8_OK;
    if (!y || !workspace) return fail(FP8_ERR_NULL, "%s: y or workspace is NULL", fn);
    if (!aligned(y, 16) || !aligned(workspace, 256)) return fail(FP8_ERR_ALIGN, "%s: y (16) / workspace (256) misaligned", fn);
    const MxPlan p = plan_mx(M, K, N);
    if (workspace_bytes < p.total) return fail(FP8_ERR_WORKSPACE, "%s: workspace %zu < %zu bytes", fn, workspace_bytes, p.total);
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    // X in tiles of 1 x 128 along K, W in blocks of 128 x 128; the block-scaled GEMM applies the power-of-two scales
    // scales between the quantizers and the GEMM: in slabs of sixteen blocks (negative leading dimension) where the GEMM takes them
    const bool slab = fp8k::gemm_mxfp8_takes_slab_scales(K, K, M, N, K);
    const int64_t ld_xe = slab ? -M : K / 32, ld_we = slab ? -N : K / 32;
    FP8_TRY(fp8k::launch_block_quant(x, M, K, K, 1, fmt_x, ws + p.xq, K, ws + p.xe, ld_xe, st));
    FP8_TRY(fp8k::launch_block_quant(w, N, K, K, 128, fmt_w, ws + p.wq, K, ws + p.we, ld_we, st));
    FP8_TRY(fp8k::launch_gemm_mxfp8(ws + p.xq, K, fmt_x, ws + p.xe, ld_xe, ws + p.wq, K, fmt_w, ws + p.we, ld_we, M, N, K, y,
                                    N, 0, st));
    return FP8_OK;
}

namespace {
// workspace of the MX backward: the four re-quantized operands and their block scales
struct MxBwdPlan { size_t dyq, dye, wtq, wte, dytq, dyte, xtq, xte, total; };
// The products contract over 128 bytes per step: the operands' contraction axes (N for dX, M for dW) are padded to
// multiples of 128 inside the workspace, with zero codes and zero scale bytes in the pad (cleared before the
// quantizers write the valid part), so the products may run over the padded lengths.
int64_t pad128(int64_t v) { return (v + 127) / 128 * 128; }
MxBwdPlan plan_mx_bwd(int64_t M, int64_t K, int64_t N) {
    MxBwdPlan p{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    const size_t Mp = (size_t)pad128(M), Np = (size_t)pad128(N);
    p.dyq = take((size_t)M * Np);
    p.dye = take((size_t)M * (Np / 32));
    p.wtq = take((size_t)K * Np);
    p.wte = take((size_t)K * (Np / 32));
    p.dytq = take((size_t)N * Mp);
    p.dyte = take((size_t)N * (Mp / 32));
    p.xtq = take((size_t)K * Mp);
    p.xte = take((size_t)K * (Mp / 32));
    p.total = o;
    return p;
}
// granule: what M and N must be multiples of - the block of 32 for MX, the tile of 128 for the blockwise recipe
int check_mx_bwd_dims(const char* fn, int64_t M, int64_t K, int64_t N, int granule) {
    if (M < 0 || K < 0 || N < 0 || M > kMaxDim - 127 || K > kMaxDim || N > kMaxDim - 127)
        return fail(FP8_ERR_SHAPE, "%s: M=%lld K=%lld N=%lld out of range", fn, (long long)M, (long long)K, (long long)N);
    if (M % granule != 0 || N % granule != 0)
        return fail(FP8_ERR_SHAPE, "%s: the backward contracts over M and N: M=%lld, N=%lld must be multiples of %d", fn,
                    (long long)M, (long long)N, granule);
    if (K % 8 != 0) return fail(FP8_ERR_SHAPE, "%s: K=%lld must be a multiple of 8 (dense bfloat16 rows)", fn, (long long)K);
    return FP8_OK;
}
}  // namespace

size_t fp8_mx_linear_bwd_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    g_err[0] = 0;
    if (check_mx_bwd_dims("fp8_mx_linear_bwd_workspace_bytes", M, K, N, 32)) return 0;
    const size_t t = plan_mx_bwd(M, K, N).total;
    return t ? t : 256;
}

int fp8_mx_linear_bwd(const void* dy, const void* x, const void* w, int64_t M, int64_t K, int64_t N, int fmt_dy,
                      int fmt_x, int fmt_w, void* dx, void* dw, void* workspace, size_t workspace_bytes, void* stream) {
    g_err[0] = 0;
    const char* fn = "fp8_mx_linear_bwd";
    if (!fmt_ok(fmt_dy) || !fmt_ok(fmt_x) || !fmt_ok(fmt_w)) return fail(FP8_ERR_ENUM, "%s: unknown fp8 format", fn);
    if (int rc = check_mx_bwd_dims(fn, M, K, N, 32)) return rc;
    if (int rc = check_bf16("fp8_mx_linear_bwd(dy)", dy, M, N, N)) return rc;
    if (dx) if (int rc = check_bf16("fp8_mx_linear_bwd(w)", w, N, K, K)) return rc;
    if (dw) if (int rc = check_bf16("fp8_mx_linear_bwd(x)", x, M, K, K)) return rc;
    if (!dx && !dw) return FP8_OK;
    if (M == 0 || N == 0 || K == 0) {
        // an empty contraction leaves an all-zero gradient
        hipStream_t st0 = static_cast<hipStream_t>(stream);
        if (dx && M > 0 && K > 0) FP8_TRY(fp8k::launch_fill_u32(static_cast<uint32_t*>(dx), M * K / 2, 0u, st0));
        if (dw && N > 0 && K > 0) FP8_TRY(fp8k::launch_fill_u32(static_cast<uint32_t*>(dw), N * K / 2, 0u, st0));
        return FP8_OK;
    }
    if (!workspace) return fail(FP8_ERR_NULL, "%s: workspace is NULL", fn);
    if ((dx && !aligned(dx, 16)) || (dw && !aligned(dw, 16)) || !aligned(workspace, 256))
        return fail(FP8_ERR_ALIGN, "%s: dx, dw (16) / workspace (256) misaligned", fn);
    const MxBwdPlan p = plan_mx_bwd(M, K, N);
    if (workspace_bytes < p.total) return fail(FP8_ERR_WORKSPACE, "%s: workspace %zu < %zu bytes", fn, workspace_bytes, p.total);
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    const int64_t Mp = pad128(M), Np = pad128(N);   // contraction lengths of dW / dX, padded with zeros
    if (Mp != M || Np != N) FP8_TRY(fp8k::launch_fill_u32(reinterpret_cast<uint32_t*>(ws), (int64_t)(p.total / 4), 0u, st));
    // scales in slabs of sixteen blocks (negative leading dimension) where the product that reads them takes them
    const bool slab_dx = dx && fp8k::gemm_mxfp8_takes_slab_scales(Np, Np, M, K, Np);
    const bool slab_dw = dw && fp8k::gemm_mxfp8_takes_slab_scales(Mp, Mp, N, K, Mp);
    const int64_t ld_dye = slab_dx ? -M : Np / 32, ld_wte = slab_dx ? -K : Np / 32;
    const int64_t ld_dyte = slab_dw ? -N : Mp / 32, ld_xte = slab_dw ? -K : Mp / 32;
    // all quantizations first, then the products back to back
    if (dx && dw) {   // the gradient in both orientations from one read
        FP8_TRY(fp8k::launch_mx_quant_t(dy, M, N, N, fmt_dy, ws + p.dytq, Mp, ws + p.dyte, ld_dyte, ws + p.dyq, Np, ws + p.dye, ld_dye, st));
    } else if (dx) {
        FP8_TRY(fp8k::launch_mx_quant(dy, M, N, N, fmt_dy, ws + p.dyq, Np, ws + p.dye, ld_dye, st));
    } else {
        FP8_TRY(fp8k::launch_mx_quant_t(dy, M, N, N, fmt_dy, ws + p.dytq, Mp, ws + p.dyte, ld_dyte, nullptr, 0, nullptr, 0, st));
    }
    if (dx) FP8_TRY(fp8k::launch_mx_quant_t(w, N, K, K, fmt_w, ws + p.wtq, Np, ws + p.wte, ld_wte, nullptr, 0, nullptr, 0, st));
    if (dw) FP8_TRY(fp8k::launch_mx_quant_t(x, M, K, K, fmt_x, ws + p.xtq, Mp, ws + p.xte, ld_xte, nullptr, 0, nullptr, 0, st));
    if (dx)
        FP8_TRY(fp8k::launch_gemm_mxfp8(ws + p.dyq, Np, fmt_dy, ws + p.dye, ld_dye, ws + p.wtq, Np, fmt_w, ws + p.wte, ld_wte,
                                        M, K, Np, dx, K, 0, st));
    if (dw)
        FP8_TRY(fp8k::launch_gemm_mxfp8(ws + p.dytq, Mp, fmt_dy, ws + p.dyte, ld_dyte, ws + p.xtq, Mp, fmt_x, ws + p.xte, ld_xte,
                                        N, K, Mp, dw, K, 0, st));
    return FP8_OK;
}

int fp8_block_quantize_t(const void* x, int64_t rows, int64_t cols, int64_t ld, int block_rows, int format, uint8_t* qt_out,
                         int64_t ld_q, uint8_t* e8m0_t_out, int64_t ld_e, void* stream) {
    g_err[0] = 0;
    const char* fn = "fp8_block_quantize_t";
    if (!fmt_ok(format)) return fail(FP8_ERR_ENUM, "%s: unknown format %d", fn, format);
    if (block_rows != 1 && block_rows != 128) return fail(FP8_ERR_ENUM, "%s: block_rows=%d must be 1 or 128", fn, block_rows);
    if (int rc = check_bf16(fn, x, rows, cols, ld)) return rc;
    if (rows % 128 != 0) return fail(FP8_ERR_SHAPE, "%s: rows=%lld must be a multiple of the block length 128", fn, (long long)rows);
    if (cols % 8 != 0) return fail(FP8_ERR_SHAPE, "%s: cols=%lld must be a multiple of 8", fn, (long long)cols);
    if (int rc = check_q_out(fn, qt_out, cols, rows, ld_q, 0)) return rc;
    if (int rc = check_e8m0(fn, e8m0_t_out, cols, rows / 32, ld_e)) return rc;
    FP8_TRY(fp8k::launch_block_quant_t(x, rows, cols, ld, block_rows, format, qt_out, ld_q, e8m0_t_out, ld_e,
                                       static_cast<hipStream_t>(stream)));
    return FP8_OK;
}

int fp8_block_quantize_row_col(const void* x, int64_t rows, int64_t cols, int64_t ld, int format, uint8_t* q_row,
                               int64_t ld_row, uint8_t* e_row, int64_t ld_er, uint8_t* q_col_t, int64_t ld_col_t,
                               uint8_t* e_col_t, int64_t ld_ec, void* stream) {
    g_err[0] = 0;
    const char* fn = "fp8_block_quantize_row_col";
    if (!fmt_ok(format)) return fail(FP8_ERR_ENUM, "%s: unknown format %d", fn, format);
    if (int rc = check_bf16(fn, x, rows, cols, ld)) return rc;
    if (rows % 128 != 0 || cols % 128 != 0)
        return fail(FP8_ERR_SHAPE, "%s: rows=%lld and cols=%lld must be multiples of the tile length 128", fn, (long long)rows, (long long)cols);
    if (int rc = check_q_out(fn, q_row, rows, cols, ld_row, 0)) return rc;
    if (int rc = check_q_out(fn, q_col_t, cols, rows, ld_col_t, 0)) return rc;
    if (int rc = check_e8m0("fp8_block_quantize_row_col(e_row)", e_row, rows, cols / 32, ld_er)) return rc;
    if (int rc = check_e8m0("fp8_block_quantize_row_col(e_col_t)", e_col_t, cols, rows / 32, ld_ec)) return rc;
    FP8_TRY(fp8k::launch_block_quant_t(x, rows, cols, ld, 1, format, q_col_t, ld_col_t, e_col_t, ld_ec, static_cast<hipStream_t>(stream),
                                       q_row, ld_row, e_row, ld_er));
    return FP8_OK;
}

size_t fp8_block_linear_bwd_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    g_err[0] = 0;
    if (check_mx_bwd_dims("fp8_block_linear_bwd_workspace_bytes", M, K, N, 128)) return 0;
    const size_t t = plan_mx_bwd(M, K, N).total;
    return t ? t : 256;
}

int fp8_block_linear_bwd(const void* dy, const void* x, const void* w, int64_t M, int64_t K, int64_t N, int fmt_dy,
                         int fmt_x, int fmt_w, void* dx, void* dw, void* workspace, size_t workspace_bytes, void* stream) {
    g_err[0] = 0;
    const char* fn = "fp8_block_linear_bwd";
    if (!fmt_ok(fmt_dy) || !fmt_ok(fmt_x) || !fmt_ok(fmt_w)) return fail(FP8_ERR_ENUM, "%s: unknown fp8 format", fn);
    if (int rc = check_mx_bwd_dims(fn, M, K, N, 128)) return rc;
    if (int rc = check_bf16("fp8_block_linear_bwd(dy)", dy, M, N, N)) return rc;
    if (dx) if (int rc = check_bf16("fp8_block_linear_bwd(w)", w, N, K, K)) return rc;
    if (dw) if (int rc = check_bf16("fp8_block_linear_bwd(x)", x, M, K, K)) return rc;
    if (!dx && !dw) return FP8_OK;
    if (M == 0 || N == 0 || K == 0) {
        hipStream_t st0 = static_cast<hipStream_t>(stream);
        if (dx && M > 0 && K > 0) FP8_TRY(fp8k::launch_fill_u32(static_cast<uint32_t*>(dx), M * K / 2, 0u, st0));
        if (dw && N > 0 && K > 0) FP8_TRY(fp8k::launch_fill_u32(static_cast<uint32_t*>(dw), N * K / 2, 0u, st0));
        return FP8_OK;
    }
    if (!workspace) return fail(FP8_ERR_NULL, "%s: workspace is NULL", fn);
    if ((dx && !aligned(dx, 16)) || (dw && !aligned(dw, 16)) || !aligned(workspace, 256))
        return fail(FP8_ERR_ALIGN, "%s: dx, dw (16) / workspace (256) misaligned", fn);
    const MxBwdPlan p = plan_mx_bwd(M, K, N);
    if (workspace_bytes < p.total) return fail(FP8_ERR_WORKSPACE, "%s: workspace %zu < %zu bytes", fn, workspace_bytes, p.total);
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    // scales in slabs of sixteen blocks (negative leading dimension) where the product that reads them takes them
    const bool slab_dx = dx && fp8k::gemm_mxfp8_takes_slab_scales(N, N, M, K, N);
    const bool slab_dw = dw && fp8k::gemm_mxfp8_takes_slab_scales(M, M, N, K, M);
    const int64_t ld_dye = slab_dx ? -M : N / 32, ld_wte = slab_dx ? -K : N / 32;
    const int64_t ld_dyte = slab_dw ? -N : M / 32, ld_xte = slab_dw ? -K : M / 32;
    // dX = dY W: dY in tiles along N, W^T [K, N] in its 128 x 128 blocks; dW = dY^T X: dY^T and X^T in tiles along M
    if (dx && dw) {   // the gradient in both orientations from one read
        FP8_TRY(fp8k::launch_block_quant_t(dy, M, N, N, 1, fmt_dy, ws + p.dytq, M, ws + p.dyte, ld_dyte, st, ws + p.dyq, N, ws + p.dye, ld_dye));
    } else if (dx) {
        FP8_TRY(fp8k::launch_block_quant(dy, M, N, N, 1, fmt_dy, ws + p.dyq, N, ws + p.dye, ld_dye, st));
    } else {
        FP8_TRY(fp8k::launch_block_quant_t(dy, M, N, N, 1, fmt_dy, ws + p.dytq, M, ws + p.dyte, ld_dyte, st));
    }
    if (dx) FP8_TRY(fp8k::launch_block_quant_t(w, N, K, K, 128, fmt_w, ws + p.wtq, N, ws + p.wte, ld_wte, st));
    if (dw) FP8_TRY(fp8k::launch_block_quant_t(x, M, K, K, 1, fmt_x, ws + p.xtq, M, ws + p.xte, ld_xte, st));
    if (dx)
        FP8_TRY(fp8k::launch_gemm_mxfp8(ws + p.dyq, N, fmt_dy, ws + p.dye, ld_dye, ws + p.wtq, N, fmt_w, ws + p.wte, ld_wte,
                                        M, K, N, dx, K, 0, st));
    if (dw)
        FP8_TRY(fp8k::launch_gemm_mxfp8(ws + p.dytq, M, fmt_dy, ws + p.dyte, ld_dyte, ws + p.xtq, M, fmt_x, ws + p.xte, ld_xte,
                                        N, K, M, dw, K, 0, st));
    return FP8_OK;
}

}  // extern "C"
