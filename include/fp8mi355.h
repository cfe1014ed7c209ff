/*
 * fp8mi355 - dynamically scaled float8 linear layer for AMD Instinct MI355X
 * (gfx950 / CDNA4).  C ABI of libfp8mi355.so.
 *
 * The library implements the hot path of the FP8 training flow described in
 * the TorchAO paper (arXiv 2507.16099), Section 2.1 "FP8 Training" and
 * Appendix A "FP8 Scaling Recipes": activations, weights and gradients are
 * cast to FP8 dynamically (amax -> scale -> saturating round-to-nearest-even
 * cast) and the matrix products run on FP8 matrix cores with fp32
 * accumulation, for the forward product Y = X W^T and the two backward
 * products dX = dY W and dW = dY^T X.
 *
 * Conventions common to every call
 * --------------------------------
 *  - All data pointers are DEVICE pointers (HBM of the current HIP device),
 *    16-byte aligned.  bfloat16 tensors are passed as const void*, fp8
 *    tensors as uint8_t* (one code per byte), scales and amax as float*.
 *  - Matrices are row-major; `ld*` arguments are leading dimensions in
 *    ELEMENTS and must be >= the number of columns and a multiple of 8 for
 *    bfloat16 inputs / 16 for fp8 tensors (keeps every row 16-byte aligned).
 *  - A "scale" s is the quantization multiplier: q = cast(x * s).  The GEMM
 *    dequantizes with 1/s.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Every call only enqueues work on that stream and returns; nothing
 *    synchronizes with the host.
 *  - Ownership: the caller owns every buffer, including the workspace.  The
 *    library allocates no device memory and keeps no state between calls.
 *  - Errors: arguments are validated on the host BEFORE anything is launched.
 *    A negative fp8_status is returned and fp8_last_error() describes it;
 *    nothing is thrown across the boundary and the process is never aborted.
 *    Inputs are expected to be finite; NaN maps to a NaN code, +-Inf saturates
 *    in fp8_cast, and amax of non-finite input is unspecified.
 *  - Empty problems (a dimension equal to 0) are accepted and do nothing.
 */
#ifndef FP8MI355_H
#define FP8MI355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* FP8 formats (OCP OFP8): E4M3 "fn" (bias 7, max 448, no Inf) for activations
 * and weights, E5M2 (bias 15, max 57344) for gradients. */
enum fp8_format { FP8_E4M3FN = 0, FP8_E5M2 = 1 };

/* Scaling granularity (Appendix A).  TENSOR: one scale for the whole matrix.
 * ROW: one scale per row (the group runs over the columns).  COL: one scale
 * per column (the group runs over the rows). */
enum fp8_gran { FP8_TENSOR = 0, FP8_ROW = 1, FP8_COL = 2 };

enum fp8_flags {
    FP8_POW2_SCALE    = 1, /* round the scale down to a power of two            */
    FP8_TRANSPOSE_OUT = 2, /* fp8_cast / fp8_quantize write q[c, r] not q[r, c] */
    FP8_OUT_FP32      = 4, /* fp8_scaled_mm writes fp32 instead of bfloat16     */
    FP8_GRAD_WEIGHT_HP = 8, /* recipe flag: dW is computed in bfloat16, not FP8  */
    FP8_EPILOGUE_SIGMOID = 32, /* fp8_scaled_mm: out = bfloat16(sigmoid(result)) instead of bfloat16(result) */
    FP8_SAVE_FOR_BWD  = 16 /* recipe flag: the forward leaves the transposed fp8 copies of X and W
                              in the workspace and the backward reuses them                    */
};

enum fp8_status {
    FP8_OK = 0,
    FP8_ERR_NULL = -1,      /* a required pointer is NULL                       */
    FP8_ERR_SHAPE = -2,     /* negative dimension, ld too small, K not % 16     */
    FP8_ERR_ENUM = -3,      /* unknown format / granularity / flag              */
    FP8_ERR_ALIGN = -4,     /* pointer or leading dimension not aligned         */
    FP8_ERR_WORKSPACE = -5, /* workspace smaller than fp8_linear_workspace_bytes */
    FP8_ERR_HIP = -6        /* a kernel launch failed (hipGetLastError)         */
};

/* Description of the last error on the calling thread ("" if none).  The
 * returned pointer refers to thread-local static storage. */
const char* fp8_last_error(void);

/* Library version string, static storage. */
const char* fp8_version(void);

/*
 * amax (Section 2.1: the cast is dynamic, so the statistic is recomputed from
 * the tensor on every call; Appendix A fixes the group).
 *   x        [rows, cols] bfloat16, leading dimension ld.
 *   gran     FP8_TENSOR -> amax_out[1]; FP8_ROW -> amax_out[rows];
 *            FP8_COL -> amax_out[cols].
 *   amax_out max over the group of |x| as fp32 (exact: a bfloat16 magnitude).
 */
int fp8_amax(const void* x, int64_t rows, int64_t cols, int64_t ld, int gran,
             float* amax_out, void* stream);

/*
 * scale (Appendix A: one factor for the whole tensor, or one per row / column).
 *   scale_out[i] = fp32( FMAX(format) / max(amax[i], 1e-12) ), the quotient
 *   correctly rounded; with FP8_POW2_SCALE it is then rounded down to 2^k.
 *   amax and scale_out have n entries and may alias.
 */
int fp8_scale(const float* amax, int64_t n, int format, int flags, float* scale_out, void* stream);

/*
 * cast (Section 2.1: cast to FP8) with given scales.
 *   q = fp8( clamp( fp32(x) * s, +-FMAX ) ), round to nearest even, saturating;
 *   s = scale[0] (TENSOR), scale[r] (ROW) or scale[c] (COL).
 *   q_out is [rows, cols] (leading dimension ld_out) or, with
 *   FP8_TRANSPOSE_OUT, [cols, rows].
 */
int fp8_cast(const void* x, int64_t rows, int64_t cols, int64_t ld, const float* scale, int gran,
             int format, int flags, uint8_t* q_out, int64_t ld_out, void* stream);

/*
 * fused amax -> scale -> cast of one operand (the "dynamic quantization" of
 * Section 2.1 as one call).  Writes the codes to q_out (layout as fp8_cast)
 * and the scales to scale_out ([1] | [rows] | [cols]).
 *   ROW without transpose is a single pass over HBM (the row stays in
 *   registers between the reduction and the cast); TENSOR and COL read the
 *   input twice.  flags: FP8_POW2_SCALE, FP8_TRANSPOSE_OUT.  q_out may serve as
 *   scratch before it receives its codes; bytes outside the [rows, cols] (or
 *   transposed [cols, rows]) window of a padded output are never written.
 */
int fp8_quantize(const void* x, int64_t rows, int64_t cols, int64_t ld, int gran, int format,
                 int flags, uint8_t* q_out, int64_t ld_out, float* scale_out, void* stream);

/*
 * one tensor quantized along BOTH axes (Appendix A, rowwise recipe: the output
 * gradient feeds dX = dY W with one scale per row and dW = dY^T X with one
 * scale per column).  Results are identical to
 *   fp8_quantize(x, ..., FP8_ROW, format, flags, q_row, ld_row, scale_row) and
 *   fp8_quantize(x, ..., FP8_COL, format, flags | FP8_TRANSPOSE_OUT, q_col_t, ld_col_t, scale_col),
 * but x is read twice instead of three times: the column maxima are gathered
 * in the pass that writes the rowwise codes.
 *   q_row [rows, cols] (ld_row), scale_row [rows]; q_col_t [cols, rows]
 *   (ld_col_t), scale_col [cols].  The four outputs must not overlap; q_col_t
 *   is also used as scratch before it receives its codes (only bytes that the
 *   codes overwrite afterwards: the padding between the rows of an output with
 *   ld_col_t > rows is never written).
 *   flags: FP8_POW2_SCALE only.
 */
int fp8_quantize_row_col(const void* x, int64_t rows, int64_t cols, int64_t ld, int format, int flags,
                         uint8_t* q_row, int64_t ld_row, float* scale_row,
                         uint8_t* q_col_t, int64_t ld_col_t, float* scale_col, void* stream);

/*
 * scaled GEMM on FP8 matrix cores (Section 2.1: the FP8 products run in GEMM
 * kernels made for the low-precision matrix units).
 *   out[m, n] = ( sum_k dec(a[m, k]) * dec(b[n, k]) ) / (sa * sb)
 *   a [M, K] and b [N, K] are fp8 codes with the contraction axis contiguous
 *   (leading dimensions lda, ldb); fmt_a / fmt_b select E4M3FN or E5M2 per
 *   operand.  sa = scale_a[0] (gran_a == FP8_TENSOR) or scale_a[m] (FP8_ROW);
 *   sb likewise with n.  Accumulation is fp32; out is [M, N] bfloat16
 *   (round to nearest even) or fp32 with FP8_OUT_FP32, leading dimension
 *   ld_out.  K must be a multiple of 16; M and N are arbitrary.
 *   FP8_EPILOGUE_SIGMOID (not with FP8_OUT_FP32; lda, ldb < 2^23): the logistic
 *   function 1 / (1 + exp(-v)) is applied to the fp32 value v before the rounding
 *   to bfloat16 - the activation behind the linear layer in the paper's float8
 *   microbenchmark (appendix "Float8 Training Microbenchmarks"), fused into the
 *   GEMM's epilogue.
 */
int fp8_scaled_mm(const uint8_t* a, int64_t lda, int fmt_a, const float* scale_a, int gran_a,
                  const uint8_t* b, int64_t ldb, int fmt_b, const float* scale_b, int gran_b,
                  int64_t M, int64_t N, int64_t K, void* out, int64_t ld_out, int flags,
                  void* stream);

/* Recipe of a linear layer (Appendix A): gran is FP8_TENSOR ("tensorwise") or
 * FP8_ROW ("rowwise": every operand scaled along the contraction axis of the
 * GEMM it feeds).  flags: FP8_POW2_SCALE, FP8_GRAD_WEIGHT_HP (with FP8_ROW this
 * is the "rowwise_gw_hp" recipe: the forward and dX run in FP8, the weight
 * gradient dW = dY^T X is computed from the unquantized bfloat16 tensors).
 * FP8_SAVE_FOR_BWD: the fp8 copies of X and W that the backward needs do not
 * depend on the gradient, so the forward can make them from the same read as
 * its own and leave them in the workspace; the backward then quantizes dY alone.
 * Tensorwise (Appendix A: one scale for the whole tensor): the same
 * codes, only transposed - one conversion into both layouts, 3 quantizations
 * per step instead of 5.  Rowwise: the per-column, transposed codes of X and W
 * next to the rowwise ones, two reads of each tensor per step instead of
 * three.  Codes, scales and results are the same as without the flag.  Both
 * calls must carry the flag and get the SAME workspace, of
 * fp8_linear_workspace_bytes(..., bwd = 1) bytes, untouched in between; x and w
 * may then be NULL in fp8_linear_bwd (x is still read for dW when the recipe
 * also carries FP8_GRAD_WEIGHT_HP). */
typedef struct fp8_recipe {
    int gran;
    int fmt_x;  /* format of activations, normally FP8_E4M3FN */
    int fmt_w;  /* format of weights,     normally FP8_E4M3FN */
    int fmt_dy; /* format of gradients,   normally FP8_E5M2   */
    int flags;
} fp8_recipe;

/* Bytes of workspace fp8_linear_fwd (bwd == 0) or fp8_linear_bwd (bwd != 0)
 * needs for X [M,K], W [N,K], dY [M,N].  Returns 0 on invalid arguments. */
size_t fp8_linear_workspace_bytes(int64_t M, int64_t K, int64_t N, const fp8_recipe* recipe, int bwd);

/*
 * forward of the float8 linear: Y[M,N] = X[M,K] W[N,K]^T.
 * X and W (bfloat16, dense row-major) are quantized along K, then multiplied.
 * y is bfloat16 [M,N] dense.  workspace holds the fp8 copies and scales.
 */
int fp8_linear_fwd(const void* x, const void* w, int64_t M, int64_t K, int64_t N,
                   const fp8_recipe* recipe, void* y, void* workspace, size_t workspace_bytes,
                   void* stream);

/*
 * backward of the float8 linear: dX[M,K] = dY[M,N] W[N,K] and
 * dW[N,K] = dY[M,N]^T X[M,K].  For dX, dY is quantized per row and W per
 * column (along N); for dW, dY and X are quantized per column (along M); the
 * per-column operands are written transposed so that every GEMM contracts
 * over a contiguous axis.  Tensorwise: one scale per tensor, only the layouts
 * change.  dx and dw are bfloat16, dense; either may be NULL to skip it.
 * K and N multiples of 16; M (tokens) arbitrary: the transposed operands of dW,
 * whose contraction axis is M, get rows padded to 16 bytes with zero codes
 * inside the workspace (token counts on the 16-byte grid take the faster
 * quantization kernels).
 */
int fp8_linear_bwd(const void* dy, const void* x, const void* w, int64_t M, int64_t K, int64_t N,
                   const fp8_recipe* recipe, void* dx, void* dw, void* workspace,
                   size_t workspace_bytes, void* stream);

/*
 * backward through Sigmoid + Linear (the block of the paper's float8 microbenchmark,
 * appendix "Float8 Training Microbenchmarks"): y [M, N] bfloat16 is the stored sigmoid
 * output, dy [M, N] the gradient arriving at it.  The gradient of the linear layer's
 * output,  dz = dy * y * (1 - y)  (binary32, one operation at a time, rounded to
 * bfloat16), takes the place of dY in fp8_linear_bwd; with the rowwise recipe and
 * M >= 1024 a multiple of 16, N a multiple of 8 in [512, 32768] it is formed inside the two
 * quantization passes and never stored, otherwise it is written once into the
 * workspace.  Everything else as fp8_linear_bwd (including FP8_SAVE_FOR_BWD, where
 * the shared workspace must then have fp8_linear_bwd_sigmoid_workspace_bytes bytes).
 */
size_t fp8_linear_bwd_sigmoid_workspace_bytes(int64_t M, int64_t K, int64_t N, const fp8_recipe* recipe);
int fp8_linear_bwd_sigmoid(const void* dy, const void* y, const void* x, const void* w, int64_t M, int64_t K,
                           int64_t N, const fp8_recipe* recipe, void* dx, void* dw, void* workspace,
                           size_t workspace_bytes, void* stream);

/*
 * weight gradient in high precision (Appendix A, rowwise_gw_hp: the grad_weight
 * GEMM kept in bfloat16):  dw[n, k] = sum_m dy[m, n] * x[m, k]
 *   dy [M, N] and x [M, K] bfloat16, dense rows; products and sums in fp32 on
 *   the bfloat16 matrix cores; dw [N, K] bfloat16 (round to nearest even).
 *   K and N multiples of 8; M arbitrary.  This is what fp8_linear_bwd runs for dW
 *   when the recipe carries FP8_GRAD_WEIGHT_HP.
 */
int fp8_grad_weight_hp(const void* dy, const void* x, int64_t M, int64_t K, int64_t N, void* dw, void* stream);

/*
 * inference-style forward with a weight that was quantized ONCE beforehand
 * (Section 3: float8 dynamic activation + float8 weight quantization, per
 * tensor or per row):  Y = X W^T with
 *   wq [N, K] fp8 codes (format fmt_w, leading dimension ldw) and scale_w
 *   ([1] for gran_w == FP8_TENSOR, [N] for FP8_ROW), e.g. from fp8_quantize;
 *   x [M, K] bfloat16 (dense rows), quantized dynamically inside the call with
 *   granularity gran_x (TENSOR | ROW) to format fmt_x; flags: FP8_POW2_SCALE
 *   (for the activation scales).  y [M, N] bfloat16, leading dimension ld_y.
 * workspace: fp8_linear_prequantized_workspace_bytes(M, K) bytes, 256-byte
 * aligned (activation codes and scales).  With few rows (M <= 32, decoding) the
 * GEMM streams wq once and is bound by that HBM read.  For a single token (and
 * up to four with M * K <= 16384; K a multiple of 512 and at most 32768, fmt_x
 * e4m3) the activation scales and codes are formed inside that GEMM's launch:
 * one launch instead of two, the same bits, and the workspace is not written.
 */
size_t fp8_linear_prequantized_workspace_bytes(int64_t M, int64_t K);
int fp8_linear_fwd_prequantized(const void* x, int64_t M, int64_t K, int fmt_x, int gran_x, int flags,
                                const uint8_t* wq, int64_t ldw, int fmt_w, const float* scale_w, int gran_w,
                                int64_t N, void* y, int64_t ld_y, void* workspace, size_t workspace_bytes,
                                void* stream);

/*
 * fp8_linear_fwd_prequantized for callers that cannot allocate device memory or
 * hand over a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, checks, kernels and results
 * as fp8_linear_fwd_prequantized, minus the workspace: the activation codes and
 * scales go into a buffer of FP8_STATIC_SCRATCH_BYTES bytes that lives inside the
 * library's device image (one copy per GPU, held until the process ends).  The
 * call allocates and frees nothing.  Problems whose
 * fp8_linear_prequantized_workspace_bytes(M, K) exceeds FP8_STATIC_SCRATCH_BYTES
 * are rejected with FP8_ERR_WORKSPACE before anything is launched (8 MiB: e.g.
 * 256 tokens x 28672 features, or 2048 x 4096).  All calls on one GPU share the
 * buffer, which keeps the previous call's contents (nothing in it has to start at
 * zero): calls that overlap in time on the same GPU, on different streams or from
 * different threads, race on it and must be serialised by the caller.
 */
#define FP8_STATIC_SCRATCH_BYTES (8u << 20)
int fp8_linear_fwd_prequantized_static(const void* x, int64_t M, int64_t K, int fmt_x, int gran_x, int flags,
                                       const uint8_t* wq, int64_t ldw, int fmt_w, const float* scale_w, int gran_w,
                                       int64_t N, void* y, int64_t ld_y, void* stream);

/*
 * Layer normalisation with the float8 cast fused into its epilogue: the block
 * in front of the linear layer in the paper's float8 microbenchmark (appendix
 * "Float8 Training Microbenchmarks": LayerNorm + Linear + Sigmoid), where the
 * paper leaves the fusion of the dynamic cast into the neighbouring operation
 * to the compiler.  One pass over x:
 *   mean_r = sum_c x[r,c] / cols,  var_r = sum_c (x[r,c] - mean_r)^2 / cols,
 *   h[r,c] = (x[r,c] - mean_r) / sqrt(var_r + eps) * gamma[c] + beta[c]
 *   (statistics and normalisation in binary64, h rounded once to bfloat16),
 *   then scale_out[r], q_out[r,:] = the rowwise quantization of the bfloat16 row
 *   h[r,:], exactly what fp8_quantize(FP8_ROW) gives on h (flags: FP8_POW2_SCALE).
 * x [rows, cols] bfloat16 (ld), gamma [cols] bfloat16, beta [cols] bfloat16 or
 * NULL (zero); cols a multiple of 8, at most 16384.  Outputs: q_out [rows, cols]
 * (ld_q % 16 == 0), scale_out [rows]; optional (NULL to skip): h_out [rows, cols]
 * bfloat16 (ld_h), mean_out [rows], rstd_out [rows] fp32 (for a backward pass).
 */
int fp8_layernorm_quantize(const void* x, int64_t rows, int64_t cols, int64_t ld, const void* gamma,
                           const void* beta, double eps, int format, int flags, void* h_out, int64_t ld_h,
                           uint8_t* q_out, int64_t ld_q, float* scale_out, float* mean_out, float* rstd_out,
                           void* stream);

/*
 * MX (microscaling) FP8, the finer scaling granularity that the paper lists
 * among its prototype features (Appendix E, "Prototype Features": MX formats, mxfp8 for training); format
 * and conversion follow the OCP Microscaling Formats (MX) specification v1.0:
 * every block of 32 consecutive elements along the contraction axis has one
 * power-of-two scale, stored as an E8M0 byte (value 2^(byte - 127)).
 *
 * fp8_mx_quantize: x [rows, cols] bfloat16, blocks along the columns
 *   (cols % 32 == 0).  byte = floor(log2(block maximum)) - emax(format) + 127,
 *   clamped to [0, 254] (emax = 8 for E4M3, 15 for E5M2; all-zero block: 0);
 *   q = fp8( x / 2^(byte - 127) ), round to nearest even, saturating.
 *   q_out [rows, cols] (ld_q % 16 == 0), e8m0_out [rows, cols / 32] (ld_e % 4 == 0).
 * fp8_mx_scaled_mm: out[m, n] = sum over blocks of
 *   2^(ea[m,blk]-127) * 2^(eb[n,blk]-127) * sum_{k in blk} dec(a[m,k]) * dec(b[n,k]),
 *   a [M, K], b [N, K] codes, ea [M, K/32], eb [N, K/32]; the scales are applied by
 *   the matrix-core instruction itself (v_mfma_scale_f32_16x16x128_f8f6f4).
 *   K % 128 == 0; ld_ea, ld_eb multiples of 4; out bfloat16 or fp32 (FP8_OUT_FP32).
 * fp8_mx_linear_fwd: Y = X W^T with both operands quantized per call into MX
 *   blocks along K; workspace of fp8_mx_linear_workspace_bytes(M, K, N) bytes.
 * fp8_mx_quantize_t: the same conversion with the blocks running down the
 *   columns of x [rows, cols] (rows % 32 == 0) and the result written transposed:
 *   qt_out [cols, rows] (ld_q % 16 == 0), e8m0_t_out [cols, rows / 32] (ld_e % 4 == 0),
 *   equal to fp8_mx_quantize of the transposed matrix.  It produces the
 *   contraction-contiguous operands of the backward products.
 * fp8_mx_quantize_row_col: both of the above from ONE read of x (rows % 32 == 0,
 *   cols % 32 == 0): q_row / e_row as fp8_mx_quantize writes them, q_col_t / e_col_t
 *   as fp8_mx_quantize_t does.  A tensor needed in both orientations (the gradient
 *   in the backward) costs 4 bytes of HBM traffic per element instead of 6.
 * fp8_mx_linear_bwd: dX [M, K] = dY W and dW [N, K] = dY^T X (bfloat16; either
 *   output may be NULL).  The MX specification (Section 6.2) defines the scaled
 *   dot product over blocks of the contracted index, so each operand is
 *   re-quantized from its bfloat16 original with the blocks along that product's
 *   contraction axis: dY along N and W^T along N for dX, dY^T along M and X^T
 *   along M for dW.  M % 32 == 0, N % 32 == 0 (whole blocks along both contraction
 *   axes), K % 8 == 0; dy [M, N], x [M, K], w [N, K] dense bfloat16; workspace of
 *   fp8_mx_linear_bwd_workspace_bytes bytes, 256-byte aligned.  (The products step
 *   through 128 contracted elements at a time: inside the workspace the contraction
 *   axes are padded to multiples of 128 with zero codes.)
 *
 * Layout of an array of E8M0 scale bytes (every ld_e* argument of the MX and blockwise
 * entry points): R scale rows of B = (contracted length) / 32 bytes.
 *   ld_e >= 0: plain rows, byte of block b of row r at e[r * ld_e + b]
 *     (ld_e >= B, a multiple of 4; e 4-byte aligned).
 *   ld_e <  0: slabs of sixteen blocks, e[((b / 16) * S + r) * 16 + b % 16] with
 *     S = -ld_e >= R rows per slab (B % 16 == 0, i.e. the contracted length a multiple of
 *     512; S * B < 2^31; e 16-byte aligned, S * B bytes).  FP8_E8M0_SLABS(S) spells the
 *     argument.  The 256 x 256 product kernel fetches the scales of four K steps of a row as
 *     one 16-byte piece; in slabs the pieces of consecutive rows are consecutive in
 *     memory (8 cache lines per wavefront load instead of 64).  fp8_mx_scaled_mm takes
 *     slabs for both operands or for neither (lda, ldb < 2^23 with slabs); rows
 *     between R and S are never read for output that is stored.  Same codes, same
 *     scale bytes, same products as with plain rows.
 */
#define FP8_E8M0_SLABS(rows_per_slab) (-(int64_t)(rows_per_slab))
int fp8_mx_quantize(const void* x, int64_t rows, int64_t cols, int64_t ld, int format,
                    uint8_t* q_out, int64_t ld_q, uint8_t* e8m0_out, int64_t ld_e, void* stream);
int fp8_mx_quantize_t(const void* x, int64_t rows, int64_t cols, int64_t ld, int format,
                      uint8_t* qt_out, int64_t ld_q, uint8_t* e8m0_t_out, int64_t ld_e, void* stream);
int fp8_mx_quantize_row_col(const void* x, int64_t rows, int64_t cols, int64_t ld, int format,
                            uint8_t* q_row, int64_t ld_row, uint8_t* e_row, int64_t ld_er,
                            uint8_t* q_col_t, int64_t ld_col_t, uint8_t* e_col_t, int64_t ld_ec, void* stream);
int fp8_mx_scaled_mm(const uint8_t* a, int64_t lda, int fmt_a, const uint8_t* ea, int64_t ld_ea,
                     const uint8_t* b, int64_t ldb, int fmt_b, const uint8_t* eb, int64_t ld_eb,
                     int64_t M, int64_t N, int64_t K, void* out, int64_t ld_out, int flags, void* stream);
size_t fp8_mx_linear_workspace_bytes(int64_t M, int64_t K, int64_t N);
int fp8_mx_linear_fwd(const void* x, const void* w, int64_t M, int64_t K, int64_t N, int fmt_x, int fmt_w,
                      void* y, void* workspace, size_t workspace_bytes, void* stream);
size_t fp8_mx_linear_bwd_workspace_bytes(int64_t M, int64_t K, int64_t N);
int fp8_mx_linear_bwd(const void* dy, const void* x, const void* w, int64_t M, int64_t K, int64_t N, int fmt_dy,
                      int fmt_x, int fmt_w, void* dx, void* dw, void* workspace, size_t workspace_bytes,
                      void* stream);

/*
 * Blockwise FP8 (Appendix E, the paper's list of prototype features, names the
 * blockwise FP8 quantization that DeepSeek introduced; the recipe is that of the
 * DeepSeek-V3 technical report, Section 3.3.2): activations are scaled per tile of
 * 1 x 128 elements along the contraction axis, weights per block of 128 x 128.
 * Here the scale of a block is s = fp32(FMAX / max(amax, 1e-12)) rounded DOWN to a
 * power of two, q = fp8(x * s) (round to nearest even; nothing saturates), and
 * 1 / s is stored as an E8M0 byte (127 - log2 s) in the layout of the MX scales:
 * e8m0_out [rows, cols / 32] holds the byte of a block four times per 128 columns
 * and, for 128 x 128 blocks, in every row of the block.  The operands therefore go
 * straight into fp8_mx_scaled_mm, whose matrix instruction applies the scales.
 *
 * fp8_block_quantize: x [rows, cols] bfloat16, cols % 128 == 0; block_rows = 1
 *   (tiles of 1 x 128) or 128 (blocks of 128 x 128, the last row of blocks may be
 *   partial); q_out [rows, cols] (ld_q % 16 == 0), e8m0_out (ld_e % 4 == 0).  One
 *   pass over HBM in both cases.
 * fp8_block_linear_fwd: Y = X W^T, X [M, K] in tiles of 1 x 128 along K, W [N, K] in
 *   blocks of 128 x 128; K % 128 == 0; y [M, N] bfloat16; workspace of
 *   fp8_block_linear_workspace_bytes(M, K, N) bytes, 256-byte aligned.
 * fp8_block_quantize_t: the same conversion of the TRANSPOSED matrix, written
 *   transposed: qt_out [cols, rows], e8m0_t_out [cols, rows / 32] equal
 *   fp8_block_quantize of x^T with the given block_rows (1: tiles of 128 rows x 1
 *   column of x; 128: blocks of 128 x 128, the same numbers as those of x itself).
 *   rows % 128 == 0, cols % 8 == 0.  One pass over HBM.
 * fp8_block_quantize_row_col: the tiles of 1 x 128 along the rows of x (q_row,
 *   e_row as fp8_block_quantize(block_rows = 1) writes them) and the tiles of
 *   128 x 1 down its columns, transposed (q_col_t, e_col_t as fp8_block_quantize_t
 *   (block_rows = 1) does) from ONE read of x; rows % 128 == 0, cols % 128 == 0.
 * fp8_block_linear_bwd: dX [M, K] = dY W and dW [N, K] = dY^T X (bfloat16; either
 *   may be NULL), each operand with its blocks along the contraction axis of the
 *   product it feeds: dY in tiles along N and W^T in its 128 x 128 blocks for dX;
 *   dY^T and X^T in tiles along M for dW.  M % 128 == 0, N % 128 == 0, K % 8 == 0;
 *   workspace of fp8_block_linear_bwd_workspace_bytes bytes, 256-byte aligned.
 */
int fp8_block_quantize(const void* x, int64_t rows, int64_t cols, int64_t ld, int block_rows, int format,
                       uint8_t* q_out, int64_t ld_q, uint8_t* e8m0_out, int64_t ld_e, void* stream);
size_t fp8_block_linear_workspace_bytes(int64_t M, int64_t K, int64_t N);
int fp8_block_linear_fwd(const void* x, const void* w, int64_t M, int64_t K, int64_t N, int fmt_x, int fmt_w,
                         void* y, void* workspace, size_t workspace_bytes, void* stream);
int fp8_block_quantize_t(const void* x, int64_t rows, int64_t cols, int64_t ld, int block_rows, int format,
                         uint8_t* qt_out, int64_t ld_q, uint8_t* e8m0_t_out, int64_t ld_e, void* stream);
int fp8_block_quantize_row_col(const void* x, int64_t rows, int64_t cols, int64_t ld, int format,
                               uint8_t* q_row, int64_t ld_row, uint8_t* e_row, int64_t ld_er,
                               uint8_t* q_col_t, int64_t ld_col_t, uint8_t* e_col_t, int64_t ld_ec, void* stream);
size_t fp8_block_linear_bwd_workspace_bytes(int64_t M, int64_t K, int64_t N);
int fp8_block_linear_bwd(const void* dy, const void* x, const void* w, int64_t M, int64_t K, int64_t N, int fmt_dy,
                         int fmt_x, int fmt_w, void* dx, void* dw, void* workspace, size_t workspace_bytes,
                         void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FP8MI355_H */
