// Internal launch functions behind the C ABI.  Arguments are assumed valid
// (the ABI layer checks them); every function only enqueues work on `st`.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fp8k {

hipError_t launch_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t st);

hipError_t launch_amax(const void* x, int64_t rows, int64_t cols, int64_t ld, int gran, float* out,
                       hipStream_t st);

// per-column scales of a tall matrix via a [G, cols] scratch matrix of partial
// maxima (hipErrorNotSupported: shape does not suit it, use launch_amax + launch_scale)
hipError_t launch_col_scales_two_level(const void* x, int64_t rows, int64_t cols, int64_t ld, int fmt, int flags,
                                       float* scale_out, void* scratch, size_t scratch_bytes, hipStream_t st);

// tensorwise quantization of a dense tensor in two launches (per-block maxima, then a cast that derives the
// scale itself); part: scratch for TENSOR_PARTIALS floats
constexpr int TENSOR_PARTIALS = 512;
hipError_t launch_quant_tensor(const void* x, int64_t rows, int64_t cols, int fmt, int flags, int transpose, uint8_t* q,
                               int64_t ld_out, uint8_t* q_plain, int64_t ld_plain, float* scale_out, float* part,
                               hipStream_t st);
// blockwise FP8 (tiles of 1 x 128 or blocks of 128 x 128, power-of-two scales as E8M0 bytes in the MX layout)
hipError_t launch_block_quant(const void* x, int64_t rows, int64_t cols, int64_t ld, int block_rows, int fmt, uint8_t* q,
                              int64_t ld_q, uint8_t* e8m0, int64_t ld_e, hipStream_t st);
// the same of the transposed matrix, written transposed (rows % 128 == 0, cols % 8 == 0)
// q_row / e_row (optional, block_rows == 1, cols % 128 == 0): the tiles along the rows of x from the same read
hipError_t launch_block_quant_t(const void* x, int64_t rows, int64_t cols, int64_t ld, int block_rows, int fmt, uint8_t* qt,
                                int64_t ld_t, uint8_t* et, int64_t ld_e, hipStream_t st, uint8_t* q_row = nullptr,
                                int64_t ld_row = 0, uint8_t* e_row = nullptr, int64_t ld_er = 0);
hipError_t launch_scale(const float* amax, int64_t n, int fmt, int flags, float* out, hipStream_t st);

// transpose != 0: q is [cols, rows]; q_plain (optional, transpose only) also
// receives the untransposed codes.
hipError_t launch_cast(const void* x, int64_t rows, int64_t cols, int64_t ld, const float* scale, int gran,
                       int fmt, int transpose, uint8_t* q, int64_t ld_out, uint8_t* q_plain, int64_t ld_plain,
                       hipStream_t st);

// single-pass rowwise amax+scale+cast; hipErrorNotSupported if a row is too
// long to keep in registers.
hipError_t launch_quant_row(const void* x, int64_t rows, int64_t cols, int64_t ld, int fmt, int flags, uint8_t* q,
                            int64_t ld_out, float* scale_out, hipStream_t st);

// out[M,N] = (a[M,K] . b[N,K]^T) / (sa * sb); scale_a/scale_b have one entry
// (row_a / row_b == 0) or one per row.
hipError_t launch_gemm_fp8(const uint8_t* a, int64_t lda, int fmt_a, const float* scale_a, int row_a,
                           const uint8_t* b, int64_t ldb, int fmt_b, const float* scale_b, int row_b,
                           int64_t M, int64_t N, int64_t K, void* out, int64_t ld_out, int out_f32,
                           hipStream_t st);
// one scaled product out[M, N] = A[M, K] . B[N, K]^T / (scale_a * scale_b), operands as for launch_gemm_fp8
struct GemmOperands {
    const uint8_t* a; int64_t lda; const float* scale_a;
    const uint8_t* b; int64_t ldb; const float* scale_b;
    int64_t M, N, K; void* out; int64_t ld_out;
};
// two small products (bfloat16 results) in one launch; hipErrorNotSupported, with nothing launched, where that does not pay
hipError_t launch_gemm_fp8_pair(const GemmOperands& g1, const GemmOperands& g2, int fmt_a, int fmt_b, int row_a, int row_b,
                                hipStream_t st);

// Rowwise quantization (codes q, scales scale_out) and the per-column scales
// scale_cols[c] = scale(max_r |x[r, c]|) from a single read of x; scratch holds
// the first-level column maxima.  hipErrorNotSupported if the shape does not suit.
hipError_t launch_quant_row_colmax(const void* x, int64_t rows, int64_t cols, int64_t ld, int fmt, int flags,
                                   uint8_t* q, int64_t ld_out, float* scale_out, float* scale_cols, void* scratch,
                                   size_t scratch_bytes, hipStream_t st);

// a dense tensor [rows, cols] for tensorwise quantization: codes q (transposed [cols, rows] if asked for, then
// optionally also untransposed in q_plain), its scale, and room for TENSOR_PARTIALS floats of per-block maxima
struct TensorOperand {
    const void* x; int64_t rows;
    uint8_t* q; int64_t ld_out; uint8_t* q_plain; int64_t ld_plain; float* scale_out; float* part;
};
// two dense tensors of the same width and format, tensorwise: two launches (instead of four)
hipError_t launch_quant_tensor_pair(const TensorOperand& a, const TensorOperand& b, int64_t cols, int fmt, int flags,
                                    int transpose, hipStream_t st);

// Paired launches: the quantizations of a linear layer come in twos and threes of the same kind; these issue them as
// twin launches (one grid, two problems) with one second-level launch for all column scales.  Results are those of the
// single-tensor functions.  hipErrorNotSupported (nothing launched): a tensor does not suit - quantize one by one.
// fold (optional): quant_fold_bytes(rows, cols) bytes of side storage, 256-byte aligned, for the first-level column
// maxima.  With it the transposing cast derives the column scales itself (one launch less); without it, or where
// quant_fold_bytes is 0, the maxima are parked in the transposed output and a second-level launch reduces them.
constexpr int64_t FOLD_ROWS = 256;
int64_t quant_fold_bytes(int64_t rows, int64_t cols);
struct RowColOperand {      // a tensor [rows, cols] quantized per row (q_row, scale_row) and per column, transposed (q_col_t [cols, rows], scale_col)
    const void* x; int64_t rows, ld;
    uint8_t* q_row; int64_t ld_row; float* scale_row;
    uint8_t* q_col_t; int64_t ld_col_t; float* scale_col;
    void* fold = nullptr;
};
struct ColOperand {         // a tensor [rows, cols] quantized per column, transposed
    const void* x; int64_t rows, ld;
    uint8_t* q_col_t; int64_t ld_col_t; float* scale_col;
    void* fold = nullptr;
};
// two tensors of the same width and format, rowwise: one launch
hipError_t launch_quant_row_pair(const void* x1, int64_t rows1, int64_t ld1, uint8_t* q1, int64_t ld_q1, float* s1, const void* x2,
                                 int64_t rows2, int64_t ld2, uint8_t* q2, int64_t ld_q2, float* s2, int64_t cols, int fmt,
                                 int flags, hipStream_t st);
// one tensor (b == nullptr) or two of the same width and format along both axes: three launches, two with folding
hipError_t launch_quant_row_col_pair(const RowColOperand& a, const RowColOperand* b, int64_t cols, int fmt, int flags, hipStream_t st);
// two tensors of the same width and format per column, transposed: three launches (instead of six)
hipError_t launch_quant_col_t_pair(const ColOperand& a, const ColOperand& b, int64_t cols, int fmt, int flags, hipStream_t st);
// the backward of the rowwise recipe: the gradient g along both axes, W and X per column: five launches (instead of nine), four with folding
hipError_t launch_quant_bwd_rowwise(const RowColOperand& g, int64_t cols_g, int fmt_g, const ColOperand& w, const ColOperand& x,
                                    int64_t cols_wx, int fmt_wx, int flags, hipStream_t st);

// 256 x 256 kernel on 16x16x128 MFMAs with LDS-DMA loads and the four-phase "snake" schedule; same contract.
// _fits: its 32-bit buffer offsets reach (leading dimensions below 2^23)
bool gemm_fp8_snake_fits(int64_t lda, int64_t ldb);
// act != 0 (bfloat16 output only): the logistic function applied to the fp32 result before rounding
hipError_t launch_gemm_fp8_snake(const uint8_t* a, int64_t lda, int fmt_a, const float* scale_a, int row_a,
                                 const uint8_t* b, int64_t ldb, int fmt_b, const float* scale_b, int row_b,
                                 int64_t M, int64_t N, int64_t K, void* out, int64_t ld_out, int out_f32,
                                 hipStream_t st, int act = 0);

// persistent form of the same kernel (gemm_fp8_stream.hip): one workgroup per CU walks many tiles, the epilogue of a
// tile is drained inside the K steps of the next.  bfloat16 output, whole tiles [0, units) of the snake kernel's tile
// order; _fits: shapes it takes (N % 8 == 0, more than two K steps, 32-bit offsets reach)
bool gemm_fp8_stream_fits(int64_t lda, int64_t ldb, int64_t ld_out, int64_t N, int64_t K, int out_f32, int act);
// tile_m: 256 (tiles [0, units) of the snake kernel's tile order) or 224 / 192 (then units must be the whole tile count
// of the problem cut into tiles of that height); gemm_fp8_stream_tile_m picks the height for an [M, N] output
int gemm_fp8_stream_tile_m(int64_t M, int64_t N);
hipError_t launch_gemm_fp8_stream(const uint8_t* a, int64_t lda, int fmt_a, const float* scale_a, int row_a,
                                  const uint8_t* b, int64_t ldb, int fmt_b, const float* scale_b, int row_b,
                                  int64_t M, int64_t N, int64_t K, void* out, int64_t ld_out, int64_t units, int tile_m,
                                  hipStream_t st);

// few rows of A (M <= 64, the decode shape of inference): B is streamed once
// from HBM by wavefronts that load their MFMA operands straight from global
// memory; same contract otherwise.
hipError_t launch_gemm_fp8_skinny(const uint8_t* a, int64_t lda, int fmt_a, const float* scale_a, int row_a,
                                  const uint8_t* b, int64_t ldb, int fmt_b, const float* scale_b, int row_b,
                                  int64_t M, int64_t N, int64_t K, void* out, int64_t ld_out, int out_f32,
                                  hipStream_t st);

// y[M, N] = fp8(x * s_x)[M, K] . b[N, K]^T / (s_x * scale_b) for up to 16 rows of bfloat16 x, in one launch: the amax of
// x (per row if row_x, else of the whole tensor), its scale (flags: FLAG_POW2) and the cast happen inside the
// few-row product.  hipErrorNotSupported (nothing launched) where that form does not apply.
hipError_t launch_linear_skinny_fused(const void* x, int64_t ldx, int fmt_x, int row_x, int flags, const uint8_t* b,
                                      int64_t ldb, int fmt_b, const float* scale_b, int row_b, int64_t M, int64_t N,
                                      int64_t K, void* out, int64_t ld_out, hipStream_t st);

// bfloat16 GEMM with the contraction on the rows of both operands:
// out[I, J] = a[C, I]^T b[C, J], fp32 accumulate, bfloat16 out (the weight gradient
// dW = dY^T X kept in high precision).  I, J and the leading dimensions are
// multiples of 8 elements, pointers 16-byte aligned.
hipError_t launch_gemm_bf16_at_b(const void* a, int64_t lda, const void* b, int64_t ldb, int64_t I, int64_t J, int64_t C,
                                 void* out, int64_t ld_out, hipStream_t st);

// the same product on the LDS-DMA "snake" schedule with transposing LDS reads (large problems;
// _fits tells whether the 32-bit buffer offsets reach)
bool gemm_bf16_at_b_snake_fits(int64_t lda, int64_t ldb, int64_t I, int64_t J, int64_t C);
hipError_t launch_gemm_bf16_at_b_snake(const void* a, int64_t lda, const void* b, int64_t ldb, int64_t I, int64_t J,
                                       int64_t C, void* out, int64_t ld_out, hipStream_t st);

// gradient through a stored sigmoid output, dz = dy * y * (1 - y): quantized along both axes without being
// materialised (hipErrorNotSupported for shapes the fused kernels do not take), or materialised (dense bf16)
hipError_t launch_quant_row_col_sigmoid_bwd(const void* dy, const void* y, int64_t rows, int64_t cols, int64_t ld,
                                            int fmt, int flags, uint8_t* q_row, int64_t ld_row, float* scale_row,
                                            uint8_t* q_col_t, int64_t ld_col_t, float* scale_col, hipStream_t st);
hipError_t launch_sigmoid_bwd(const void* dy, const void* y, int64_t n, void* dz, hipStream_t st);

// layer normalisation over the rows with the rowwise fp8 quantization of its bfloat16 result fused in
// (cols % 8 == 0, cols <= 16384, else hipErrorNotSupported; h, mean_out, rstd_out optional)
hipError_t launch_layernorm_quant_row(const void* x, int64_t rows, int64_t cols, int64_t ld, const void* gamma,
                                      const void* beta, double eps, int fmt, int flags, void* h, int64_t ld_h, uint8_t* q,
                                      int64_t ld_q, float* scale_out, float* mean_out, float* rstd_out, hipStream_t st);

// MX (microscaling) FP8: blocks of 32 along the contiguous axis, one E8M0 byte per block
// (cols % 32 == 0), and the GEMM whose matrix-core instruction applies the block scales
// (K % 128 == 0, ld_ea and ld_eb multiples of 4, 4-byte aligned scale pointers)
hipError_t launch_mx_quant(const void* x, int64_t rows, int64_t cols, int64_t ld, int fmt, uint8_t* q, int64_t ld_q,
                           uint8_t* e8m0, int64_t ld_e, hipStream_t st);
// blocks of 32 down the columns of x (rows % 32 == 0), output transposed: qt [cols, rows], et [cols, rows / 32];
// with q_row != nullptr also the blocks along the rows (cols % 32 == 0) from the same read: q_row [rows, cols],
// e_row [rows, cols / 32] (ld_er % 4 == 0)
hipError_t launch_mx_quant_t(const void* x, int64_t rows, int64_t cols, int64_t ld, int fmt, uint8_t* qt, int64_t ld_t,
                             uint8_t* et, int64_t ld_e, uint8_t* q_row, int64_t ld_row, uint8_t* e_row, int64_t ld_er,
                             hipStream_t st);
bool gemm_mxfp8_takes_slab_scales(int64_t lda, int64_t ldb, int64_t M, int64_t N, int64_t K);
hipError_t launch_gemm_mxfp8(const uint8_t* a, int64_t lda, int fmt_a, const uint8_t* ea, int64_t ld_ea,
                             const uint8_t* b, int64_t ldb, int fmt_b, const uint8_t* eb, int64_t ld_eb, int64_t M,
                             int64_t N, int64_t K, void* out, int64_t ld_out, int out_f32, hipStream_t st);
// the same product on the LDS-DMA "snake" schedule (large problems; leading dimensions below 2^23)
hipError_t launch_gemm_mxfp8_snake(const uint8_t* a, int64_t lda, int fmt_a, const uint8_t* ea, int64_t ld_ea,
                                   const uint8_t* b, int64_t ldb, int fmt_b, const uint8_t* eb, int64_t ld_eb, int64_t M,
                                   int64_t N, int64_t K, void* out, int64_t ld_out, int out_f32, hipStream_t st);

}  // namespace fp8k
