/*
 * Sanitizer driver for the CPU oracle (test infrastructure, like the oracle itself).
 *
 * Built together with fp8_oracle.c under -fsanitize=address,undefined by
 * tests/test_oracle_sanitizers.py and run as a plain executable: every exported
 * function of the oracle is called on small, ragged problems whose buffers are
 * heap blocks of exactly the documented size (padded leading dimensions, row
 * subsets, transposed outputs, partial bottom blocks), so that any access outside
 * them, any misaligned or overflowing arithmetic, aborts the run.  The values are
 * not checked here - the pins in tests/test_oracle_*.py do that.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

float orc_bf16_to_f32(uint16_t b);
uint16_t orc_f32_to_bf16(float f);
int orc_num_threads(void);
float orc_fp8_max(int fmt);
float orc_fp8_decode(uint8_t code, int fmt);
uint8_t orc_fp8_encode_search(float v, int fmt);
uint8_t orc_fp8_encode_bits(float v, int fmt);
void orc_fp8_encode_array(const float* v, int64_t n, int fmt, int use_search, uint8_t* out);
void orc_f32_to_bf16_array(const float* v, int64_t n, uint16_t* out);
void orc_amax(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, int gran, float* out);
void orc_scale(const float* amax, int64_t n, int fmt, int flags, float* scale);
void orc_cast(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, const float* scale, int gran, int fmt, int flags,
              uint8_t* q, int64_t ld_out, int use_search);
void orc_cast_stats(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, const float* scale, int gran, int fmt,
                    double* stats);
void orc_scaled_mm(const uint8_t* a, int64_t lda, int fmt_a, const float* scale_a, int gran_a, const uint8_t* b, int64_t ldb,
                   int fmt_b, const float* scale_b, int gran_b, int64_t M, int64_t N, int64_t K, const int64_t* row_idx,
                   int64_t n_rows_out, float* out32, uint16_t* out16, double* acc64);
void orc_mx_quantize(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, int fmt, uint8_t* q, int64_t ld_q,
                     uint8_t* e8m0, int64_t ld_e);
void orc_block_quantize(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, int64_t br, int64_t bc, int fmt, uint8_t* q,
                        int64_t ld_q, uint8_t* e8m0, int64_t ld_e);
double orc_mx_value(uint8_t code, int fmt, uint8_t e8m0);
void orc_mx_mm(const uint8_t* a, int64_t lda, int fmt_a, const uint8_t* ea, int64_t ld_ea, const uint8_t* b, int64_t ldb,
               int fmt_b, const uint8_t* eb, int64_t ld_eb, int64_t M, int64_t N, int64_t K, const int64_t* row_idx,
               int64_t n_rows_out, float* out32, uint16_t* out16, double* acc64);
void orc_bf16_mm_f64(const uint16_t* a, int64_t lda, const uint16_t* b, int64_t ldb, int64_t M, int64_t N, int64_t K,
                     const int64_t* row_idx, int64_t n_rows_out, double* out);
uint16_t orc_f64_to_bf16(double d);
void orc_layernorm(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, const uint16_t* gamma, const uint16_t* beta,
                   double eps, uint16_t* h, int64_t ld_h, double* mean_out, double* rstd_out);
void orc_sigmoid_bf16(const float* v, int64_t n, uint16_t* out);
void orc_sigmoid_bwd(const uint16_t* dy, const uint16_t* y, int64_t n, uint16_t* dz);

enum { E4M3 = 0, E5M2 = 1, TENSOR = 0, ROW = 1, COL = 2, POW2 = 1, TRANSPOSE = 2 };

static uint32_t rng_state = 12345u;
static uint32_t rnd(void) { rng_state = rng_state * 1664525u + 1013904223u; return rng_state >> 8; }
static float rnd_float(void) {          /* wide dynamic range, both signs, some zeros */
    const uint32_t r = rnd();
    if ((r & 63u) == 0) return 0.0f;
    const float m = (float)(rnd() & 0xFFFF) / 65536.0f + 0.5f;
    return ldexpf((r & 1u) ? m : -m, (int)((r >> 1) % 40u) - 24);
}
static void* must(size_t n) { void* p = malloc(n ? n : 1); if (!p) { perror("malloc"); exit(2); } return p; }

/* bfloat16 matrix [rows, cols] with leading dimension ld, allocated with exactly (rows - 1) * ld + cols elements */
static uint16_t* bf16_matrix(int64_t rows, int64_t cols, int64_t ld) {
    const int64_t n = rows > 0 ? (rows - 1) * ld + cols : 0;
    uint16_t* x = must(sizeof(uint16_t) * (size_t)n);
    for (int64_t i = 0; i < n; ++i) x[i] = orc_f32_to_bf16(rnd_float());
    return x;
}

static void quantization_case(int64_t rows, int64_t cols, int64_t ld, int fmt) {
    uint16_t* x = bf16_matrix(rows, cols, ld);
    const int64_t groups[3] = {1, rows, cols};
    for (int gran = TENSOR; gran <= COL; ++gran) {
        float* am = must(sizeof(float) * (size_t)groups[gran]);
        float* sc = must(sizeof(float) * (size_t)groups[gran]);
        orc_amax(x, rows, cols, ld, gran, am);
        for (int flags = 0; flags <= POW2; ++flags) {
            orc_scale(am, groups[gran], fmt, flags, sc);
            for (int tr = 0; tr <= 1; ++tr) {
                const int64_t orows = tr ? cols : rows, ocols = tr ? rows : cols, ld_out = ocols + 3;
                uint8_t* q = must((size_t)((orows - 1) * ld_out + ocols));
                orc_cast(x, rows, cols, ld, sc, gran, fmt, tr ? TRANSPOSE : 0, q, ld_out, tr);
                free(q);
            }
            double st[5];
            orc_cast_stats(x, rows, cols, ld, sc, gran, fmt, st);
        }
        free(am);
        free(sc);
    }
    free(x);
}

static uint8_t* codes(int64_t rows, int64_t cols, int64_t ld, int fmt) {
    uint8_t* c = must((size_t)((rows - 1) * ld + cols));
    const int top = fmt == E4M3 ? 0x7E : 0x7B;
    for (int64_t i = 0; i < (rows - 1) * ld + cols; ++i) c[i] = (uint8_t)((rnd() % (uint32_t)(top + 1)) | ((rnd() & 1u) << 7));
    return c;
}

static void gemm_case(int64_t M, int64_t N, int64_t K, int fa, int fb, int ga, int gb) {
    const int64_t lda = K + 5, ldb = K + 16;
    uint8_t *a = codes(M, K, lda, fa), *b = codes(N, K, ldb, fb);
    const int64_t na = ga == TENSOR ? 1 : M, nb = gb == TENSOR ? 1 : N;
    float *sa = must(sizeof(float) * (size_t)na), *sb = must(sizeof(float) * (size_t)nb);
    for (int64_t i = 0; i < na; ++i) sa[i] = 0.5f + (float)(rnd() & 255);
    for (int64_t i = 0; i < nb; ++i) sb[i] = 0.25f + (float)(rnd() & 63);
    /* all rows, then a subset in arbitrary order, with and without the binary64 shadow */
    float* o32 = must(sizeof(float) * (size_t)(M * N));
    uint16_t* o16 = must(sizeof(uint16_t) * (size_t)(M * N));
    double* a64 = must(sizeof(double) * (size_t)(M * N));
    orc_scaled_mm(a, lda, fa, sa, ga, b, ldb, fb, sb, gb, M, N, K, NULL, M, o32, o16, a64);
    const int64_t nr = M > 2 ? 2 : 1;
    int64_t idx[2] = {M - 1, 0};
    orc_scaled_mm(a, lda, fa, sa, ga, b, ldb, fb, sb, gb, M, N, K, idx, nr, o32, o16, NULL);
    free(o32); free(o16); free(a64); free(sa); free(sb); free(a); free(b);
}

static void mx_case(int64_t M, int64_t N, int64_t K, int fmt) {
    /* MX and blockwise quantization (K a multiple of 128 here so that both apply), then the block-scaled product */
    const int64_t ldx = K + 8, ldq = K + 16, lde = K / 32 + 4;
    uint16_t *x = bf16_matrix(M, K, ldx), *w = bf16_matrix(N, K, ldx);
    uint8_t *xq = must((size_t)((M - 1) * ldq + K)), *wq = must((size_t)((N - 1) * ldq + K));
    uint8_t *xe = must((size_t)((M - 1) * lde + K / 32)), *we = must((size_t)((N - 1) * lde + K / 32));
    orc_mx_quantize(x, M, K, ldx, fmt, xq, ldq, xe, lde);
    orc_mx_quantize(w, N, K, ldx, fmt, wq, ldq, we, lde);
    float* o32 = must(sizeof(float) * (size_t)(M * N));
    uint16_t* o16 = must(sizeof(uint16_t) * (size_t)(M * N));
    double* a64 = must(sizeof(double) * (size_t)(M * N));
    orc_mx_mm(xq, ldq, fmt, xe, lde, wq, ldq, fmt, we, lde, M, N, K, NULL, M, o32, o16, a64);
    int64_t idx[1] = {M - 1};
    orc_mx_mm(xq, ldq, fmt, xe, lde, wq, ldq, fmt, we, lde, M, N, K, idx, 1, o32, o16, NULL);
    orc_block_quantize(x, M, K, ldx, 1, 128, fmt, xq, ldq, xe, lde);          /* tiles of 1 x 128 */
    orc_block_quantize(w, N, K, ldx, 128, 128, fmt, wq, ldq, we, lde);        /* 128 x 128, partial bottom block */
    orc_mx_mm(xq, ldq, fmt, xe, lde, wq, ldq, fmt, we, lde, M, N, K, NULL, M, o32, o16, a64);
    double* f64 = must(sizeof(double) * (size_t)(M * N));
    orc_bf16_mm_f64(x, ldx, w, ldx, M, N, K, NULL, M, f64);
    orc_bf16_mm_f64(x, ldx, w, ldx, M, N, K, idx, 1, f64);
    free(f64); free(o32); free(o16); free(a64); free(xq); free(wq); free(xe); free(we); free(x); free(w);
}

static void elementwise_case(int64_t rows, int64_t cols) {
    const int64_t ld = cols + 8;
    uint16_t *x = bf16_matrix(rows, cols, ld), *gamma = bf16_matrix(1, cols, cols), *beta = bf16_matrix(1, cols, cols);
    uint16_t* h = must(sizeof(uint16_t) * (size_t)((rows - 1) * ld + cols));
    double *mean = must(sizeof(double) * (size_t)rows), *rstd = must(sizeof(double) * (size_t)rows);
    orc_layernorm(x, rows, cols, ld, gamma, beta, 1e-5, h, ld, mean, rstd);
    orc_layernorm(x, rows, cols, ld, gamma, NULL, 0.0, h, ld, NULL, NULL);
    const int64_t n = rows * cols;
    float* v = must(sizeof(float) * (size_t)n);
    for (int64_t i = 0; i < n; ++i) v[i] = rnd_float() * 64.0f;
    uint16_t *y = must(sizeof(uint16_t) * (size_t)n), *dz = must(sizeof(uint16_t) * (size_t)n);
    orc_sigmoid_bf16(v, n, y);
    orc_f32_to_bf16_array(v, n, dz);
    orc_sigmoid_bwd(dz, y, n, dz);
    uint8_t* c = must((size_t)n);
    orc_fp8_encode_array(v, n, E4M3, 0, c);
    orc_fp8_encode_array(v, n, E5M2, 1, c);
    free(c); free(v); free(y); free(dz); free(mean); free(rstd); free(h); free(x); free(gamma); free(beta);
}

int main(void) {
    /* scalar functions over every code and the special values */
    const float specials[] = {0.0f, -0.0f, 448.0f, 449.0f, 464.0f, 470.0f, 57344.0f, 6e4f, 1e30f, -1e30f, INFINITY, -INFINITY,
                              NAN, 0x1p-10f, 0x1p-17f, 0x1p-149f, -0x1p-149f, 3.4e38f};
    double sink = 0.0;
    for (int fmt = E4M3; fmt <= E5M2; ++fmt) {
        sink += orc_fp8_max(fmt);
        for (int c = 0; c < 256; ++c) {
            const float v = orc_fp8_decode((uint8_t)c, fmt);
            sink += (double)orc_fp8_encode_search(v, fmt) + (double)orc_fp8_encode_bits(v, fmt);
            sink += orc_mx_value((uint8_t)c, fmt, (uint8_t)c) > 0.0 ? 1.0 : 0.0;
        }
        for (size_t i = 0; i < sizeof(specials) / sizeof(specials[0]); ++i)
            sink += (double)orc_fp8_encode_search(specials[i], fmt) + (double)orc_fp8_encode_bits(specials[i], fmt);
    }
    for (uint32_t b = 0; b < 65536u; b += 7u) sink += (double)orc_f32_to_bf16(orc_bf16_to_f32((uint16_t)b));
    const double f64s[] = {0.0, 1.0, -1.0, 1.00390625, 3.3895313892515355e38, 1e-45, -1e-320, 1e300, (double)INFINITY, (double)NAN};
    for (size_t i = 0; i < sizeof(f64s) / sizeof(f64s[0]); ++i) sink += (double)orc_f64_to_bf16(f64s[i]);

    for (int fmt = E4M3; fmt <= E5M2; ++fmt) {
        quantization_case(1, 1, 8, fmt);
        quantization_case(7, 33, 40, fmt);
        quantization_case(130, 17, 24, fmt);
        mx_case(5, 3, 128, fmt);
        mx_case(131, 130, 256, fmt);
    }
    gemm_case(3, 5, 7, E4M3, E4M3, TENSOR, TENSOR);
    gemm_case(33, 17, 256, E5M2, E4M3, ROW, ROW);
    gemm_case(1, 40, 16, E4M3, E5M2, ROW, TENSOR);
    elementwise_case(1, 8);
    elementwise_case(9, 200);
    printf("sanitize_check ok (threads %d, sink %g)\n", orc_num_threads(), sink != sink ? 0.0 : 1.0);
    return 0;
}
