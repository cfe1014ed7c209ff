/*
 * CPU oracle for the dynamically scaled float8 linear layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  It shares no code with the HIP path and
 * nothing in the product may call it.
 *
 * What it follows:
 *   - The paper's FP8 training section (Section 2.1, "FP8 Training"): the
 *     activations, weights and gradients are cast to FP8 dynamically (the
 *     statistics are recomputed from the tensor at every call) and the matrix
 *     product runs on the FP8 operands.
 *   - The paper's Appendix A (FP8 scaling recipes): "tensorwise" takes one
 *     scaling factor per tensor; "rowwise" takes one per logical row of the
 *     left GEMM operand and one per logical column of the right operand, i.e.
 *     every scale spans the contraction axis of its operand.
 *   - The paper is silent about the numeric formats.  They are the two OCP
 *     8-bit floating point formats (OFP8 specification, Section 5: E4M3 with
 *     no infinities and a single NaN mantissa pattern, E5M2 IEEE-like), with
 *     saturating round-to-nearest-even conversion.
 *
 * Floating point contract: compile with -ffp-contract=off (and no
 * -ffast-math) so that every fp32 product and sum below rounds exactly once.
 *
 * Parity pins: every exported function is pinned by tests/test_oracle_*.py
 * (closed forms, exhaustive round trips, an independent search encoder, brute
 * force, library special cases).  Not pinned ("parity unpinned"): the payload
 * and sign of NaN codes, and amax of inputs that contain NaN.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_E4M3FN 0
#define ORC_E5M2 1

#define ORC_TENSOR 0
#define ORC_ROW 1 /* one scale per row: the group runs over the columns  */
#define ORC_COL 2 /* one scale per column: the group runs over the rows  */

#define ORC_POW2_SCALE 1
#define ORC_TRANSPOSE_OUT 2

/* ---------------------------------------------------------------- helpers */

static inline uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static inline float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* bfloat16 is the upper half of an IEEE binary32: widening is exact. */
float orc_bf16_to_f32(uint16_t b) { return bits_f32((uint32_t)b << 16); }

/* binary32 -> bfloat16, round to nearest, ties to even. */
uint16_t orc_f32_to_bf16(float f) {
    uint32_t u = f32_bits(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u); /* quiet NaN */
    uint32_t lsb = (u >> 16) & 1u;
    return (uint16_t)((u + 0x7FFFu + lsb) >> 16);
}

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Format parameters (OFP8 specification, Table 1). */
static inline int fmt_mbits(int fmt) { return fmt == ORC_E4M3FN ? 3 : 2; }
static inline int fmt_bias(int fmt) { return fmt == ORC_E4M3FN ? 7 : 15; }
static inline int fmt_max_code(int fmt) { return fmt == ORC_E4M3FN ? 0x7E : 0x7B; }

float orc_fp8_max(int fmt) { return fmt == ORC_E4M3FN ? 448.0f : 57344.0f; }

/* ------------------------------------------------------------ O1: decode */
/*
 * code = S EEEE MMM (E4M3, bias 7) or S EEEEE MM (E5M2, bias 15).
 *   E == 0        : subnormal, (M / 2^mbits) * 2^(1 - bias)
 *   otherwise     : (1 + M / 2^mbits) * 2^(E - bias)
 * E4M3 has no infinity; S.1111.111 is NaN and S.1111.110 = 448 is the largest
 * finite value.  E5M2 follows IEEE: E == 31 is Inf (M == 0) or NaN.
 */
float orc_fp8_decode(uint8_t code, int fmt) {
    const int mb = fmt_mbits(fmt), bias = fmt_bias(fmt);
    const int sign = code >> 7;
    const int e = (code & 0x7F) >> mb;
    const int m = code & ((1 << mb) - 1);
    double v;
    if (fmt == ORC_E4M3FN) {
        if (e == 15 && m == 7) return sign ? -NAN : NAN;
    } else {
        if (e == 31) return m ? (sign ? -NAN : NAN) : (sign ? -INFINITY : INFINITY);
    }
    if (e == 0) v = ldexp((double)m, 1 - bias - mb);
    else        v = ldexp((double)((1 << mb) + m), e - bias - mb);
    return (float)(sign ? -v : v);
}

/* ------------------------------------------------------------ O2: encode */
/*
 * Saturating round-to-nearest-even, implementation A: the plain definition.
 * Clamp the magnitude to the largest finite value, then pick the finite
 * non-negative code whose value is nearest; on an exact tie pick the code
 * whose mantissa LSB is 0 (codes are consecutive integers, so that is the
 * even code).  The sign bit is copied from the input.
 */
uint8_t orc_fp8_encode_search(float v, int fmt) {
    const uint8_t sign = (uint8_t)((f32_bits(v) >> 24) & 0x80u);
    if (v != v) return (uint8_t)(sign | 0x7F);
    double a = fabs((double)v);
    const double fmax = (double)orc_fp8_max(fmt);
    if (a > fmax) a = fmax;
    int best = 0;
    double best_d = INFINITY;
    for (int c = 0; c <= fmt_max_code(fmt); ++c) {
        double d = fabs((double)orc_fp8_decode((uint8_t)c, fmt) - a);
        if (d < best_d || (d == best_d && (c & 1) == 0)) { best = c; best_d = d; }
    }
    return (uint8_t)(sign | best);
}

/*
 * Implementation B: the same function by integer manipulation of the
 * binary32 bits (used on large tensors).  Normal results: add half an fp8 ulp
 * minus one plus the LSB that will be kept, then truncate (classic RNE); a
 * carry out of the mantissa bumps the exponent, which is the right answer.
 * Subnormal results: adding 2^(23 + emin - mbits) in binary32 leaves the
 * RNE-rounded multiple of the subnormal step in the low mantissa bits.
 */
uint8_t orc_fp8_encode_bits(float v, int fmt) {
    const int mb = fmt_mbits(fmt), bias = fmt_bias(fmt);
    const uint32_t u = f32_bits(v);
    const uint8_t sign = (uint8_t)((u >> 24) & 0x80u);
    const uint32_t mag = u & 0x7FFFFFFFu;
    const uint32_t max_code = (uint32_t)fmt_max_code(fmt);
    if (mag > 0x7F800000u) return (uint8_t)(sign | 0x7F);
    if (mag >= f32_bits(orc_fp8_max(fmt))) return (uint8_t)(sign | max_code);
    const uint32_t min_normal_exp = (uint32_t)(127 + 1 - bias);
    uint32_t code;
    if ((mag >> 23) >= min_normal_exp) {
        const int shift = 23 - mb;
        const uint32_t lsb = (mag >> shift) & 1u;
        const uint32_t r = mag + ((1u << (shift - 1)) - 1u) + lsb;
        code = (r >> shift) - ((uint32_t)(127 - bias) << mb);
        if (code > max_code) code = max_code; /* rounded past the top: saturate */
    } else {
        const float magic = bits_f32((uint32_t)(127 + 23 + 1 - bias - mb) << 23);
        const float t = bits_f32(mag) + magic;
        code = f32_bits(t) - f32_bits(magic);
    }
    return (uint8_t)(sign | code);
}


/* Array forms of the scalar functions above (same arithmetic, one call). */
void orc_fp8_encode_array(const float* v, int64_t n, int fmt, int use_search, uint8_t* out) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        out[i] = use_search ? orc_fp8_encode_search(v[i], fmt) : orc_fp8_encode_bits(v[i], fmt);
}

void orc_f32_to_bf16_array(const float* v, int64_t n, uint16_t* out) {
    for (int64_t i = 0; i < n; ++i) out[i] = orc_f32_to_bf16(v[i]);
}

/* -------------------------------------------------------------- O3: amax */
/*
 * amax_g = max over the group of |x|, on bfloat16 values widened to binary32.
 * x is [rows, cols] with leading dimension ld (elements).
 *   TENSOR: out[1];  ROW: out[rows];  COL: out[cols].
 */
void orc_amax(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, int gran, float* out) {
    if (gran == ORC_TENSOR) {
        float m = 0.0f;
        for (int64_t r = 0; r < rows; ++r)
            for (int64_t c = 0; c < cols; ++c) {
                float a = fabsf(orc_bf16_to_f32(x[r * ld + c]));
                if (a > m) m = a;
            }
        out[0] = m;
    } else if (gran == ORC_ROW) {
#pragma omp parallel for schedule(static)
        for (int64_t r = 0; r < rows; ++r) {
            float m = 0.0f;
            for (int64_t c = 0; c < cols; ++c) {
                float a = fabsf(orc_bf16_to_f32(x[r * ld + c]));
                if (a > m) m = a;
            }
            out[r] = m;
        }
    } else {
#pragma omp parallel for schedule(static)
        for (int64_t c = 0; c < cols; ++c) {
            float m = 0.0f;
            for (int64_t r = 0; r < rows; ++r) {
                float a = fabsf(orc_bf16_to_f32(x[r * ld + c]));
                if (a > m) m = a;
            }
            out[c] = m;
        }
    }
}

/* ------------------------------------------------------------- O4: scale */
/*
 * s = FMAX / max(amax, 1e-12), the division carried out in binary64 and the
 * quotient rounded to binary32.  With POW2 the scale is rounded DOWN to a
 * power of two (mantissa cleared), so that amax * s never exceeds FMAX.
 */
void orc_scale(const float* amax, int64_t n, int fmt, int flags, float* scale) {
    const double fmax = (double)orc_fp8_max(fmt);
    for (int64_t i = 0; i < n; ++i) {
        double a = (double)amax[i];
        if (!(a > 1e-12)) a = 1e-12;
        float s = (float)(fmax / a);
        if (flags & ORC_POW2_SCALE) s = bits_f32(f32_bits(s) & 0xFF800000u);
        scale[i] = s;
    }
}

/* -------------------------------------------------------------- O5: cast */
/*
 * q = encode( fp32(x) * s ): one binary32 rounding for the product, then the
 * saturating RNE narrowing.  s is scale[0] (TENSOR), scale[r] (ROW) or
 * scale[c] (COL).  With TRANSPOSE_OUT the byte for x[r,c] goes to
 * q[c * ld_out + r], otherwise to q[r * ld_out + c].  use_search selects
 * encoder A (slow) instead of B.
 */
void orc_cast(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, const float* scale,
              int gran, int fmt, int flags, uint8_t* q, int64_t ld_out, int use_search) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t c = 0; c < cols; ++c) {
            const float s = gran == ORC_TENSOR ? scale[0] : (gran == ORC_ROW ? scale[r] : scale[c]);
            volatile float p = orc_bf16_to_f32(x[r * ld + c]) * s;
            const uint8_t code = use_search ? orc_fp8_encode_search(p, fmt) : orc_fp8_encode_bits(p, fmt);
            if (flags & ORC_TRANSPOSE_OUT) q[c * ld_out + r] = code;
            else                           q[r * ld_out + c] = code;
        }
    }
}

/* -------------------------------------------------------- O8: cast stats */
/*
 * stats[0] = n_sat       : |fp32(x) * s| > FMAX (clamped by the cast)
 * stats[1] = n_zero      : x != 0 but the code is +-0
 * stats[2] = n_subnormal : nonzero code with exponent field 0
 * stats[3] = signal power  sum x^2             (binary64)
 * stats[4] = noise power   sum (dec(q)/s - x)^2 (binary64)
 */
void orc_cast_stats(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, const float* scale,
                    int gran, int fmt, double* stats) {
    double n_sat = 0, n_zero = 0, n_sub = 0, sig = 0, noise = 0;
    const float fmax = orc_fp8_max(fmt);
    const int mb = fmt_mbits(fmt);
#pragma omp parallel for schedule(static) reduction(+ : n_sat, n_zero, n_sub, sig, noise)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t c = 0; c < cols; ++c) {
            const float s = gran == ORC_TENSOR ? scale[0] : (gran == ORC_ROW ? scale[r] : scale[c]);
            const float xv = orc_bf16_to_f32(x[r * ld + c]);
            volatile float p = xv * s;
            const uint8_t code = orc_fp8_encode_bits(p, fmt);
            if (fabsf(p) > fmax) n_sat += 1;
            if (xv != 0.0f && (code & 0x7F) == 0) n_zero += 1;
            if ((code & 0x7F) != 0 && ((code & 0x7F) >> mb) == 0) n_sub += 1;
            const double back = (double)orc_fp8_decode(code, fmt) / (double)s;
            sig += (double)xv * (double)xv;
            noise += (back - (double)xv) * (back - (double)xv);
        }
    }
    stats[0] = n_sat; stats[1] = n_zero; stats[2] = n_sub; stats[3] = sig; stats[4] = noise;
}

/* ----------------------------------------------------- O6: scaled matmul */
/*
 * a: [M, K] fp8 codes, K contiguous (leading dimension lda);
 * b: [N, K] fp8 codes, K contiguous (leading dimension ldb).
 * For the output rows listed in row_idx (or all rows when row_idx == NULL):
 *   acc[m, n]   = sum over k ascending of dec(a[m,k]) * dec(b[n,k]) in binary32
 *                 (each product of two fp8 values is exact in binary32)
 *   out32[i, n] = (acc * (1 / sa)) * (1 / sb)     in binary32
 *   out16[i, n] = bfloat16 RNE of out32
 *   acc64[i, n] = the same sum in binary64, times the reciprocal scales in
 *                 binary64 (kept for error budgeting; may be NULL)
 * sa is scale_a[0] (TENSOR) or scale_a[m] (ROW); likewise sb with n.
 * Outputs are dense [n_rows_out, N].
 */
void orc_scaled_mm(const uint8_t* a, int64_t lda, int fmt_a, const float* scale_a, int gran_a,
                   const uint8_t* b, int64_t ldb, int fmt_b, const float* scale_b, int gran_b,
                   int64_t M, int64_t N, int64_t K, const int64_t* row_idx, int64_t n_rows_out,
                   float* out32, uint16_t* out16, double* acc64) {
    float lut_a[256], lut_b[256];
    for (int c = 0; c < 256; ++c) {
        lut_a[c] = orc_fp8_decode((uint8_t)c, fmt_a);
        lut_b[c] = orc_fp8_decode((uint8_t)c, fmt_b);
    }
    const int64_t rows = row_idx ? n_rows_out : M;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        for (int64_t n = 0; n < N; ++n) {
            const int64_t m = row_idx ? row_idx[i] : i;
            const uint8_t* ar = a + m * lda;
            const uint8_t* br = b + n * ldb;
            float acc = 0.0f;
            double accd = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                const float fa = lut_a[ar[k]], fb = lut_b[br[k]];
                acc = acc + fa * fb;
                accd = accd + (double)fa * (double)fb;
            }
            const float sa = gran_a == ORC_TENSOR ? scale_a[0] : scale_a[m];
            const float sb = gran_b == ORC_TENSOR ? scale_b[0] : scale_b[n];
            const float ra = 1.0f / sa, rb = 1.0f / sb;
            const float o = (acc * ra) * rb;
            if (out32) out32[i * N + n] = o;
            if (out16) out16[i * N + n] = orc_f32_to_bf16(o);
            if (acc64) acc64[i * N + n] = accd / (double)sa / (double)sb;
        }
    }
}

/* ------------------------------------------------------------------ MX blocks
 *
 * Microscaling (the paper lists the MX formats, "mxfp8 for training", among
 * its prototype features; the format and its conversion are defined by the
 * OCP Microscaling Formats (MX) specification v1.0, Sections 5 and 6.3):
 * 32 consecutive elements along the contraction axis share one power-of-two
 * scale X stored as an E8M0 byte (value 2^(byte - 127); 255 = NaN), and the
 * elements are FP8 codes P_i with  value_i = X * dec(P_i).
 *
 * Conversion of a block V_0..V_31 (Section 6.3 of that specification):
 *   shared_exp = floor(log2(max_i |V_i|)) - emax_elem      (emax_elem = 8 for E4M3: 448 = 1.75 * 2^8,
 *                                                            15 for E5M2: 57344 = 1.75 * 2^15)
 *   X = 2^shared_exp, E8M0 byte = shared_exp + 127 clamped to [0, 254]
 *   P_i = FP8 of V_i / X, round to nearest even, magnitudes above the largest
 *         normal clamped to it (the block maximum lands in [2^emax, 2^(emax+1))
 *         before rounding, so it can round past 448 / 57344 and saturate).
 * Reading where the specification leaves a choice: an all-zero block gets the
 * byte 0 (X = 2^-127) and all-zero codes.  NaN / Inf inputs: unspecified here
 * ("parity unpinned").
 */
static int orc_emax_elem(int fmt) { return fmt == ORC_E4M3FN ? 8 : 15; }

void orc_mx_quantize(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, int fmt,
                     uint8_t* q, int64_t ld_q, uint8_t* e8m0, int64_t ld_e) {
    const int64_t nblk = cols / 32;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t b = 0; b < nblk; ++b) {
            const uint16_t* v = x + r * ld + b * 32;
            double amax = 0.0;
            for (int i = 0; i < 32; ++i) {
                const double a = fabs((double)orc_bf16_to_f32(v[i]));
                if (a > amax) amax = a;
            }
            int byte = 0;
            if (amax > 0.0) {
                int e;
                (void)frexp(amax, &e);            /* amax = f * 2^e, 0.5 <= f < 1: floor(log2 amax) = e - 1 */
                const int shared = (e - 1) - orc_emax_elem(fmt);
                byte = shared + 127;
                if (byte < 0) byte = 0;
                if (byte > 254) byte = 254;
            }
            e8m0[r * ld_e + b] = (uint8_t)byte;
            const double X = ldexp(1.0, byte - 127);
            for (int i = 0; i < 32; ++i) {
                /* V / X is exact in binary64; as a binary32 it is exact too unless it is
                 * far below the smallest FP8 subnormal, where the code is a signed zero anyway */
                const float scaled = (float)((double)orc_bf16_to_f32(v[i]) / X);
                q[r * ld_q + b * 32 + i] = orc_fp8_encode_bits(scaled, fmt);
            }
        }
    }
}

/* ------------------------------------------------------- blockwise FP8
 *
 * "Blockwise FP8: FP8 blockwise quantization introduced by DeepSeek" is on the
 * paper's list of prototype features; the paper gives no further detail.  The
 * recipe (DeepSeek-V3 technical report, Section 3.3.2 "fine-grained
 * quantization"): activations are scaled per tile of 1 x 128 elements (one
 * token, 128 channels along the contraction axis), weights per block of
 * 128 x 128, each scale chosen so that the block's amax lands on the largest
 * FP8 value, and the partial sums of every 128 contracted elements are
 * dequantized with the two block scales.
 * Readings: the scale is that of the tensorwise / rowwise recipes applied to
 * the block, s = fp32(FMAX / max(amax, 1e-12)), rounded DOWN to a power of two
 * (mantissa cleared) so that CDNA4's block-scaled matrix instruction can apply
 * its reciprocal as an E8M0 byte: byte = 127 - log2(s), dequantized value =
 * 2^(byte - 127) * dec(code).  The byte of a block is written for every row of
 * the block and every group of 32 columns in it, i.e. in the layout of the MX
 * scales ([rows, cols / 32]), so orc_mx_mm is the product of two blockwise
 * operands as well.  br x bc is the block (1 x 128 or 128 x 128; any br >= 1 and
 * bc a multiple of 32 work); blocks at the bottom edge may be partial, cols must
 * be a multiple of bc.  NaN / Inf inputs: unspecified here ("parity unpinned").
 */
void orc_block_quantize(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, int64_t br, int64_t bc, int fmt,
                        uint8_t* q, int64_t ld_q, uint8_t* e8m0, int64_t ld_e) {
    const int64_t nrb = (rows + br - 1) / br, ncb = cols / bc;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t rb = 0; rb < nrb; ++rb) {
        for (int64_t cb = 0; cb < ncb; ++cb) {
            const int64_t r0 = rb * br, r1 = r0 + br < rows ? r0 + br : rows, c0 = cb * bc;
            float amax = 0.0f;
            for (int64_t r = r0; r < r1; ++r)
                for (int64_t c = c0; c < c0 + bc; ++c) {
                    const float a = fabsf(orc_bf16_to_f32(x[r * ld + c]));
                    if (a > amax) amax = a;
                }
            float s;
            orc_scale(&amax, 1, fmt, ORC_POW2_SCALE, &s);
            int byte = 127 - ((int)(f32_bits(s) >> 23) - 127);      /* s = 2^k, k = exponent field - 127 */
            if (byte < 0) byte = 0;
            if (byte > 254) byte = 254;
            for (int64_t r = r0; r < r1; ++r) {
                for (int64_t j = 0; j < bc / 32; ++j) e8m0[r * ld_e + c0 / 32 + j] = (uint8_t)byte;
                for (int64_t c = c0; c < c0 + bc; ++c)
                    q[r * ld_q + c] = orc_fp8_encode_bits(orc_bf16_to_f32(x[r * ld + c]) * s, fmt);
            }
        }
    }
}

/* value of an MX element: X * dec(P) in binary64 (exact) */
double orc_mx_value(uint8_t code, int fmt, uint8_t e8m0) {
    return ldexp((double)orc_fp8_decode(code, fmt), (int)e8m0 - 127);
}

/*
 * MX matrix product on two block-scaled operands, both K-contiguous, blocks of
 * 32 along K (K % 32 == 0):
 *   out[m, n] = sum_blocks 2^(ea[m,blk] - 127) * 2^(eb[n,blk] - 127) * sum_{k in blk} dec(a[m,k]) * dec(b[n,k])
 * Order: products of a block summed k-ascending in binary32, scaled by the
 * (exact) power of two, blocks added in ascending order in binary32; a
 * binary64 shadow of the same sum is returned in acc64.  out16 = bfloat16 RNE.
 */
void orc_mx_mm(const uint8_t* a, int64_t lda, int fmt_a, const uint8_t* ea, int64_t ld_ea,
               const uint8_t* b, int64_t ldb, int fmt_b, const uint8_t* eb, int64_t ld_eb,
               int64_t M, int64_t N, int64_t K, const int64_t* row_idx, int64_t n_rows_out,
               float* out32, uint16_t* out16, double* acc64) {
    float lut_a[256], lut_b[256];
    for (int c = 0; c < 256; ++c) {
        lut_a[c] = orc_fp8_decode((uint8_t)c, fmt_a);
        lut_b[c] = orc_fp8_decode((uint8_t)c, fmt_b);
    }
    const int64_t rows = row_idx ? n_rows_out : M;
    const int64_t nblk = K / 32;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        for (int64_t n = 0; n < N; ++n) {
            const int64_t m = row_idx ? row_idx[i] : i;
            float acc = 0.0f;
            double accd = 0.0;
            for (int64_t blk = 0; blk < nblk; ++blk) {
                const uint8_t* ar = a + m * lda + blk * 32;
                const uint8_t* br = b + n * ldb + blk * 32;
                float p = 0.0f;
                double pd = 0.0;
                for (int k = 0; k < 32; ++k) {
                    const float fa = lut_a[ar[k]], fb = lut_b[br[k]];
                    p = p + fa * fb;
                    pd = pd + (double)fa * (double)fb;
                }
                const int e = (int)ea[m * ld_ea + blk] + (int)eb[n * ld_eb + blk] - 254;
                acc = acc + ldexpf(p, e);
                accd = accd + ldexp(pd, e);
            }
            if (out32) out32[i * N + n] = acc;
            if (out16) out16[i * N + n] = orc_f32_to_bf16(acc);
            if (acc64) acc64[i * N + n] = accd;
        }
    }
}

/*
 * High-precision linear on the unquantized bfloat16 operands (report only:
 * measures the quantization error of the fp8 path, not used for parity).
 * out[i, n] = sum_k a[m,k] * b[n,k] in binary64, a and b K-contiguous.
 */
void orc_bf16_mm_f64(const uint16_t* a, int64_t lda, const uint16_t* b, int64_t ldb,
                     int64_t M, int64_t N, int64_t K, const int64_t* row_idx, int64_t n_rows_out,
                     double* out) {
    const int64_t rows = row_idx ? n_rows_out : M;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        for (int64_t n = 0; n < N; ++n) {
            const int64_t m = row_idx ? row_idx[i] : i;
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += (double)orc_bf16_to_f32(a[m * lda + k]) * (double)orc_bf16_to_f32(b[n * ldb + k]);
            out[i * N + n] = acc;
        }
    }
}

/*
 * Round a binary64 value to bfloat16, to nearest, ties to even, in ONE rounding
 * (going through binary32 first would round twice).  Written from the format:
 * 8 exponent bits (bias 127), 7 fraction bits, subnormals with quantum 2^-133.
 */
uint16_t orc_f64_to_bf16(double d) {
    if (isnan(d)) return 0x7FC0;
    const uint16_t sign = signbit(d) ? 0x8000 : 0;
    const double a = fabs(d);
    if (a == 0.0) return sign;
    if (isinf(a)) return sign | 0x7F80;
    int e;
    (void)frexp(a, &e);                       /* a = m * 2^e, m in [0.5, 1): leading bit has weight 2^(e-1) */
    int E = e - 1;
    if (E < -126) E = -126;                   /* subnormal range: fixed quantum */
    const double quantum = ldexp(1.0, E - 7);
    const double n = rint(a / quantum);       /* exact division by a power of two; rint = ties to even */
    const double v = n * quantum;             /* representable in bfloat16 (or 2^128 = overflow) */
    if (v >= ldexp(1.0, 128)) return sign | 0x7F80;
    const float f = (float)v;                 /* exact */
    return sign | (uint16_t)(f32_bits(f) >> 16);
}

/*
 * Layer normalisation over the last axis, the operation in front of the linear
 * layer in the paper's float8 microbenchmark (appendix "Float8 Training
 * Microbenchmarks": LayerNorm + Linear + Sigmoid), whose output is what the
 * forward casts to float8.  Definition, in binary64:
 *   mean_r = sum_c x[r,c] / C;  var_r = sum_c (x[r,c] - mean_r)^2 / C   (biased)
 *   rstd_r = 1 / sqrt(var_r + eps)
 *   h[r,c] = (x[r,c] - mean_r) * rstd_r * gamma[c] + beta[c]            (beta == NULL: 0)
 * h is rounded once to bfloat16 (the tensor a bfloat16 model materialises).
 */
void orc_layernorm(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, const uint16_t* gamma,
                   const uint16_t* beta, double eps, uint16_t* h, int64_t ld_h, double* mean_out, double* rstd_out) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const uint16_t* row = x + r * ld;
        double sum = 0.0;
        for (int64_t c = 0; c < cols; ++c) sum += (double)orc_bf16_to_f32(row[c]);
        const double mean = sum / (double)cols;
        double sq = 0.0;
        for (int64_t c = 0; c < cols; ++c) {
            const double dlt = (double)orc_bf16_to_f32(row[c]) - mean;
            sq += dlt * dlt;
        }
        const double rstd = 1.0 / sqrt(sq / (double)cols + eps);
        for (int64_t c = 0; c < cols; ++c) {
            const double g = (double)orc_bf16_to_f32(gamma[c]);
            const double b = beta ? (double)orc_bf16_to_f32(beta[c]) : 0.0;
            h[r * ld_h + c] = orc_f64_to_bf16(((double)orc_bf16_to_f32(row[c]) - mean) * rstd * g + b);
        }
        if (mean_out) mean_out[r] = mean;
        if (rstd_out) rstd_out[r] = rstd;
    }
}

/*
 * Logistic function of a dequantized GEMM result, the activation behind the linear
 * layer in the same microbenchmark: y = 1 / (1 + exp(-v)) in binary64 on the fp32
 * value v, rounded once to bfloat16.
 */
void orc_sigmoid_bf16(const float* v, int64_t n, uint16_t* out) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) out[i] = orc_f64_to_bf16(1.0 / (1.0 + exp(-(double)v[i])));
}

/*
 * Gradient through the sigmoid behind the linear layer (same microbenchmark block):
 * with y = sigmoid(z) stored in bfloat16 and the incoming gradient dy in bfloat16,
 *   dz = dy * y * (1 - y),
 * evaluated in binary32, one operation at a time, left to right: t1 = dy * y (exact:
 * two 8-bit significands), t2 = 1 - y, dz = t1 * t2, then rounded to bfloat16 - the
 * tensor that the backward of the linear layer quantizes.
 */
void orc_sigmoid_bwd(const uint16_t* dy, const uint16_t* y, int64_t n, uint16_t* dz) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const float g = orc_bf16_to_f32(dy[i]), s = orc_bf16_to_f32(y[i]);
        volatile float t1 = g * s;
        volatile float t2 = 1.0f - s;
        volatile float t = t1 * t2;
        dz[i] = orc_f32_to_bf16(t);
    }
}

