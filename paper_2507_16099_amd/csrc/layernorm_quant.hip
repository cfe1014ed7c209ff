// Layer normalisation with the float8 cast fused into its epilogue: the block in
// front of the linear layer in the paper's float8 microbenchmark (appendix
// "Float8 Training Microbenchmarks": LayerNorm + Linear + Sigmoid), where the
// paper relies on torch.compile to fuse the dynamic cast into the neighbouring
// operation.  Here the fusion is done by hand: ONE pass over x produces
//   h = LayerNorm(x) * gamma + beta      (bfloat16, optional output),
//   the rowwise scale of h and its fp8 codes (what fp8_quantize(ROW) would give),
// for 2 bytes read and 1 (+2 with h) written per element, instead of 2 + 2 for the
// normalisation followed by 2 + 1 for the quantization.
//
// A row lives in registers between the three reductions (sum, sum of squared
// deviations, amax of the normalised row).  The fp8 codes are integers decided
// by a floating-point reduction, so the statistics and the normalisation are
// computed in binary64 and h is rounded ONCE to bfloat16 (through a binary32
// value, see f64_to_bf16_bits): whatever the summation order, the bfloat16 result is the
// correctly rounded one except when the binary64 value lies within ~1e-16 of a
// rounding boundary (the bit-parity with a reference that sums in another order is
// therefore statistical, not by construction).  The binary64 work makes the kernel
// ALU-bound: about 38 instructions per element, measured at 0.45 of the HBM rate
// that its 5 bytes per element would allow.
#include "fp8_device.hpp"
#include "launchers.hpp"

namespace fp8k {

// binary64 -> bfloat16 bits, round to nearest even in ONE rounding.  Rounding to binary32 first is
// harmless unless the binary32 value lands exactly on a bfloat16 tie (low half 0x8000) that the
// binary64 value was not on: rounding is monotone and every tie is a binary32 number, so in all other
// cases both values lie on the same side of every tie.  In that one case the side is decided by
// comparing the magnitudes.
__device__ __forceinline__ uint32_t f64_to_bf16_bits(double d) {
    const float f = (float)d;
    const double back = (double)f;
    const uint32_t b = __float_as_uint(f);
    const uint32_t rne = (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
    const uint32_t alt = (b >> 16) + (fabs(d) > fabs(back) ? 1u : 0u);
    return ((b & 0xFFFFu) == 0x8000u && back != d) ? alt : rne;
}

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// TX threads per row (64: one wavefront, four rows per block; 256: the block), NV 128-bit vectors per thread
template <int FMT, int TX, int NV>
__global__ __launch_bounds__(256) void layernorm_quant_row_kernel(
    const uint16_t* __restrict__ x, int64_t rows, int64_t cols, int64_t ld, const uint16_t* __restrict__ gamma,
    const uint16_t* __restrict__ beta, double eps, int flags, uint16_t* __restrict__ h, int64_t ld_h,
    uint8_t* __restrict__ q, int64_t ld_q, float* __restrict__ scale_out, float* __restrict__ mean_out,
    float* __restrict__ rstd_out) {
    constexpr int TY = 256 / TX;
    const int tx = threadIdx.x % TX, ty = threadIdx.x / TX;
    const int64_t r = (int64_t)blockIdx.x * TY + ty;
    const bool live = r < rows;
    const int64_t nvec = cols >> 3;                      // cols % 8 == 0
    const uint4* rv = reinterpret_cast<const uint4*>(x + (live ? r : 0) * ld);
    __shared__ double red_sum[4], red_sq[4], bc_stat[2];
    __shared__ uint32_t red_max[4];
    __shared__ float bc_scale;
    // The per-row scalar work (two divisions and a square root in binary64, the scale's division) is a
    // few hundred instructions per WAVEFRONT whatever the number of active lanes; with four wavefronts
    // per row it would cost as much as the row's element-wise work, so wavefront 0 does it alone and
    // hands the result to the others through LDS.
    const bool wave0 = (threadIdx.x >> 6) == 0;

    uint4 v[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int64_t vi = tx + (int64_t)j * TX;
        v[j] = (live && vi < nvec) ? load_stream(rv + vi) : make_uint4(0, 0, 0, 0);
    }
    auto block_sum = [&](double part, double* red) {
        double s = wave_sum_f64(part);
        if constexpr (TX > 64) {
            if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
            __syncthreads();
            s = (red[0] + red[1]) + (red[2] + red[3]);
        }
        return s;
    };
    auto elem = [&](const uint4& w, int e) -> double {
        const uint32_t word = e < 2 ? w.x : (e < 4 ? w.y : (e < 6 ? w.z : w.w));
        return (double)((e & 1) ? bf16_hi(word) : bf16_lo(word));
    };

    // mean (zeros of the padding lanes add nothing)
    double part = 0.0;
#pragma unroll
    for (int j = 0; j < NV; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) part += elem(v[j], e);
    double mean;
    {
        const double total = block_sum(part, red_sum);
        if constexpr (TX > 64) {
            if (wave0) {
                const double m_ = total / (double)cols;
                if (threadIdx.x == 0) bc_stat[0] = m_;
            }
            __syncthreads();
            mean = bc_stat[0];
        } else {
            mean = total / (double)cols;
        }
    }
    // biased variance from the deviations (second pass over the registers)
    part = 0.0;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int64_t vi = tx + (int64_t)j * TX;
        if (vi < nvec) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const double dlt = elem(v[j], e) - mean;
                part += dlt * dlt;
            }
        }
    }
    double rstd;
    {
        const double total = block_sum(part, red_sq);
        if constexpr (TX > 64) {
            if (wave0) {
                const double r_ = 1.0 / sqrt(total / (double)cols + eps);
                if (threadIdx.x == 0) bc_stat[1] = r_;
            }
            __syncthreads();
            rstd = bc_stat[1];
        } else {
            rstd = 1.0 / sqrt(total / (double)cols + eps);
        }
    }

    // normalise, affine, one rounding to bfloat16; the bfloat16 row replaces x in the registers
    uint32_t acc = 0;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int64_t vi = tx + (int64_t)j * TX;
        uint4 hv = make_uint4(0, 0, 0, 0);
        if (vi < nvec) {
            const uint4 g4 = reinterpret_cast<const uint4*>(gamma)[vi];
            const uint4 b4 = beta ? reinterpret_cast<const uint4*>(beta)[vi] : make_uint4(0, 0, 0, 0);
            uint32_t hb[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                // ((x - mean) * rstd) * gamma + beta, every operation rounded by itself (no contraction)
                const double t = __dmul_rn(__dmul_rn(__dsub_rn(elem(v[j], e), mean), rstd), elem(g4, e));
                hb[e] = f64_to_bf16_bits(__dadd_rn(t, elem(b4, e)));
            }
            hv = make_uint4(hb[0] | (hb[1] << 16), hb[2] | (hb[3] << 16), hb[4] | (hb[5] << 16), hb[6] | (hb[7] << 16));
        }
        v[j] = hv;
        acc = pk_absmax4(acc, hv);
    }
    uint32_t m = wave_max_u32<64>(pk_fold(acc));
    if constexpr (TX > 64) {
        if ((threadIdx.x & 63) == 0) red_max[threadIdx.x >> 6] = m;
        __syncthreads();
        m = red_max[0];
#pragma unroll
        for (int i = 1; i < 4; ++i) m = red_max[i] > m ? red_max[i] : m;
    }
    float s;
    if constexpr (TX > 64) {
        if (wave0) {
            const float s_ = scale_from_amax(mag_to_float(m), FMT, flags);
            if (threadIdx.x == 0) bc_scale = s_;
        }
        __syncthreads();
        s = bc_scale;
    } else {
        s = scale_from_amax(mag_to_float(m), FMT, flags);
    }
    if (!live) return;
    if (tx == 0) {
        scale_out[r] = s;
        if (mean_out) mean_out[r] = (float)mean;
        if (rstd_out) rstd_out[r] = (float)rstd;
    }
    uint8_t* qrow = q + r * ld_q;
    uint16_t* hrow = h ? h + r * ld_h : nullptr;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int64_t vi = tx + (int64_t)j * TX;
        if (vi < nvec) {
            store_stream(reinterpret_cast<uint2*>(qrow) + vi, cast8<FMT>(v[j], s));
            if (hrow) store_stream(reinterpret_cast<uint4*>(hrow) + vi, v[j]);
        }
    }
}

template <int FMT>
static bool launch_lnq_t(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, const uint16_t* gamma,
                         const uint16_t* beta, double eps, int flags, uint16_t* h, int64_t ld_h, uint8_t* q, int64_t ld_q,
                         float* scale_out, float* mean_out, float* rstd_out, hipStream_t st) {
    const int64_t nvec = cols / 8;
#define FP8K_LNQ(TX, NV)                                                                                          \
    layernorm_quant_row_kernel<FMT, TX, NV><<<dim3((unsigned)((rows + (256 / TX) - 1) / (256 / TX))), dim3(256), 0, st>>>( \
        x, rows, cols, ld, gamma, beta, eps, flags, h, ld_h, q, ld_q, scale_out, mean_out, rstd_out)
    // up to 2048 columns a wavefront owns a row (no barriers, the per-row scalar work once per row)
    if (nvec <= 64) FP8K_LNQ(64, 1);
    else if (nvec <= 128) FP8K_LNQ(64, 2);
    else if (nvec <= 256) FP8K_LNQ(64, 4);
    else if (nvec <= 512) FP8K_LNQ(256, 2);
    else if (nvec <= 1024) FP8K_LNQ(256, 4);
    else if (nvec <= 2048) FP8K_LNQ(256, 8);
    else return false;
#undef FP8K_LNQ
    return true;
}

// cols a multiple of 8 and at most 16384; hipErrorNotSupported for wider rows
hipError_t launch_layernorm_quant_row(const void* x, int64_t rows, int64_t cols, int64_t ld, const void* gamma,
                                      const void* beta, double eps, int fmt, int flags, void* h, int64_t ld_h, uint8_t* q,
                                      int64_t ld_q, float* scale_out, float* mean_out, float* rstd_out, hipStream_t st) {
    if (rows == 0 || cols == 0) return hipSuccess;
    if ((rows + 3) / 4 > 0x7FFFFFFF) return hipErrorInvalidValue;
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    const uint16_t* gp = static_cast<const uint16_t*>(gamma);
    const uint16_t* bp = static_cast<const uint16_t*>(beta);
    uint16_t* hp = static_cast<uint16_t*>(h);
    const bool ok = fmt == FMT_E4M3FN
                        ? launch_lnq_t<FMT_E4M3FN>(xp, rows, cols, ld, gp, bp, eps, flags, hp, ld_h, q, ld_q, scale_out, mean_out, rstd_out, st)
                        : launch_lnq_t<FMT_E5M2>(xp, rows, cols, ld, gp, bp, eps, flags, hp, ld_h, q, ld_q, scale_out, mean_out, rstd_out, st);
    if (!ok) return hipErrorNotSupported;
    return hipGetLastError();
}

}  // namespace fp8k
