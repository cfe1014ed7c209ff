// Scaled FP8 GEMM for few rows of A (M <= 64): out[M,N] = (A[M,K] . B[N,K]^T) / (sa * sb).
// This is the shape of inference with pre-quantized weights (Section 3 of the
// paper: dynamic activation + weight FP8 quantization) at decode batch sizes:
// B (the weight) is read once and the kernel is bound by that HBM stream, N*K
// bytes, not by the matrix cores.
//
// No LDS staging and no barriers in the main loop.  A wavefront owns 16 rows
// of B (16 output columns) and a contiguous part of K; per 128-byte K step
// lane l loads bytes [16*(l/16), +16) and [64 + 16*(l/16), +16) of row l%16
// straight from global memory into the MFMA operand registers (any assignment
// of K bytes to lanes works as long as both operands use the same one; this
// one makes each load instruction cover 64 contiguous bytes per row), B with
// the streaming hint.  The few rows of A are loaded the same way;
// every wavefront of the chip reads the same A, so those loads are served by
// the L1 / L2 caches.  One v_mfma_f32_16x16x128_f8f6f4 per 16 rows of A and K
// step; B is the first operand, so a lane ends up with 4 consecutive output
// columns of one output row.  A wavefront takes 1, 2 or 4 such column tiles.  K can be split over 2 or 4 wavefronts of the
// workgroup (summed through LDS at the end) when N alone does not give enough
// wavefronts to keep the memory system busy.
#include "fp8_device.hpp"
#include "launchers.hpp"


namespace fp8k {

typedef int v8i_k __attribute__((ext_vector_type(8)));
typedef float v4f_k __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_k __attribute__((ext_vector_type(2)));
typedef float f32x2_k __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t sk_pack_bf16(float a, float b) {
    f32x2_k v = {a, b};
    bf16x2_k h = __builtin_convertvector(v, bf16x2_k);
    uint32_t r;
    __builtin_memcpy(&r, &h, 4);
    return r;
}

template <int FA, int FB, int MT, int KS, int NW>
__global__ __launch_bounds__(256) void gemm_fp8_skinny_kernel(
    const uint8_t* __restrict__ A, int64_t lda, const uint8_t* __restrict__ B, int64_t ldb,
    const float* __restrict__ scale_a, int row_a, const float* __restrict__ scale_b, int row_b, int M, int N,
    int K, void* __restrict__ out, int64_t ld_out, int out_f32) {
    constexpr int NTW = 4 / KS;          // wavefront column groups per workgroup
    constexpr int U = 2;                 // K steps per batch of loads (registers: 8 * U * (2 * NW + MT))
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int n0 = (blockIdx.x * NTW + wave / KS) * (16 * NW);   // this wavefront's 16 * NW columns
    const int kp = wave % KS;

    // this wavefront's K steps [s_begin, s_end)
    const int ksteps = (K + 127) / 128;
    const int per = (ksteps + KS - 1) / KS;
    const int s_begin = kp * per;
    const int s_end = s_begin + per < ksteps ? s_begin + per : ksteps;

    // rows past N / M are clamped to the last valid one (their results are not stored)
    const uint8_t* bp[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const int n = n0 + 16 * w + i < N ? n0 + 16 * w + i : N - 1;
        bp[w] = B + (int64_t)n * ldb;
    }
    const uint8_t* ap[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int m = 16 * t + i < M ? 16 * t + i : M - 1;
        ap[t] = A + (int64_t)m * lda;
    }

    // scales of this lane's outputs, requested now so that they are there at the end
    float sc_b[NW][4], sc_a[MT];
#pragma unroll
    for (int w = 0; w < NW; ++w)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int n = n0 + 16 * w + 4 * g + r;
            sc_b[w][r] = scale_b[row_b ? (n < N ? n : N - 1) : 0];
        }
#pragma unroll
    for (int t = 0; t < MT; ++t) sc_a[t] = scale_a[row_a ? (16 * t + i < M ? 16 * t + i : M - 1) : 0];

    v4f_k acc[NW][MT];
#pragma unroll
    for (int w = 0; w < NW; ++w)
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[w][t] = v4f_k{0.f, 0.f, 0.f, 0.f};

    // lane (i, g) takes bytes [16g, 16g + 16) and [64 + 16g, 64 + 16g + 16) of the 128-byte step of row i
    const int koff = 16 * g;
    auto frag = [](const uint4& lo, const uint4& hi) {
        return v8i_k{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
    };

    // K steps that lie entirely inside K: batches of U steps, every load of a batch
    // (B with the streaming hint, A through the caches) issued before its first use,
    // and the B loads of the next batch before the MFMAs of this one
    const int full = K / 128;
    const int s_full = s_end < full ? s_end : full;
    int s = s_begin;
    v8i_k bf[U][NW], bn[U][NW];
    auto load_b = [&](int s0, v8i_k (&dst)[U][NW]) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const uint8_t* p = bp[w] + (s0 + u) * 128 + koff;
                dst[u][w] = frag(load_stream(p), load_stream(p + 64));
            }
    };
    if (s + U <= s_full) load_b(s, bf);
    for (; s + U <= s_full; s += U) {
        v8i_k af[U][MT];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                const uint8_t* p = ap[t] + (s + u) * 128 + koff;
                af[u][t] = frag(*reinterpret_cast<const uint4*>(p), *reinterpret_cast<const uint4*>(p + 64));
            }
        const bool more = s + 2 * U <= s_full;
        if (more) load_b(s + U, bn);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int t = 0; t < MT; ++t)
                    acc[w][t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bf[u][w], af[u][t], acc[w][t], FB, FA, 0,
                                                                               0, 0, 0);
        if (more) {
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int w = 0; w < NW; ++w) bf[u][w] = bn[u][w];
        }
    }
    // the steps left over, one at a time, zeros past K (K % 16 == 0)
    for (; s < s_end; ++s) {
        const int k = s * 128 + koff;
        const uint4 z = make_uint4(0, 0, 0, 0);
        v8i_k afr[MT];
#pragma unroll
        for (int t = 0; t < MT; ++t)
            afr[t] = frag(k < K ? *reinterpret_cast<const uint4*>(ap[t] + k) : z,
                          k + 64 < K ? *reinterpret_cast<const uint4*>(ap[t] + k + 64) : z);
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const v8i_k bfr = frag(k < K ? load_stream(bp[w] + k) : z, k + 64 < K ? load_stream(bp[w] + k + 64) : z);
#pragma unroll
            for (int t = 0; t < MT; ++t)
                acc[w][t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bfr, afr[t], acc[w][t], FB, FA, 0, 0, 0, 0);
        }
    }

    // ---- sum the K parts of a column group through LDS
    if constexpr (KS > 1) {
        __shared__ v4f_k part[NTW][KS - 1][NW * MT][64];
        if (kp > 0) {
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int t = 0; t < MT; ++t) part[wave / KS][kp - 1][w * MT + t][lane] = acc[w][t];
        }
        __syncthreads();
        if (kp > 0) return;
#pragma unroll
        for (int p = 0; p < KS - 1; ++p)
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    const v4f_k o = part[wave / KS][p][w * MT + t][lane];
                    acc[w][t] += o;
                }
    }

    // ---- epilogue: lane holds out[16*t + i][n0 + 16*w + 4*g + r], r = 0..3
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const int nb = n0 + 16 * w + 4 * g;
        if (nb >= N) continue;
        float inv_b[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) inv_b[r] = 1.0f / sc_b[w][r];
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const int m = 16 * t + i;
            if (m >= M) continue;
            const float inv_a = 1.0f / sc_a[t];
            float v[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] = (acc[w][t][r] * inv_a) * inv_b[r];
            if (out_f32) {
                float* dst = static_cast<float*>(out) + (int64_t)m * ld_out + nb;
                if (nb + 4 <= N) *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
                else for (int r = 0; nb + r < N; ++r) dst[r] = v[r];
            } else {
                uint16_t* dst = static_cast<uint16_t*>(out) + (int64_t)m * ld_out + nb;
                const uint32_t p0 = sk_pack_bf16(v[0], v[1]), p1 = sk_pack_bf16(v[2], v[3]);
                if (nb + 4 <= N) {
                    *reinterpret_cast<uint2*>(dst) = make_uint2(p0, p1);
                } else {
                    const uint32_t w2[2] = {p0, p1};
                    for (int r = 0; nb + r < N; ++r) dst[r] = (uint16_t)(w2[r >> 1] >> ((r & 1) * 16));
                }
            }
        }
    }
}

template <int FA, int FB>
static hipError_t launch_sk(const uint8_t* a, int64_t lda, const float* sa, int row_a, const uint8_t* b, int64_t ldb,
                            const float* sb, int row_b, int M, int N, int K, void* out, int64_t ld_out, int out_f32,
                            hipStream_t st) {
    const int mt = (M + 15) / 16;                 // 1..4
    // columns per wavefront: 16, 32 or 64.  Wider groups reuse every fragment of A for
    // two or four MFMAs (the loads of A through the L1 cache are what limits this
    // kernel as M grows), narrower ones give more wavefronts; measured crossovers
    const int nw = N >= 12288 ? 4 : (N >= 6144 ? 2 : 1);
    const int64_t groups = ((int64_t)N + 16 * nw - 1) / (16 * nw);
    // split K over the wavefronts of a workgroup until about 2048 wavefronts stream B
    int ks = 1;
    while (ks < 4 && groups * ks < 2048 && K / (ks * 2) >= 512) ks *= 2;
    const int64_t grid = (groups + (4 / ks) - 1) / (4 / ks);
    if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
#define FP8K_SK(MT_, KS_, NW_)                                                                                \
    if (mt == MT_ && ks == KS_ && nw == NW_)                                                                  \
        gemm_fp8_skinny_kernel<FA, FB, MT_, KS_, NW_><<<dim3((unsigned)grid), dim3(256), 0, st>>>(            \
            a, lda, b, ldb, sa, row_a, sb, row_b, M, N, K, out, ld_out, out_f32)
#define FP8K_SK3(MT_) \
    FP8K_SK(MT_, 1, 1); FP8K_SK(MT_, 2, 1); FP8K_SK(MT_, 4, 1); FP8K_SK(MT_, 1, 2); FP8K_SK(MT_, 2, 2); FP8K_SK(MT_, 4, 2); \
    FP8K_SK(MT_, 1, 4); FP8K_SK(MT_, 2, 4); FP8K_SK(MT_, 4, 4)
    FP8K_SK3(1); FP8K_SK3(2); FP8K_SK3(3); FP8K_SK3(4);
#undef FP8K_SK3
#undef FP8K_SK
    return hipGetLastError();
}

hipError_t launch_gemm_fp8_skinny(const uint8_t* a, int64_t lda, int fmt_a, const float* scale_a, int row_a,
                                  const uint8_t* b, int64_t ldb, int fmt_b, const float* scale_b, int row_b,
                                  int64_t M, int64_t N, int64_t K, void* out, int64_t ld_out, int out_f32,
                                  hipStream_t st) {
    if (M == 0 || N == 0) return hipSuccess;
    if (M > 64) return hipErrorInvalidValue;
    const int m = (int)M, n = (int)N, k = (int)K;
#define FP8K_SKF(FA_, FB_)               \
    if (fmt_a == FA_ && fmt_b == FB_)    \
        return launch_sk<FA_, FB_>(a, lda, scale_a, row_a, b, ldb, scale_b, row_b, m, n, k, out, ld_out, out_f32, st)
    FP8K_SKF(FMT_E4M3FN, FMT_E4M3FN);
    FP8K_SKF(FMT_E5M2, FMT_E4M3FN);
    FP8K_SKF(FMT_E4M3FN, FMT_E5M2);
    FP8K_SKF(FMT_E5M2, FMT_E5M2);
#undef FP8K_SKF
    return hipErrorInvalidValue;
}

}  // namespace fp8k
