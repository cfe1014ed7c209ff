// MX (microscaling) FP8 GEMM for gfx950: both operands carry one E8M0 scale
// per block of 32 elements along K (OCP MX specification v1.0; the paper lists
// mxfp8 training among its prototype features), and the matrix cores apply
// the block scales themselves: v_mfma_scale_f32_16x16x128_f8f6f4 takes, per
// lane, 32 K-bytes of one operand row and ONE scale byte for them.
//     out[m, n] = sum_blk 2^(ea[m,blk]-127) 2^(eb[n,blk]-127) sum_{k in blk} dec(a[m,k]) dec(b[n,k])
//
// Structure: the register-staged scheme of gemm_fp8.hip (256 x 256 tile, two LDS
// stages, next step's global loads in flight during the MFMAs) with 4
// wavefronts of 128 x 128 (one per SIMD: with 8 wavefronts the fragments, the
// scales and the staging registers no longer fit beside 128 accumulators).  How the instruction pairs data and scales (measured with
// one-hot blocks; it is the layout the plain kernels already use): lane
// (l % 16, g = l / 16) supplies the 16-byte chunks g and g + 4 of its row's 128
// K-bytes, and the scale byte in lane (l % 16, g) is the one of block g
// (K-bytes [32 g, 32 g + 32), i.e. chunks 2g and 2g+1, which sit in lanes of
// groups g' = 2g mod 4 .. and their upper halves): the hardware routes each
// scale to the lanes that hold its block.  So:
//   - operands are read from LDS exactly as in the plain kernels (chunks g, g+4;
//     swizzle keys: A rows (row >> 1) & 7, B rows ((row >> 1) & 1) | (((row >> 4) & 3) << 1));
//   - each K step also stages the 4 scale bytes of every tile row (one dword per
//     row, blocks 4*step .. 4*step+3); lane (l % 16, g) reads byte g of its row's dword;
//   - no scaling in the epilogue.
// B rows are dealt to the MFMA row index i as n = 16*(i/4) + 4*t + i%4 (t =
// fragment) so that a lane ends up with 16 consecutive output columns.
#include "fp8_device.hpp"
#include "launchers.hpp"
#include "tuning.hpp"


namespace fp8k {

typedef int v8i_m __attribute__((ext_vector_type(8)));
typedef float v4f_m __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_m __attribute__((ext_vector_type(2)));
typedef float f32x2_m __attribute__((ext_vector_type(2)));

namespace mx {
constexpr int BM = 256, BN = 256, BK = 128;
constexpr int NT = 256;                      // 4 wavefronts, 2 (m) x 2 (n): one per SIMD, 512 registers each
constexpr int WM = 128, WN = 128;
constexpr int FM = WM / 16, FN = WN / 16;
constexpr int TILE = (BM + BN) * BK;         // 64 KB of codes
constexpr int STAGE = TILE + (BM + BN) * 4;  // + one dword of scales per row
constexpr int GROUP_M = 4, NUM_XCD = 8;
}  // namespace mx

__device__ __forceinline__ uint32_t mx_pack_bf16(float a, float b) {
    f32x2_m v = {a, b};
    bf16x2_m h = __builtin_convertvector(v, bf16x2_m);
    uint32_t r;
    __builtin_memcpy(&r, &h, 4);
    return r;
}

template <int FA, int FB, bool OUT_F32>
__global__ __launch_bounds__(mx::NT) void gemm_mxfp8_kernel(
    const uint8_t* __restrict__ A, int64_t lda, const uint8_t* __restrict__ EA, int64_t ld_ea,
    const uint8_t* __restrict__ B, int64_t ldb, const uint8_t* __restrict__ EB, int64_t ld_eb, int M, int N, int K,
    void* __restrict__ out, int64_t ld_out, int tiles_m, int tiles_n) {
    using namespace mx;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int ntiles = tiles_m * tiles_n;
    const int per_xcd = gridDim.x / NUM_XCD;
    const int logical = (blockIdx.x % NUM_XCD) * per_xcd + blockIdx.x / NUM_XCD;
    if (logical >= ntiles) return;
    const int in_group = GROUP_M * tiles_n;
    const int first_m = (logical / in_group) * GROUP_M;
    const int gsize = tiles_m - first_m < GROUP_M ? tiles_m - first_m : GROUP_M;
    const int tm = first_m + (logical % in_group) % gsize;
    const int tn = (logical % in_group) / gsize;
    const int m0 = tm * BM, n0 = tn * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;

    // ---- global -> registers -> LDS: thread t owns chunk slot t & 7 of rows (t >> 3) + 32 i, i = 0..7.
    //      The B key depends on bit 5 of the row, i.e. on the parity of i.
    const int srow = tid >> 3, spc = tid & 7;
    const int ca = spc ^ ((srow >> 1) & 7);
    const int cb_e = spc ^ (((srow >> 1) & 1) | (((srow >> 4) & 3) << 1));
    const int cb_o = spc ^ (((srow >> 1) & 1) | ((((srow >> 4) + 2) & 3) << 1));
    const uint8_t* a_ptr = A + (int64_t)(m0 + srow) * lda + ca * 16;
    const uint8_t* b_ptr = B + (int64_t)(n0 + srow) * ldb;
    const int64_t a_step = 32 * lda, b_step = 32 * ldb;
    // scales: thread t owns A row t and B row t of the tile
    const bool sa_ok = m0 + tid < M, sb_ok = n0 + tid < N;
    const uint8_t* sa_ptr = EA + (int64_t)(m0 + tid) * ld_ea;
    const uint8_t* sb_ptr = EB + (int64_t)(n0 + tid) * ld_eb;

    uint4 ra[8], rb[8];
    uint32_t rsa, rsb;
    auto gload = [&](int kt) {
        const int k0 = kt * BK;                      // K % 128 == 0: every chunk of a step is inside K
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            ra[i] = (m0 + srow + 32 * i < M) ? *reinterpret_cast<const uint4*>(a_ptr + i * a_step + k0) : make_uint4(0, 0, 0, 0);
            rb[i] = (n0 + srow + 32 * i < N)
                        ? *reinterpret_cast<const uint4*>(b_ptr + i * b_step + k0 + ((i & 1) ? cb_o : cb_e) * 16)
                        : make_uint4(0, 0, 0, 0);
        }
        rsa = sa_ok ? *reinterpret_cast<const uint32_t*>(sa_ptr + 4 * kt) : 0u;   // blocks 4 kt .. 4 kt + 3 of the row
        rsb = sb_ok ? *reinterpret_cast<const uint32_t*>(sb_ptr + 4 * kt) : 0u;
    };
    auto lstore = [&](int stage) {
        uint8_t* as = smem + stage * STAGE + tid * 16;
        uint8_t* bs = as + BM * BK;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            *reinterpret_cast<uint4*>(as + i * NT * 16) = ra[i];
            *reinterpret_cast<uint4*>(bs + i * NT * 16) = rb[i];
        }
        *reinterpret_cast<uint32_t*>(smem + stage * STAGE + TILE + tid * 4) = rsa;            // A rows
        *reinterpret_cast<uint32_t*>(smem + stage * STAGE + TILE + BM * 4 + tid * 4) = rsb;   // B rows
    };

    // ---- LDS -> MFMA operands
    const int li = lane & 15, g = lane >> 4;
    const int key_a = (li >> 1) & 7;
    const int key_b = ((li >> 1) & 1) | ((li >> 2) << 1);
    const int a_lo = (wm0 + li) * BK + ((g ^ key_a) << 4), a_hi = (wm0 + li) * BK + (((g + 4) ^ key_a) << 4);
    const int b_row = wn0 + 16 * (li >> 2) + (li & 3);          // + 64 grp + 4 t for fragment (grp, t)
    const int b_lo = BM * BK + b_row * BK + ((g ^ key_b) << 4), b_hi = BM * BK + b_row * BK + (((g + 4) ^ key_b) << 4);
    const int sa_off = TILE + (wm0 + li) * 4 + g, sb_off = TILE + BM * 4 + b_row * 4 + g;

    v4f_m acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = v4f_m{0.f, 0.f, 0.f, 0.f};

    auto frag = [&](const uint8_t* base, int lo, int hi) {
        const uint4 x0 = *reinterpret_cast<const uint4*>(base + lo);
        const uint4 x1 = *reinterpret_cast<const uint4*>(base + hi);
        return v8i_m{(int)x0.x, (int)x0.y, (int)x0.z, (int)x0.w, (int)x1.x, (int)x1.y, (int)x1.z, (int)x1.w};
    };
    // The scaled MFMA as inline assembly with the accumulator tied to the destination: through the
    // builtin the compiler picks a different destination and copies every accumulator back.  An
    // accumulator is touched once per 64 MFMAs and read by other instructions only after the loop.
    auto mfma = [&](v4f_m& c, const v8i_m& b, const v8i_m& a, int sbv, int sav) {
#define MX_MFMA(FMT)                                                                               \
    asm volatile("v_mfma_scale_f32_16x16x128_f8f6f4 %0, %1, %2, %0, %3, %4 op_sel_hi:[0,0,0]" FMT \
                 : "+a"(c)                                                                         \
                 : "v"(b), "v"(a), "v"(sbv), "v"(sav))
        if constexpr (FB == 0 && FA == 0) MX_MFMA("");
        if constexpr (FB == 1 && FA == 0) MX_MFMA(" cbsz:1");
        if constexpr (FB == 0 && FA == 1) MX_MFMA(" blgp:1");
        if constexpr (FB == 1 && FA == 1) MX_MFMA(" cbsz:1 blgp:1");
#undef MX_MFMA
    };
    auto compute = [&](int stage) {
        const uint8_t* base = smem + stage * STAGE;
        v8i_m bf[FN];
        int sb[FN];
#pragma unroll
        for (int j = 0; j < FN; ++j) {               // fragment j = (grp, t) = (j / 4, j % 4)
            const int rows = 64 * (j >> 2) + 4 * (j & 3);
            bf[j] = frag(base + rows * BK, b_lo, b_hi);
            sb[j] = base[sb_off + rows * 4];
        }
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            const v8i_m af = frag(base + 16 * i * BK, a_lo, a_hi);
            const int sa = base[sa_off + 64 * i];
#pragma unroll
            for (int j = 0; j < FN; ++j) mfma(acc[i][j], bf[j], af, sb[j], sa);
        }
    };

    const int ksteps = K / BK;
    if (ksteps > 0) {
        gload(0);
        lstore(0);
        __syncthreads();
        for (int kt = 0; kt < ksteps; ++kt) {
            const bool more = kt + 1 < ksteps;
            if (more) gload(kt + 1);
            compute(kt & 1);
            if (more) lstore((kt + 1) & 1);
            __syncthreads();
        }
    }

    // ---- epilogue: lane holds out[m0 + wm0 + 16 i + l%16][n0 + wn0 + 64 grp + 16 g + 4 t + r]
#pragma unroll
    for (int grp = 0; grp < FN / 4; ++grp) {
        const int nb = n0 + wn0 + 64 * grp + 16 * g;
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            const int m = m0 + wm0 + 16 * i + li;
            if (m >= M || nb >= N) continue;
            float v[16];
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) v[4 * t + r] = acc[i][grp * 4 + t][r];
            if constexpr (OUT_F32) {
                float* dst = static_cast<float*>(out) + (int64_t)m * ld_out + nb;
                if (nb + 16 <= N) {
#pragma unroll
                    for (int e = 0; e < 16; e += 4)
                        *reinterpret_cast<float4*>(dst + e) = make_float4(v[e], v[e + 1], v[e + 2], v[e + 3]);
                } else {
                    for (int e = 0; nb + e < N; ++e) dst[e] = v[e];
                }
            } else {
                uint16_t* dst = static_cast<uint16_t*>(out) + (int64_t)m * ld_out + nb;
                uint32_t p[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) p[e] = mx_pack_bf16(v[2 * e], v[2 * e + 1]);
                if (nb + 16 <= N) {
                    *reinterpret_cast<uint4*>(dst) = make_uint4(p[0], p[1], p[2], p[3]);
                    *reinterpret_cast<uint4*>(dst + 8) = make_uint4(p[4], p[5], p[6], p[7]);
                } else {
                    for (int e = 0; nb + e < N; ++e) dst[e] = (uint16_t)(p[e >> 1] >> ((e & 1) * 16));
                }
            }
        }
    }
}

template <int FA, int FB, bool OUT_F32>
static hipError_t launch_mx_t(const uint8_t* a, int64_t lda, const uint8_t* ea, int64_t ld_ea, const uint8_t* b,
                              int64_t ldb, const uint8_t* eb, int64_t ld_eb, int M, int N, int K, void* out,
                              int64_t ld_out, hipStream_t st) {
    using namespace mx;
    auto kern = gemm_mxfp8_kernel<FA, FB, OUT_F32>;
    constexpr int lds = 2 * STAGE;
    static DynamicLdsOnce attr;
    if (hipError_t e = attr.ensure(reinterpret_cast<const void*>(kern), lds); e != hipSuccess) return e;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int64_t ntiles = (int64_t)tiles_m * tiles_n;
    const int64_t grid = (ntiles + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
    if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
    kern<<<dim3((unsigned)grid), dim3(NT), lds, st>>>(a, lda, ea, ld_ea, b, ldb, eb, ld_eb, M, N, K, out, ld_out, tiles_m,
                                                      tiles_n);
    return hipGetLastError();
}

// K must be a multiple of 128 and ld_ea, ld_eb multiples of 4 (a K step reads one aligned
// dword of scales per row); checked by the caller
// large problems: the LDS-DMA kernel (the switch MX_VARIANT = 0 forces this file's kernel, 1 the other)
static bool mx_snake_possible(int64_t lda, int64_t ldb, int64_t K) { return K > 0 && gemm_fp8_snake_fits(lda, ldb); }
static bool mx_takes_snake(int64_t lda, int64_t ldb, int64_t M, int64_t N, int64_t K) {
    const int64_t tiles256 = ((M + 255) / 256) * ((N + 255) / 256);
    const int forced = knob(KNOB_MX_VARIANT);
    const bool big = forced >= 0 ? forced == 1 : tiles256 > 64;
    return big && mx_snake_possible(lda, ldb, K);
}
// shapes whose scales can lie in slabs of sixteen blocks (whole 16-byte scale pieces, 32-bit offsets reach)
static bool mx_slab_possible(int64_t lda, int64_t ldb, int64_t M, int64_t N, int64_t K) {
    return mx_snake_possible(lda, ldb, K) && K % 512 == 0 && M * (K / 32) < (1ll << 31) && N * (K / 32) < (1ll << 31);
}

// True when the MX / blockwise linear calls should hand their scales to launch_gemm_mxfp8 in slabs of sixteen
// blocks (a negative leading dimension, see there).  The caller decides ONCE per call with this function and
// passes the decision down through the sign of the leading dimensions; the switch MX_SLAB = 0 turns it off.
bool gemm_mxfp8_takes_slab_scales(int64_t lda, int64_t ldb, int64_t M, int64_t N, int64_t K) {
    if (knob(KNOB_MX_SLAB) == 0) return false;
    return mx_takes_snake(lda, ldb, M, N, K) && mx_slab_possible(lda, ldb, M, N, K);
}

// ld_ea / ld_eb >= 0: scale rows of that many bytes.  < 0: slabs of sixteen blocks, [K / 512][-ld rows][16 bytes]
// (for both operands alike; only the LDS-DMA kernel reads that layout, so it is taken whatever the switches say).
hipError_t launch_gemm_mxfp8(const uint8_t* a, int64_t lda, int fmt_a, const uint8_t* ea, int64_t ld_ea,
                             const uint8_t* b, int64_t ldb, int fmt_b, const uint8_t* eb, int64_t ld_eb, int64_t M,
                             int64_t N, int64_t K, void* out, int64_t ld_out, int out_f32, hipStream_t st) {
    if (M == 0 || N == 0) return hipSuccess;
    if (ld_ea < 0 || ld_eb < 0) {
        if (!(ld_ea < 0 && ld_eb < 0) || -ld_ea < M || -ld_eb < N || !mx_slab_possible(lda, ldb, M, N, K))
            return hipErrorInvalidValue;
        return launch_gemm_mxfp8_snake(a, lda, fmt_a, ea, ld_ea, b, ldb, fmt_b, eb, ld_eb, M, N, K, out, ld_out, out_f32, st);
    }
    if (mx_takes_snake(lda, ldb, M, N, K) && ld_ea < (1 << 23) && ld_eb < (1 << 23))
        return launch_gemm_mxfp8_snake(a, lda, fmt_a, ea, ld_ea, b, ldb, fmt_b, eb, ld_eb, M, N, K, out, ld_out, out_f32, st);
    const int m = (int)M, n = (int)N, k = (int)K;
#define FP8K_MX(FA_, FB_)                                                                                  \
    if (fmt_a == FA_ && fmt_b == FB_)                                                                      \
        return out_f32 ? launch_mx_t<FA_, FB_, true>(a, lda, ea, ld_ea, b, ldb, eb, ld_eb, m, n, k, out, ld_out, st) \
                       : launch_mx_t<FA_, FB_, false>(a, lda, ea, ld_ea, b, ldb, eb, ld_eb, m, n, k, out, ld_out, st)
    FP8K_MX(FMT_E4M3FN, FMT_E4M3FN);
    FP8K_MX(FMT_E5M2, FMT_E4M3FN);
    FP8K_MX(FMT_E4M3FN, FMT_E5M2);
    FP8K_MX(FMT_E5M2, FMT_E5M2);
#undef FP8K_MX
    return hipErrorInvalidValue;
}

}  // namespace fp8k
