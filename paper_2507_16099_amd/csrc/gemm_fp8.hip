// Scaled FP8 GEMM for gfx950 on the CDNA4 matrix cores
// (v_mfma_f32_16x16x128_f8f6f4): out[M,N] = (A[M,K] . B[N,K]^T) / (sa * sb).
//
// The paper (Section 2.1) leaves the FP8 products to the hardware vendor's GEMM
// kernels; this is this library's own kernel for problems of few tiles, and the dispatch.
//
// Layout of the work
//   - Both operands have the contraction axis contiguous.  A workgroup owns a
//     BM x BN tile of the output and walks K in steps of 128 bytes.
//   - Each K step stages BM + BN rows of 128 bytes in LDS.  A row is eight
//     16-byte chunks; chunk c of a row is stored at chunk position c ^ key(row)
//     so that the 128-bit LDS reads of one MFMA operand (16 rows, same logical
//     chunk) fall into different banks.
//   - One MFMA takes 16 rows x 128 K-bytes of each operand: lane l supplies 32
//     bytes of row l%16, here chunks l/16 and l/16 + 4.  The assignment of K
//     bytes to lanes is the same for both operands, which is all a dot product
//     needs; this one makes every 64-lane 128-bit LDS read touch each of the
//     16 bank groups (16 bytes wide, 256-byte wrap) exactly four times, the
//     conflict-free pattern (chunks 2*(l/16), 2*(l/16)+1 would use only half
//     of the bank groups and run at half the LDS rate).
//   - The B tile is the FIRST MFMA operand and the A tile the second, so a lane
//     ends up with accumulators for one output row m and several n.  The rows
//     of a 64-wide B group are dealt to the four MFMA tiles such that lane l
//     holds 16 CONSECUTIVE n (n = 16*(l/16) + 4*t + r for tile t, register r):
//     the epilogue scales, rounds to bfloat16 and stores 32 contiguous bytes
//     per lane straight from registers.
//   - Workgroup ids are remapped so that each XCD (ids are dealt round-robin to
//     the 8 XCDs) works on one contiguous range of tiles, walked in groups of
//     tile rows, which keeps the operand panels of concurrently running tiles
//     in that XCD's L2.
#include "fp8_device.hpp"
#include "launchers.hpp"
#include "tuning.hpp"

namespace fp8k {

typedef int v8i_t __attribute__((ext_vector_type(8)));
typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef float v4f_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

constexpr int BK = 128;          // bytes of K per step
constexpr int GROUP_M = 4;       // tile rows walked together
constexpr int NUM_XCD = 8;

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    f32x2_t v = {a, b};
    bf16x2_t h = __builtin_convertvector(v, bf16x2_t);
    uint32_t r;
    __builtin_memcpy(&r, &h, 4);
    return r;
}

// PD: how many K steps ahead of the matrix cores the global loads run (register sets in flight).  A
// workgroup that is alone on its CU has nothing else to hide the load latency with (about 1 us per step
// at PD = 1, whatever the tile); the small tiles, used when there are few of them, take PD = 4.
// One product as the kernel sees it.  A launch can carry two of them (same formats, same kinds of scale): workgroups
// from `split` on, a multiple of 8, work on the second, so that the two small products of a backward step share
// one launch and run side by side.
struct TnProblem {
    const uint8_t* A; int64_t lda; const uint8_t* B; int64_t ldb;
    const float* scale_a; const float* scale_b; int M, N, K; void* out; int64_t ld_out; int tiles_m, tiles_n;
};
constexpr int ONE_PROBLEM = 0x7FFFFFFF;

template <int BM, int BN, int WAVES_M, int WAVES_N, int FA, int FB, bool OUT_F32, int PD = 1>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void gemm_fp8_tn_kernel(TnProblem p1, int row_a, int row_b, int split,
                                                                            TnProblem p2) {
    const bool second = (int)blockIdx.x >= split;
    const TnProblem& p = second ? p2 : p1;
    const uint8_t* __restrict__ A = p.A;
    const uint8_t* __restrict__ B = p.B;
    const float* __restrict__ scale_a = p.scale_a;
    const float* __restrict__ scale_b = p.scale_b;
    void* __restrict__ out = p.out;
    const int64_t lda = p.lda, ldb = p.ldb, ld_out = p.ld_out;
    const int M = p.M, N = p.N, K = p.K, tiles_m = p.tiles_m, tiles_n = p.tiles_n;
    const int bid = second ? (int)blockIdx.x - split : (int)blockIdx.x;
    const int nblocks = second ? (int)gridDim.x - split : (split == ONE_PROBLEM ? (int)gridDim.x : split);
    constexpr int NT = WAVES_M * WAVES_N * 64;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int FM = WM / 16;       // A fragments (16 rows each) per wave
    constexpr int NG = WN / 64;       // 64-wide B groups per wave
    constexpr int FN = NG * 4;        // B fragments per wave
    constexpr int NLA = BM * 8 / NT;  // 16-byte chunks each thread stages per step
    constexpr int NLB = BN * 8 / NT;
    constexpr int STAGE = (BM + BN) * BK;
    static_assert(WM % 16 == 0 && WN % 64 == 0 && (BM * 8) % NT == 0 && (BN * 8) % NT == 0 && (NT / 8) % 32 == 0, "tile");

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // ---- workgroup -> tile
    const int ntiles = tiles_m * tiles_n;
    const int per_xcd = nblocks / NUM_XCD;
    const int logical = (bid % NUM_XCD) * per_xcd + bid / NUM_XCD;
    if (logical >= ntiles) return;
    const int in_group = GROUP_M * tiles_n;
    const int first_m = (logical / in_group) * GROUP_M;
    const int gsize = tiles_m - first_m < GROUP_M ? tiles_m - first_m : GROUP_M;
    const int tm = first_m + (logical % in_group) % gsize;
    const int tn = (logical % in_group) / gsize;
    const int m0 = tm * BM, n0 = tn * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;

    // ---- global -> LDS staging: thread t owns LDS chunk slots i*NT + t
    const int srow = tid >> 3, spc = tid & 7;
    const int ca = spc ^ (srow & 7);                                   // logical chunk, A rows
    const int cb = spc ^ ((srow & 3) | ((srow >> 2) & 4));             // logical chunk, B rows
    // PD == 1: plain global loads, guarded by branches (any size of tensor).  PD > 1: buffer loads, which
    // return zeros beyond the end of the tensor without a branch, so that the loop body is straight-line
    // code and the compiler leaves the loads of later steps in flight (a branch around a load makes it
    // drain them all); the launcher uses this form only where 32-bit offsets suffice.
    const uint8_t* a_ptr = A + (int64_t)(m0 + srow) * lda + ca * 16;
    const uint8_t* b_ptr = B + (int64_t)(n0 + srow) * ldb + cb * 16;
    const int64_t a_step = (int64_t)(NT / 8) * lda, b_step = (int64_t)(NT / 8) * ldb;
    const __amdgpu_buffer_rsrc_t rs_a = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(A), 0, PD > 1 ? (int)((int64_t)(M - 1) * lda + K) : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_b = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(B), 0, PD > 1 ? (int)((int64_t)(N - 1) * ldb + K) : 0, 0x00020000);
    constexpr uint32_t OUTSIDE = 0x80000000u;   // beyond any tensor this form is used for
    uint32_t va[NLA], vb[NLB];                  // byte offsets of this thread's rows (PD > 1)
#pragma unroll
    for (int i = 0; i < NLA; ++i) {
        const int r = m0 + srow + i * (NT / 8);
        va[i] = r < M ? (uint32_t)r * (uint32_t)lda + ca * 16 : OUTSIDE;
    }
#pragma unroll
    for (int i = 0; i < NLB; ++i) {
        const int r = n0 + srow + i * (NT / 8);
        vb[i] = r < N ? (uint32_t)r * (uint32_t)ldb + cb * 16 : OUTSIDE;
    }

    uint4 ra[PD][NLA], rb[PD][NLB];
    auto gload = [&](int k0, uint4 (&xa)[NLA], uint4 (&xb)[NLB]) {
        const bool ka = k0 + ca * 16 < K, kb = k0 + cb * 16 < K;
        if constexpr (PD > 1) {
#pragma unroll
            for (int i = 0; i < NLA; ++i) {
                const uint32_t off = (ka && va[i] != OUTSIDE) ? va[i] + (uint32_t)k0 : OUTSIDE;
                const v4i_t v = __builtin_amdgcn_raw_buffer_load_b128(rs_a, (int)off, 0, 0);
                xa[i] = make_uint4((uint32_t)v.x, (uint32_t)v.y, (uint32_t)v.z, (uint32_t)v.w);
            }
#pragma unroll
            for (int i = 0; i < NLB; ++i) {
                const uint32_t off = (kb && vb[i] != OUTSIDE) ? vb[i] + (uint32_t)k0 : OUTSIDE;
                const v4i_t v = __builtin_amdgcn_raw_buffer_load_b128(rs_b, (int)off, 0, 0);
                xb[i] = make_uint4((uint32_t)v.x, (uint32_t)v.y, (uint32_t)v.z, (uint32_t)v.w);
            }
        } else {
#pragma unroll
            for (int i = 0; i < NLA; ++i) {
                const bool ok = ka && (m0 + srow + i * (NT / 8) < M);
                xa[i] = ok ? *reinterpret_cast<const uint4*>(a_ptr + i * a_step + k0) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < NLB; ++i) {
                const bool ok = kb && (n0 + srow + i * (NT / 8) < N);
                xb[i] = ok ? *reinterpret_cast<const uint4*>(b_ptr + i * b_step + k0) : make_uint4(0, 0, 0, 0);
            }
        }
    };
    auto lstore = [&](int stage, const uint4 (&xa)[NLA], const uint4 (&xb)[NLB]) {
        uint8_t* as = smem + stage * STAGE + tid * 16;
        uint8_t* bs = as + BM * BK;
#pragma unroll
        for (int i = 0; i < NLA; ++i) *reinterpret_cast<uint4*>(as + i * NT * 16) = xa[i];
#pragma unroll
        for (int i = 0; i < NLB; ++i) *reinterpret_cast<uint4*>(bs + i * NT * 16) = xb[i];
    };

    // ---- LDS -> MFMA operands
    const int key = lane & 7;
    const int off_lo = ((lane >> 4) ^ key) << 4, off_hi = (((lane >> 4) + 4) ^ key) << 4;
    const int a_row_off = (wm0 + (lane & 15)) * BK;
    const int b_row_off = (wn0 + 16 * ((lane & 15) >> 2) + (lane & 3)) * BK;

    v4f_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = v4f_t{0.f, 0.f, 0.f, 0.f};

    auto frag = [&](const uint8_t* base) {
        const uint4 lo = *reinterpret_cast<const uint4*>(base + off_lo);
        const uint4 hi = *reinterpret_cast<const uint4*>(base + off_hi);
        return v8i_t{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
    };
    auto compute = [&](int stage) {
        const uint8_t* as = smem + stage * STAGE + a_row_off;
        const uint8_t* bs = smem + stage * STAGE + BM * BK + b_row_off;
        v8i_t bf[FN];
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int t = 0; t < 4; ++t) bf[g * 4 + t] = frag(bs + (64 * g + 4 * t) * BK);
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            const v8i_t af = frag(as + 16 * i * BK);
#pragma unroll
            for (int j = 0; j < FN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bf[j], af, acc[i][j], FB, FA, 0, 0, 0, 0);
        }
    };

    // ---- main loop, two LDS stages; step s travels through register set s % PD.  The step count is
    // rounded up to a multiple of PD (steps beyond K load zeros), which keeps the unrolled body free of
    // conditions.
    const int ksteps = (K + BK - 1) / BK;
    const int kpad = (ksteps + PD - 1) / PD * PD;
    // the scales of this tile's rows and columns are requested now, so that their latency lies under the K loop
    // (problems of few tiles are bound by such fixed costs: a trip to memory is about as long as two K steps)
    float sa_raw[FM], sb_raw[NG][16];
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int m = m0 + wm0 + 16 * i + (lane & 15);
        sa_raw[i] = row_a ? (m < M ? scale_a[m] : 1.0f) : scale_a[0];
    }
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int n = n0 + wn0 + 64 * g + 16 * (lane >> 4) + e;
            sb_raw[g][e] = row_b ? (n < N ? scale_b[n] : 1.0f) : scale_b[0];
        }
    if (ksteps > 0) {
        // all PD register sets are requested before the first one is awaited (loads return in issue order)
#pragma unroll
        for (int s_ = 0; s_ < PD; ++s_) gload(s_ * BK, ra[s_], rb[s_]);
        lstore(0, ra[0], rb[0]);
        __syncthreads();
        for (int kb = 0; kb < kpad; kb += PD) {
#pragma unroll
            for (int u = 0; u < PD; ++u) {
                const int kt = kb + u;
                gload((kt + PD) * BK, ra[u], rb[u]);   // set u is free: step kt sits in LDS
                compute(kt & 1);
                lstore((kt + 1) & 1, ra[(u + 1) % PD], rb[(u + 1) % PD]);
                __syncthreads();
            }
        }
    }

    // ---- epilogue: (acc * 1/sa) * 1/sb, round, store 16 consecutive n per lane
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const int nb = n0 + wn0 + 64 * g + 16 * (lane >> 4);
        float inv_b[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) inv_b[e] = (nb + e < N) ? 1.0f / sb_raw[g][e] : 0.f;
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            const int m = m0 + wm0 + 16 * i + (lane & 15);
            if (m >= M || nb >= N) continue;
            const float inv_a = 1.0f / sa_raw[i];
            float v[16];
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) v[4 * t + r] = (acc[i][g * 4 + t][r] * inv_a) * inv_b[4 * t + r];
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
                for (int e = 0; e < 8; ++e) p[e] = pack_bf16(v[2 * e], v[2 * e + 1]);
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

// g2 == nullptr: one product
template <int BM, int BN, int WAVES_M, int WAVES_N, int FA, int FB, bool OUT_F32, int PD = 1>
static hipError_t launch_variant(const GemmOperands& g1, const GemmOperands* g2, int row_a, int row_b, hipStream_t st) {
    auto kern = gemm_fp8_tn_kernel<BM, BN, WAVES_M, WAVES_N, FA, FB, OUT_F32, PD>;
    constexpr int lds = 2 * (BM + BN) * BK;
    static DynamicLdsOnce attr;     // one per instantiation
    if (hipError_t e = attr.ensure(reinterpret_cast<const void*>(kern), lds); e != hipSuccess) return e;
    int64_t blocks[2] = {0, 0};
    auto problem = [&](const GemmOperands& g, int64_t* nb) {
        const int tiles_m = (int)((g.M + BM - 1) / BM), tiles_n = (int)((g.N + BN - 1) / BN);
        *nb = ((int64_t)tiles_m * tiles_n + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
        return TnProblem{g.a, g.lda, g.b, g.ldb, g.scale_a, g.scale_b, (int)g.M, (int)g.N, (int)g.K, g.out, g.ld_out, tiles_m, tiles_n};
    };
    const TnProblem p1 = problem(g1, &blocks[0]);
    const TnProblem p2 = g2 ? problem(*g2, &blocks[1]) : p1;
    if (blocks[0] + blocks[1] > 0x7FFFFFF0) return hipErrorInvalidValue;
    kern<<<dim3((unsigned)(blocks[0] + blocks[1])), dim3(WAVES_M * WAVES_N * 64), lds, st>>>(
        p1, row_a, row_b, g2 ? (int)blocks[0] : ONE_PROBLEM, p2);
    return hipGetLastError();
}

template <int FA, int FB, bool OUT_F32>
static hipError_t launch_fmt(int variant, const GemmOperands& g1, const GemmOperands* g2, int row_a, int row_b, hipStream_t st) {
    if (variant == 6) return launch_variant<64, 64, 4, 1, FA, FB, OUT_F32, 4>(g1, g2, row_a, row_b, st);
    if (variant == 7) return launch_variant<128, 128, 2, 2, FA, FB, OUT_F32, 4>(g1, g2, row_a, row_b, st);
    return launch_variant<128, 128, 2, 2, FA, FB, OUT_F32>(g1, g2, row_a, row_b, st);
}

// Kernel choice: the few-row kernel of gemm_fp8_skinny.hip (variant 5) for
// M <= 32 (measured 2-7x faster there; from 33 to 64 rows its loads of A
// through the L1 cache cost as much as the tiled kernels' padding); otherwise by the number of 128 x 128 tiles of
// the output: up to 128 of them 64 x 64 tiles, up to 256 of them 128 x 128 tiles, beyond that the 256 x 256 kernels
// of gemm_fp8_snake.hip / gemm_fp8_stream.hip (variant 4).
// Measured per product, ten in a HIP graph, K = 1024 / 4096 / 16384 (us):
//      64 tiles (1024 x 1024):   64x64  8.1 / 15.3 /   -     128x128 13.5 / 29.5 /   -     256x256 10.5 / 24.5 /   -
//     128 tiles (1024 x 2048):         10.1 / 22.0 /   -             13.9 / 30.7 /   -             10.8 / 31.3 /   -
//     192 tiles (1536 x 2048):         13.2 / 27.3 /  86             14.2 / 30.8 /  95             10.8 / 31.3 / 103
//     256 tiles (2048 x 2048):         16.2 / 35.1 / 114             14.6 / 31.4 /  95             10.8 / 31.4 / 104
//     384 tiles (2048 x 3072):         22.3 / 48.4 / 163             26.8 / 58.6 / 186             10.8 / 31.8 / 105
//     512 tiles (2048 x 4096):         29.1 / 62.1 / 215             27.8 / 59.6 / 188             12.0 / 34.1 / 112
// With few tiles the K loop of a lone workgroup per CU is bound by the latency of its loads, about 1 us per step
// whatever the tile, so more and smaller tiles finish sooner; once every CU has a workgroup the time of the small
// tiles grows with the work, while sixty-four 256 x 256 tiles still take what one takes.  At 129-256 tiles the
// 128 x 128 tiles are kept although the table favours the large ones for short contractions: inside whole
// forward + backward steps they came out ahead (3-6 us per step at 1024 x 1024 x 4096 and 4096 x 1024 x 1024), and
// the two products of a backward step can then share one launch (launch_gemm_fp8_pair), which in steps of
// 4096 x 1024 x 4096 and five other shapes of that class saved 22-65 us (13-15 %).
// Switches (tuning and test aid): GEMM_BIG_FROM moves the tile count from which the 256 x 256 kernels are used;
// GEMM_VARIANT forces a kernel: 0 = 128x128 / 4 waves (register-staged; also the fallback where the 32-bit
// offsets of the others do not reach), 4 = 256 x 256, 5 = few-row kernel (only where M <= 64), 6 = 64x64 / 4 waves
// with loads 4 steps ahead, 7 = 128x128 / 4 waves likewise (both register-staged through buffer loads; eight steps ahead
// measured 5-35 % slower on the small tile, three steps ahead 4-6 % slower on the large one).
static int pick_variant(int64_t M, int64_t N) {
    if (const int v = knob(KNOB_GEMM_VARIANT); v == 0 || (v >= 4 && v <= 7)) return v;
    if (M <= 32) return 5;
    const int64_t tiles128 = ((M + 127) / 128) * ((N + 127) / 128);
    const int big = knob(KNOB_GEMM_BIG_FROM);
    if (tiles128 >= (big > 0 ? big : 257)) return 4;
    return tiles128 <= 128 ? 6 : 7;   // (launch_gemm_fp8 falls back to 0 where their 32-bit offsets do not reach)
}

hipError_t launch_gemm_fp8(const uint8_t* a, int64_t lda, int fmt_a, const float* scale_a, int row_a,
                           const uint8_t* b, int64_t ldb, int fmt_b, const float* scale_b, int row_b,
                           int64_t M, int64_t N, int64_t K, void* out, int64_t ld_out, int out_f32,
                           hipStream_t st) {
    if (M == 0 || N == 0) return hipSuccess;
    int v = pick_variant(M, N);
    // the forms with loads several steps ahead address their operands with 32-bit byte offsets (a tile may
    // reach up to 127 rows past the end)
    if ((v == 6 || v == 7) && ((M + 128) * lda + K >= (int64_t)1 << 31 || (N + 128) * ldb + K >= (int64_t)1 << 31)) v = 0;
    if (v == 5 && M <= 64 && K > 0)
        return launch_gemm_fp8_skinny(a, lda, fmt_a, scale_a, row_a, b, ldb, fmt_b, scale_b, row_b, M, N, K, out, ld_out,
                                      out_f32, st);
    if (v == 4 && gemm_fp8_snake_fits(lda, ldb))   // else: the 128 x 128 register-staged kernel below
        return launch_gemm_fp8_snake(a, lda, fmt_a, scale_a, row_a, b, ldb, fmt_b, scale_b, row_b, M, N, K, out, ld_out,
                                     out_f32, st);
    if (v == 4 || v == 5) v = 0;
    const GemmOperands g{a, lda, scale_a, b, ldb, scale_b, M, N, K, out, ld_out};
#define FP8K_GEMM(FA_, FB_)                                                                    \
    if (fmt_a == FA_ && fmt_b == FB_)                                                          \
        return out_f32 ? launch_fmt<FA_, FB_, true>(v, g, nullptr, row_a, row_b, st)          \
                       : launch_fmt<FA_, FB_, false>(v, g, nullptr, row_a, row_b, st)
    FP8K_GEMM(FMT_E4M3FN, FMT_E4M3FN);
    FP8K_GEMM(FMT_E5M2, FMT_E4M3FN);
    FP8K_GEMM(FMT_E4M3FN, FMT_E5M2);
    FP8K_GEMM(FMT_E5M2, FMT_E5M2);
#undef FP8K_GEMM
    return hipErrorInvalidValue;
}

// Two products of the same formats and kinds of scale (bfloat16 results) in ONE launch, for the pair dX, dW of a
// backward step whose products are too small to fill the chip one at a time.  hipErrorNotSupported (nothing
// launched) where either is large enough for the 256 x 256 kernels, has few rows, or the two would take different
// tiles: the caller then launches them one after the other.
hipError_t launch_gemm_fp8_pair(const GemmOperands& g1, const GemmOperands& g2, int fmt_a, int fmt_b, int row_a, int row_b,
                                hipStream_t st) {
    if (g1.M == 0 || g1.N == 0 || g2.M == 0 || g2.N == 0 || knob(KNOB_PAIRS) == 0) return hipErrorNotSupported;
    const int v1 = pick_variant(g1.M, g1.N), v2 = pick_variant(g2.M, g2.N);
    if ((v1 != 6 && v1 != 7) || v1 != v2) return hipErrorNotSupported;
    auto reach = [](const GemmOperands& g) {
        return (g.M + 128) * g.lda + g.K < (int64_t)1 << 31 && (g.N + 128) * g.ldb + g.K < (int64_t)1 << 31;
    };
    if (!reach(g1) || !reach(g2)) return hipErrorNotSupported;
    const int v = v1;   // (a product with few tiles and a long contraction, sharing a launch on the larger tile of the other, took 2-3x longer)
#define FP8K_GEMM(FA_, FB_) \
    if (fmt_a == FA_ && fmt_b == FB_) return launch_fmt<FA_, FB_, false>(v, g1, &g2, row_a, row_b, st)
    FP8K_GEMM(FMT_E4M3FN, FMT_E4M3FN);
    FP8K_GEMM(FMT_E5M2, FMT_E4M3FN);
    FP8K_GEMM(FMT_E4M3FN, FMT_E5M2);
    FP8K_GEMM(FMT_E5M2, FMT_E5M2);
#undef FP8K_GEMM
    return hipErrorInvalidValue;
}

}  // namespace fp8k
