// Scaled FP8 GEMM for gfx950 on v_mfma_f32_16x16x128_f8f6f4, 256 x 256 tile,
// four wavefronts (2 x 2), each owning a 128 x 128 quadrant as 8 x 8 MFMA tiles.
// out[M,N] = (A[M,K] . B[N,K]^T) / (sa * sb), both operands K-contiguous.
//
// Why 16x16x128: under the board power limit the sustained rate of this
// instruction on random data measures ~10 % above that of 32x32x64 (register
// only loop: ~4.1-4.4 vs ~3.7-3.9 PFLOP/s), and the GEMM is power-bound.
//
// Schedule ("snake").  A K step (128 bytes) is four phases of 16 MFMAs, each
// phase pairing one half of the wave's A fragments (4 x 16 rows) with one half
// of its B fragments:  (A0,Bf) (A0,Bm) (A1,Bm) (A1,Bf), where Bf/Bm alternate
// between B0/B1 from step to step.  Every phase keeps one half of the previous
// phase, so only ONE half (4 fragments = 32 registers) has to arrive per phase,
// and it is read into the registers of the half that died one phase earlier:
// 128 fragment registers in total, each LDS read issued a full phase (512
// matrix-core cycles) before its first use.  Stage k is read in phases 3, 4 of
// step k-1 and 1, 2 of step k; the barrier in the middle of step k releases its
// buffer, which is then refilled with step k+2 during phases 3 and 4 (one
// LDS-DMA load every second MFMA slot).
//
// Data movement
//   - global -> LDS by buffer_load_dwordx4 ... lds, 8 rows x 128 bytes per wave
//     instruction, XOR swizzle applied on the global side, rows past M / N and
//     chunks past K zero-filled by the buffer descriptor's bounds check;
//   - an MFMA operand is 16 rows x 128 bytes; lane l supplies chunks {g, g+4}
//     (g = l/16) of row l%16, the same assignment for both operands.  A 64-lane
//     128-bit LDS read is served as two halves of 32 lanes, each of which may
//     hit every 16-byte bank group (256-byte wrap) twice; the swizzle keys
//     below make the 16 rows of a fragment distinct in (row parity, key):
//       A rows: key = (row >> 1) & 7
//       B rows: key = ((row >> 1) & 1) | (((row >> 4) & 3) << 1)
//     (B rows are dealt to the MFMA row index i as n = 16*(i/4) + 4*t + i%4
//     inside a 64-wide group, t = fragment, so that a lane's accumulators of a
//     group are 16 consecutive n);
//   - the B tile is the first MFMA operand, A the second: a lane's accumulators
//     belong to one output row m.  The epilogue scales by the reciprocal scales
//     (computed once per tile into LDS while the first stage is in flight),
//     rounds to bfloat16 and, 16 rows at a time, parks them in LDS and streams
//     out whole 256-byte rows with non-temporal stores, so the stores of one
//     group of rows overlap the arithmetic of the next.
#include "fp8_device.hpp"
#include "launchers.hpp"
#include "tuning.hpp"

#include <type_traits>

namespace fp8k {

typedef int v4i_s __attribute__((ext_vector_type(4)));
typedef unsigned v4u_s __attribute__((ext_vector_type(4)));
typedef int v8i_s __attribute__((ext_vector_type(8)));
typedef float v4f_s __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_s __attribute__((ext_vector_type(2)));
typedef float f32x2_s __attribute__((ext_vector_type(2)));

namespace sn {
constexpr int BM = 256, BN = 256, BK = 128;
constexpr int NT = 256;
constexpr int WM = 128, WN = 128;
constexpr int STAGE = (BM + BN) * BK;    // 64 KB
constexpr int GROUP_M = 4;
constexpr int NUM_XCD = 8;
}  // namespace sn

__device__ __forceinline__ uint32_t sn_pack_bf16(float a, float b) {
    f32x2_s v = {a, b};
    bf16x2_s h = __builtin_convertvector(v, bf16x2_s);
    uint32_t r;
    __builtin_memcpy(&r, &h, 4);
    return r;
}

// 16 bytes per lane from a raw buffer straight into LDS at lds_addr + lane * 16
// (lds_addr wave-uniform).  Out-of-range lanes deliver zeros.  Inline assembly
// on purpose: the compiler must not know that these loads write LDS, or it
// would drain them before every LDS read and undo the prefetch.
__device__ __forceinline__ void sn_lds_dma16(v4i_s rsrc, uint32_t lds_addr, uint32_t voffset) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voffset), "s"(rsrc)
                 : "memory", "m0");
}
__device__ __forceinline__ void sn_wait_all_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// Workgroup barrier behind the wave's own LDS reads (no wait for loads in flight).
__device__ __forceinline__ void sn_barrier_lds() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}
// Wait until at most the five youngest loads are in flight (loads complete in issue order), own LDS reads done, barrier.
__device__ __forceinline__ void sn_wait_vmem_but5_barrier() {
    asm volatile("s_waitcnt vmcnt(5) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// logistic function of the dequantized result, for the fused activation epilogue (ACT)
__device__ __forceinline__ float sn_sigmoid(float x) { return __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }

// ACT (bfloat16 output only): out = bfloat16(sigmoid(dequantized product)), the activation behind the
// linear layer in the paper's float8 microbenchmark, applied to the fp32 value before it is rounded
//
// HALF: a workgroup computes HALF a tile - of each wave's 128 x 128 quadrant the rows of ONE A half (64 rows),
// against the whole width.  A launch covers `units` units starting at tile `tile_first`: whole tiles, or with
// HALF the two halves of each tile.  The launcher uses it for the tiles of a last, at most half filled round
// (the weight gradient of the benchmark has 3.5 rounds of tiles): twice as many workgroups of half the
// duration keep every CU busy instead of half of them idling for a whole tile.  A K step is then two
// phases: (A,B0) while B1 arrives, barrier, (A,B1) while the next step's A and B0 arrive and the buffer is
// refilled (12 LDS-DMA loads: only the A rows of this half are fetched).
template <int FA, int FB, bool OUT_F32, bool ACT = false, bool HALF = false>
__global__ __launch_bounds__(sn::NT) void gemm_fp8_snake_kernel(
    const uint8_t* __restrict__ A, int64_t lda, const uint8_t* __restrict__ B, int64_t ldb,
    const float* __restrict__ scale_a, int row_a, const float* __restrict__ scale_b, int row_b, int M, int N,
    int K, void* __restrict__ out, int64_t ld_out, int tiles_m, int tiles_n, int tile_first, int units) {
    using namespace sn;
    static_assert(!(HALF && OUT_F32), "half tiles are built for the bfloat16 epilogue only");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // ---- workgroup -> tile (XCD-aware: ids are dealt round-robin to the 8 XCDs;
    //      each XCD gets a contiguous range of tiles walked in groups of tile rows)
    const int per_xcd = gridDim.x / NUM_XCD;
    const int unit = (blockIdx.x % NUM_XCD) * per_xcd + blockIdx.x / NUM_XCD;
    if (unit >= units) return;
    const int logical = tile_first + (HALF ? unit >> 1 : unit);
    const int ah = HALF ? __builtin_amdgcn_readfirstlane(unit & 1) : 0;     // which A half of every quadrant
    const int in_group = GROUP_M * tiles_n;
    const int first_m = (logical / in_group) * GROUP_M;
    const int gsize = tiles_m - first_m < GROUP_M ? tiles_m - first_m : GROUP_M;
    const int tm = first_m + (logical % in_group) % gsize;
    const int tn = (logical % in_group) / gsize;
    const int m0 = tm * BM, n0 = tn * BN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;

    // ---- buffer descriptors of this tile's operand panels (raw buffers, sizes in bytes)
    const int rows_a = M - m0 < BM ? M - m0 : BM, rows_b = N - n0 < BN ? N - n0 : BN;
    const uint64_t pa = reinterpret_cast<uint64_t>(A + (int64_t)m0 * lda);
    const uint64_t pb = reinterpret_cast<uint64_t>(B + (int64_t)n0 * ldb);
    const v4i_s rsrc_a = {(int)(uint32_t)pa, (int)(uint32_t)(pa >> 32), (int)((int64_t)(rows_a - 1) * lda + K), 0x00020000};
    const v4i_s rsrc_b = {(int)(uint32_t)pb, (int)(uint32_t)(pb >> 32), (int)((int64_t)(rows_b - 1) * ldb + K), 0x00020000};

    // ---- global -> LDS.  Wave w fills row groups w, w+4, ... (8 rows each) of both
    //      tiles; lane l fills (row l/8, chunk slot l%8) with logical chunk slot ^ key(row),
    //      row = 8 * (4 * i + w) + l/8 for load i.
    const int lrow = lane >> 3;
    const int ca = (lane & 7) ^ ((4 * (wave & 1) + (lrow >> 1)) & 7);                 // A: (row >> 1) & 7
    const int cb_e = (lane & 7) ^ (((lrow >> 1) & 1) | (((wave >> 1) & 3) << 1));     // B, even i: (row >> 4) & 3 = wave >> 1
    const int cb_o = (lane & 7) ^ (((lrow >> 1) & 1) | (((2 + (wave >> 1)) & 3) << 1)); // B, odd i
    const uint32_t va0 = (uint32_t)((wave * 8 + lrow) * (int)lda + ca * 16);
    const uint32_t vb0_e = (uint32_t)((wave * 8 + lrow) * (int)ldb + cb_e * 16);
    const uint32_t vb0_o = (uint32_t)((wave * 8 + lrow) * (int)ldb + cb_o * 16);
    const uint32_t va_step = (uint32_t)(32 * (int)lda), vb_step = (uint32_t)(32 * (int)ldb);
    const uint32_t lds_base = (uint32_t)(size_t)smem + (uint32_t)wave * 1024u;
    // a panel offset never reaches 2^31 (checked on the host): adding 2^31 puts a
    // lane outside its descriptor and zeros arrive
    constexpr uint32_t OOB = 0x80000000u;

    auto issue_loads = [&](int stage, int k0) {
        const uint32_t ka = (k0 + ca * 16 < K) ? (uint32_t)k0 : OOB;
        const uint32_t ke = (k0 + cb_e * 16 < K) ? (uint32_t)k0 : OOB;
        const uint32_t ko = (k0 + cb_o * 16 < K) ? (uint32_t)k0 : OOB;
        const uint32_t la = lds_base + (uint32_t)(stage * STAGE), lb = la + BM * BK;
        if constexpr (HALF) {
            // load i covers tile rows [32 i, 32 i + 32): this half needs i = 2 ah + {0, 1, 4, 5}
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                const int i = 2 * ah + (h & 1) + 4 * (h >> 1);
                sn_lds_dma16(rsrc_a, la + (uint32_t)i * 4096u, va0 + (uint32_t)i * va_step + ka);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) sn_lds_dma16(rsrc_a, la + i * 4096, va0 + (uint32_t)i * va_step + ka);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
            sn_lds_dma16(rsrc_b, lb + i * 4096, ((i & 1) ? vb0_o + ko : vb0_e + ke) + (uint32_t)i * vb_step);
    };

    // ---- LDS -> fragments
    const int r16 = lane & 15, g = lane >> 4;
    const int key_a = (r16 >> 1) & 7;
    const int key_b = ((r16 >> 1) & 1) | ((r16 >> 2) << 1);
    int offa[2], offb[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        offa[c] = (wm0 + 64 * ah + r16) * BK + (((g + 4 * c) ^ key_a) << 4);
        offb[c] = BM * BK + (wn0 + 16 * (r16 >> 2) + (r16 & 3)) * BK + (((g + 4 * c) ^ key_b) << 4);
    }
    v8i_s af[2][4], bf[2][4];   // [half][fragment in half]
    auto read_a = [&](const uint8_t* s, int half, int f) {
        const int row_off = (half * 4 + f) * 16 * BK;
        const uint4 x0 = *reinterpret_cast<const uint4*>(s + offa[0] + row_off);
        const uint4 x1 = *reinterpret_cast<const uint4*>(s + offa[1] + row_off);
        af[half][f] = v8i_s{(int)x0.x, (int)x0.y, (int)x0.z, (int)x0.w, (int)x1.x, (int)x1.y, (int)x1.z, (int)x1.w};
    };
    auto read_b = [&](const uint8_t* s, int half, int f) {
        const int row_off = (half * 64 + f * 4) * BK;   // group `half`, fragment t = f
        const uint4 x0 = *reinterpret_cast<const uint4*>(s + offb[0] + row_off);
        const uint4 x1 = *reinterpret_cast<const uint4*>(s + offb[1] + row_off);
        bf[half][f] = v8i_s{(int)x0.x, (int)x0.y, (int)x0.z, (int)x0.w, (int)x1.x, (int)x1.y, (int)x1.z, (int)x1.w};
    };

    // HALF: the four A fragments of this half (its rows are already in offa) into fragment set `dst`
    auto read_ah = [&](const uint8_t* s, auto dst_t, int f) {
        constexpr int DST = decltype(dst_t)::value;
        const int row_off = f * 16 * BK;
        const uint4 x0 = *reinterpret_cast<const uint4*>(s + offa[0] + row_off);
        const uint4 x1 = *reinterpret_cast<const uint4*>(s + offa[1] + row_off);
        af[DST][f] = v8i_s{(int)x0.x, (int)x0.y, (int)x0.z, (int)x0.w, (int)x1.x, (int)x1.y, (int)x1.z, (int)x1.w};
    };

    v4f_s acc[8][8];   // [A fragment][B fragment]
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = v4f_s{0.f, 0.f, 0.f, 0.f};

    // one phase: 16 MFMAs of A half AH x B half BH; in its slots, optionally the
    // reads of one fragment half (RD_A: 1 = A half RH, 0 = B half RH, -1 = none)
    // from stage `rs`, and CNT of the step's sixteen LDS-DMA refill loads, from
    // number L0 on (0-7: the B part, 8-15: the A part).
    auto phase = [&](auto ah_t, auto bh_t, auto rda_t, auto rh_t, auto l0_t, auto cnt_t, const uint8_t* rs, uint32_t la, uint32_t lb,
                     uint32_t ka, uint32_t ke, uint32_t ko) {
        constexpr int AH = decltype(ah_t)::value, BH = decltype(bh_t)::value, RDA = decltype(rda_t)::value,
                      RH = decltype(rh_t)::value, L0 = decltype(l0_t)::value, CNT = decltype(cnt_t)::value;
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            const int i = t >> 2, j = (i & 1) ? 3 - (t & 3) : (t & 3);   // boustrophedon: one operand stays between neighbours
            acc[AH * 4 + i][BH * 4 + j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                bf[BH][j], af[AH][i], acc[AH * 4 + i][BH * 4 + j], FB, FA, 0, 0, 0, 0);
            if constexpr (RDA == 1) { if (t % 2 == 0 && t < 8) read_a(rs, RH, t / 2); }
            if constexpr (RDA == 0) { if (t % 2 == 0 && t < 8) read_b(rs, RH, t / 2); }
            if (t % 2 == 1 && t / 2 < CNT) {
                const int q = L0 + t / 2;
                if (q < 8) sn_lds_dma16(rsrc_b, lb + q * 4096, ((q & 1) ? vb0_o + ko : vb0_e + ke) + (uint32_t)q * vb_step);
                else sn_lds_dma16(rsrc_a, la + (q - 8) * 4096, va0 + (uint32_t)(q - 8) * va_step + ka);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I5 = std::integral_constant<int, 5>;
    using I6 = std::integral_constant<int, 6>;
    using I11 = std::integral_constant<int, 11>;

    // K steps are processed in pairs (the B halves swap roles every step); an odd
    // number of steps gets one phantom step whose loads are all out of range (zeros).
    const int ksteps = (K + BK - 1) / BK;
    const int kpairs = (ksteps + 1) / 2;
    // reciprocal scales of the tile's 256 rows and 256 columns (one correctly
    // rounded divide per thread), computed while the first stage is in flight;
    // the tables sit behind the two stages, where no load ever lands
    float* inv_tab = reinterpret_cast<float*>(smem + 2 * STAGE);       // [0,256): 1/sa, [256,512): 1/sb
    if (ksteps > 0) issue_loads(0, 0);
    {
        const int m = m0 + tid, n = n0 + tid;
        inv_tab[tid] = row_a ? (m < M ? 1.0f / scale_a[m] : 0.f) : 1.0f / scale_a[0];
        inv_tab[256 + tid] = row_b ? (n < N ? 1.0f / scale_b[n] : 0.f) : 1.0f / scale_b[0];
    }
    if (ksteps > 0) {
        sn_wait_all_vmem();
        __syncthreads();                       // stage 0 landed for every wave
        issue_loads(1, BK);                    // (out of range if there is no step 1)
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            if constexpr (HALF) read_ah(smem, I0{}, f); else read_a(smem, 0, f);
            read_b(smem, 0, f);
        }
        __builtin_amdgcn_sched_barrier(0);

        if constexpr (HALF) {
            // two phases per step; fragment set of A and the stage alternate with the step's parity
            auto hstep = [&](auto par_t, int k) {
                constexpr int PAR = decltype(par_t)::value;
                using PN = std::integral_constant<int, PAR ^ 1>;
                const uint8_t* s_cur = smem + PAR * STAGE;
                const uint8_t* s_nxt = smem + (PAR ^ 1) * STAGE;
                const int k2 = (k + 2) * BK;
                const uint32_t ka = (k2 + ca * 16 < K) ? (uint32_t)k2 : OOB;
                const uint32_t ke = (k2 + cb_e * 16 < K) ? (uint32_t)k2 : OOB;
                const uint32_t ko = (k2 + cb_o * 16 < K) ? (uint32_t)k2 : OOB;
                const uint32_t la = lds_base + (uint32_t)(PAR * STAGE), lb = la + BM * BK;
#pragma unroll
                for (int t = 0; t < 16; ++t) {                  // (A, B0) | read B1 of this step
                    const int i = t >> 2, j = (i & 1) ? 3 - (t & 3) : (t & 3);
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bf[0][j], af[PAR][i], acc[i][j], FB, FA, 0, 0, 0, 0);
                    if (t % 2 == 0 && t < 8) read_b(s_cur, 1, t / 2);
                    __builtin_amdgcn_sched_barrier(0);
                }
                sn_wait_all_vmem();                // my part of step k+1 has landed
                __syncthreads();                   // ... and everyone's; this step's buffer is read out
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < 16; ++t) {                  // (A, B1) | read A, B0 of step k+1, refill (12 loads)
                    const int i = t >> 2, j = (i & 1) ? 3 - (t & 3) : (t & 3);
                    acc[i][4 + j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bf[1][j], af[PAR][i], acc[i][4 + j], FB, FA, 0, 0, 0, 0);
                    if (t % 2 == 0 && t < 8) read_ah(s_nxt, PN{}, t / 2);
                    if (t % 2 == 1 && t < 8) read_b(s_nxt, 0, t / 2);
                    if (t >= 4 && t < 8) {
                        const int ia = 2 * ah + ((t - 4) & 1) + 4 * ((t - 4) >> 1);
                        sn_lds_dma16(rsrc_a, la + (uint32_t)ia * 4096u, va0 + (uint32_t)ia * va_step + ka);
                    }
                    if (t >= 8) {
                        const int ib = t - 8;
                        sn_lds_dma16(rsrc_b, lb + ib * 4096, ((ib & 1) ? vb0_o + ko : vb0_e + ke) + (uint32_t)ib * vb_step);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            for (int kp = 0; kp < kpairs; ++kp) {
                hstep(I0{}, 2 * kp);
                hstep(I1{}, 2 * kp + 1);
            }
        } else
        for (int kp = 0; kp < kpairs; ++kp) {
#pragma unroll
            for (int par = 0; par < 2; ++par) {
                const int k = 2 * kp + par;
                const uint8_t* s_cur = smem + par * STAGE;
                const uint8_t* s_nxt = smem + (par ^ 1) * STAGE;
                const int k2 = (k + 2) * BK;   // refill of this step's buffer (all out of range past K)
                const uint32_t ka = (k2 + ca * 16 < K) ? (uint32_t)k2 : OOB;
                const uint32_t ke = (k2 + cb_e * 16 < K) ? (uint32_t)k2 : OOB;
                const uint32_t ko = (k2 + cb_o * 16 < K) ? (uint32_t)k2 : OOB;
                const uint32_t la = lds_base + (uint32_t)(par * STAGE), lb = la + BM * BK;
                // The refill of this step's buffer (sixteen loads) is spread over phases 2-4, so that no phase asks
                // more of the LDS than it has: B part first (read out after phase 1), then the A part (after phase 2).
                if (par == 0) {
                    // even step: B order 0,1,1,0.  Holds A0, B0 of this step.
                    phase(I0{}, I0{}, I0{}, I1{}, I0{}, I0{}, s_cur, la, lb, ka, ke, ko);    // (A0,B0) | read B1 of this step
                    sn_barrier_lds();                  // this step's B part is read out by everyone
                    phase(I0{}, I1{}, I1{}, I1{}, I0{}, I5{}, s_cur, la, lb, ka, ke, ko);    // (A0,B1) | read A1 of this step, refill B 0-4
                    sn_wait_vmem_but5_barrier();       // step k+1 has landed for everyone; this step's A part is read out
                    phase(I1{}, I1{}, I1{}, I0{}, I5{}, I6{}, s_nxt, la, lb, ka, ke, ko);    // (A1,B1) | read A0 of step k+1, refill B 5-7, A 0-2
                    phase(I1{}, I0{}, I0{}, I1{}, I11{}, I5{}, s_nxt, la, lb, ka, ke, ko);   // (A1,B0) | read B1 of step k+1, refill A 3-7
                } else {
                    // odd step: B order 1,0,0,1.  Holds A0, B1 of this step.
                    phase(I0{}, I1{}, I0{}, I0{}, I0{}, I0{}, s_cur, la, lb, ka, ke, ko);    // (A0,B1) | read B0 of this step
                    sn_barrier_lds();
                    phase(I0{}, I0{}, I1{}, I1{}, I0{}, I5{}, s_cur, la, lb, ka, ke, ko);    // (A0,B0) | read A1 of this step, refill B 0-4
                    sn_wait_vmem_but5_barrier();
                    phase(I1{}, I0{}, I1{}, I0{}, I5{}, I6{}, s_nxt, la, lb, ka, ke, ko);    // (A1,B0) | read A0 of step k+1, refill B 5-7, A 0-2
                    phase(I1{}, I1{}, I0{}, I0{}, I11{}, I5{}, s_nxt, la, lb, ka, ke, ko);   // (A1,B1) | read B0 of step k+1, refill A 3-7
                }
            }
        }
        sn_wait_all_vmem();    // trailing (out-of-range) refills must not land in the epilogue's LDS
    }

    // ---- epilogue.  Lane holds output row m = 16*fi + l%16 and, per 64-wide B group,
    //      the 16 consecutive columns 16*g + 4*t + r (fragment t, accumulator r).
    __syncthreads();   // tables visible; nobody's trailing refill can land in the staging rows below

    float inv_b[2][16];
#pragma unroll
    for (int grp = 0; grp < 2; ++grp)
#pragma unroll
        for (int e = 0; e < 16; e += 4) {
            const float4 t4 = *reinterpret_cast<const float4*>(inv_tab + 256 + wn0 + 64 * grp + 16 * g + e);
            inv_b[grp][e] = t4.x; inv_b[grp][e + 1] = t4.y; inv_b[grp][e + 2] = t4.z; inv_b[grp][e + 3] = t4.w;
        }

    if constexpr (OUT_F32) {
#pragma unroll
        for (int fi = 0; fi < 8; ++fi) {
            const int r_loc = 16 * fi + r16;               // row inside the wave's quadrant
            const float inv_a = inv_tab[wm0 + r_loc];
            const int m = m0 + wm0 + r_loc;
#pragma unroll
            for (int grp = 0; grp < 2; ++grp) {
                float v[16];
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[4 * t + r] = (acc[fi][grp * 4 + t][r] * inv_a) * inv_b[grp][4 * t + r];
                const int nb = n0 + wn0 + 64 * grp + 16 * g;
                if (m < M && nb < N) {
                    float* dst = static_cast<float*>(out) + (int64_t)m * ld_out + nb;
                    if (nb + 16 <= N) {
#pragma unroll
                        for (int e = 0; e < 16; e += 4)
                            *reinterpret_cast<float4*>(dst + e) = make_float4(v[e], v[e + 1], v[e + 2], v[e + 3]);
                    } else {
                        for (int e = 0; nb + e < N; ++e) dst[e] = v[e];
                    }
                }
            }
        }
    } else {
        // bfloat16: 16 rows at a time are scaled, rounded, parked in this wave's own
        // 32 KB of LDS (row = 256 bytes = 16 chunks, chunk c stored at c ^ (row & 15))
        // and streamed out as whole 256-byte rows, so the stores of one group of
        // rows overlap the arithmetic of the next.  LDS operations of one wave
        // execute in order; the wave barrier only keeps the compiler from moving
        // the reads above the writes.
        uint8_t* q = smem + wave * 32768;
        const int c_rd = lane & 15;                        // chunk this lane streams out
        const int n_rd = n0 + wn0 + c_rd * 8;
        const bool interior = m0 + BM <= M && n0 + BN <= N;
        uint16_t* orow = static_cast<uint16_t*>(out) + (int64_t)(m0 + wm0 + 64 * ah + (lane >> 4)) * ld_out + n_rd;
#pragma unroll
        for (int fi = 0; fi < (HALF ? 4 : 8); ++fi) {
            const int r_loc = 64 * ah + 16 * fi + r16;
            const float inv_a = inv_tab[wm0 + r_loc];
            uint8_t* row = q + r_loc * 256;
#pragma unroll
            for (int grp = 0; grp < 2; ++grp) {
                uint32_t p[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int e0 = 2 * e, e1 = 2 * e + 1;
                    float u0 = (acc[fi][grp * 4 + (e0 >> 2)][e0 & 3] * inv_a) * inv_b[grp][e0];
                    float u1 = (acc[fi][grp * 4 + (e1 >> 2)][e1 & 3] * inv_a) * inv_b[grp][e1];
                    if constexpr (ACT) { u0 = sn_sigmoid(u0); u1 = sn_sigmoid(u1); }
                    p[e] = sn_pack_bf16(u0, u1);
                }
                const int c = 8 * grp + 2 * g;
                *reinterpret_cast<uint4*>(row + ((c ^ r16) << 4)) = make_uint4(p[0], p[1], p[2], p[3]);
                *reinterpret_cast<uint4*>(row + (((c + 1) ^ r16) << 4)) = make_uint4(p[4], p[5], p[6], p[7]);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int rr = 64 * ah + 16 * fi + 4 * it + (lane >> 4);      // row in the quadrant
                const uint4 v = *reinterpret_cast<const uint4*>(q + rr * 256 + ((c_rd ^ (rr & 15)) << 4));
                uint16_t* dst = orow + (int64_t)(16 * fi + 4 * it) * ld_out;
                if (interior) {
                    // streaming store: the output is not read again by this kernel and
                    // should not push the operand panels out of L2
                    __builtin_nontemporal_store(v4u_s{v.x, v.y, v.z, v.w}, reinterpret_cast<v4u_s*>(dst));
                } else if (m0 + wm0 + rr < M && n_rd < N) {
                    if (n_rd + 8 <= N) {
                        __builtin_nontemporal_store(v4u_s{v.x, v.y, v.z, v.w}, reinterpret_cast<v4u_s*>(dst));
                    } else {
                        const uint32_t w4[4] = {v.x, v.y, v.z, v.w};
                        for (int e = 0; n_rd + e < N; ++e) dst[e] = (uint16_t)(w4[e >> 1] >> ((e & 1) * 16));
                    }
                }
            }
        }
    }
}

template <int FA, int FB, bool OUT_F32, bool ACT, bool HALF>
static hipError_t launch_sn_part(const uint8_t* a, int64_t lda, const float* sa, int row_a, const uint8_t* b, int64_t ldb,
                                 const float* sb, int row_b, int M, int N, int K, void* out, int64_t ld_out, int tiles_m,
                                 int tiles_n, int tile_first, int64_t units, hipStream_t st) {
    using namespace sn;
    auto kern = gemm_fp8_snake_kernel<FA, FB, OUT_F32, ACT, HALF>;
    constexpr int lds = 2 * STAGE + 2048;   // two stages + the reciprocal-scale tables of the epilogue
    static DynamicLdsOnce attr;
    if (hipError_t e = attr.ensure(reinterpret_cast<const void*>(kern), lds); e != hipSuccess) return e;
    const int64_t grid = (units + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
    if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
    kern<<<dim3((unsigned)grid), dim3(NT), lds, st>>>(a, lda, b, ldb, sa, row_a, sb, row_b, M, N, K, out, ld_out,
                                                      tiles_m, tiles_n, tile_first, (int)units);
    return hipGetLastError();
}

template <int FA, int FB, bool OUT_F32, bool ACT = false>
static hipError_t launch_sn(const uint8_t* a, int64_t lda, const float* sa, int row_a, const uint8_t* b, int64_t ldb,
                            const float* sb, int row_b, int M, int N, int K, void* out, int64_t ld_out,
                            hipStream_t st) {
    using namespace sn;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int64_t ntiles = (int64_t)tiles_m * tiles_n;
    if (ntiles > 0x3FFFFFFF) return hipErrorInvalidValue;
    // whole tiles go to the persistent form of this kernel when there is more than one round of them (it overlaps a
    // tile's epilogue with the next tile's products: nothing to overlap with one tile per CU)
    const int sw = knob(KNOB_GEMM_STREAM);
    const bool stream_ok = sw != 0 && gemm_fp8_stream_fits(lda, ldb, ld_out, N, K, OUT_F32, ACT);
    auto whole_tiles = [&](int64_t count) -> hipError_t {
        if (stream_ok && (sw >= 2 || count > compute_units()))
            return launch_gemm_fp8_stream(a, lda, FA, sa, row_a, b, ldb, FB, sb, row_b, M, N, K, out, ld_out, count, 256, st);
        return launch_sn_part<FA, FB, OUT_F32, ACT, false>(a, lda, sa, row_a, b, ldb, sb, row_b, M, N, K, out, ld_out, tiles_m, tiles_n,
                                                          0, count, st);
    };
    if (stream_ok && (sw >= 2 || ntiles > compute_units())) {
        // a lower tile (224 or 192 rows) when its tile count fills whole rounds of workgroups better than 256-row
        // tiles with their partly filled last round do: then the persistent kernel takes every tile
        const int tm = gemm_fp8_stream_tile_m(M, N);
        if (tm != 256) {
            const int64_t cus = compute_units() > 0 ? compute_units() : 256;
            const int64_t rest = ntiles % cus;
            // cost of the 256-row plan in rows per CU: whole rounds, plus a last round of half tiles (measured at
            // 0.85 of a whole round) or of whole tiles
            const double cost256 = 256.0 * ((double)(ntiles / cus) + (rest == 0 ? 0.0 : (2 * rest <= cus ? 0.85 : 1.0)));
            const int64_t tiles_tm = ((int64_t)M + tm - 1) / tm * tiles_n;
            const double cost_tm = (double)tm * (double)((tiles_tm + cus - 1) / cus);
            if (cost_tm < 0.97 * cost256 || knob(KNOB_GEMM_TILE_M) == tm)
                return launch_gemm_fp8_stream(a, lda, FA, sa, row_a, b, ldb, FB, sb, row_b, M, N, K, out, ld_out, tiles_tm, tm, st);
        }
    }
    if constexpr (!OUT_F32) {
        // A last round that would fill at most half of the CUs runs as half tiles instead: twice the
        // workgroups, half the duration each (the switch SNAKE_HALF = 0 keeps whole tiles; tuning and test aid).
        const int cus = compute_units();
        const int64_t rest = cus > 0 ? ntiles % cus : 0;
        if (knob(KNOB_SNAKE_HALF) != 0 && cus >= 16 && cus % NUM_XCD == 0 && rest > 0 && 2 * rest <= cus) {
            const int64_t full = ntiles - rest;
            if (full > 0) {
                hipError_t err = whole_tiles(full);
                if (err != hipSuccess) return err;
            }
            return launch_sn_part<FA, FB, OUT_F32, ACT, true>(a, lda, sa, row_a, b, ldb, sb, row_b, M, N, K, out, ld_out, tiles_m,
                                                              tiles_n, (int)full, 2 * rest, st);
        }
    }
    return whole_tiles(ntiles);
}

bool gemm_fp8_snake_fits(int64_t lda, int64_t ldb) { return lda < (1 << 23) && ldb < (1 << 23); }

hipError_t launch_gemm_fp8_snake(const uint8_t* a, int64_t lda, int fmt_a, const float* scale_a, int row_a,
                                 const uint8_t* b, int64_t ldb, int fmt_b, const float* scale_b, int row_b,
                                 int64_t M, int64_t N, int64_t K, void* out, int64_t ld_out, int out_f32,
                                 hipStream_t st, int act) {
    if (M == 0 || N == 0) return hipSuccess;
    if (act && out_f32) return hipErrorInvalidValue;
    const int m = (int)M, n = (int)N, k = (int)K;
#define FP8K_SNA(FA_, FB_)                                                                                 \
    if (act && fmt_a == FA_ && fmt_b == FB_)                                                               \
        return launch_sn<FA_, FB_, false, true>(a, lda, scale_a, row_a, b, ldb, scale_b, row_b, m, n, k, out, ld_out, st)
    FP8K_SNA(FMT_E4M3FN, FMT_E4M3FN);
    FP8K_SNA(FMT_E5M2, FMT_E4M3FN);
    FP8K_SNA(FMT_E4M3FN, FMT_E5M2);
    FP8K_SNA(FMT_E5M2, FMT_E5M2);
#undef FP8K_SNA
#define FP8K_SN(FA_, FB_)                                                                                  \
    if (fmt_a == FA_ && fmt_b == FB_)                                                                      \
        return out_f32 ? launch_sn<FA_, FB_, true>(a, lda, scale_a, row_a, b, ldb, scale_b, row_b, m, n, k, out, ld_out, st) \
                       : launch_sn<FA_, FB_, false>(a, lda, scale_a, row_a, b, ldb, scale_b, row_b, m, n, k, out, ld_out, st)
    FP8K_SN(FMT_E4M3FN, FMT_E4M3FN);
    FP8K_SN(FMT_E5M2, FMT_E4M3FN);
    FP8K_SN(FMT_E4M3FN, FMT_E5M2);
    FP8K_SN(FMT_E5M2, FMT_E5M2);
#undef FP8K_SN
    return hipErrorInvalidValue;
}

}  // namespace fp8k
