// Pipelined scaled FP8 GEMM for gfx950: 256 x 256 tile, four wavefronts, each
// owning a 128 x 128 quadrant as 4 x 4 tiles of v_mfma_f32_32x32x64_f8f6f4.
// out[M,N] = (A[M,K] . B[N,K]^T) / (sa * sb), both operands K-contiguous.
//
// Why this shape: at the dense FP8 rate a 256 x 256 x 128 step is 2048 matrix
// core cycles per CU while it moves 64 KB from L2 (half of the CU's 64 B/clk)
// and 128 KB out of LDS (a quarter of its 256 B/clk); smaller tiles or
// narrower wave tiles raise those fractions past what can overlap.
//
// Data movement
//   - Global -> LDS goes through buffer_load_dwordx4 ... lds (no staging
//     registers): one wave instruction fills 1024 contiguous LDS bytes = 8 rows
//     of 128 K-bytes.  Lane l fills (row l/8, chunk slot l%8) and therefore
//     fetches logical 16-byte chunk (l%8) ^ key(row) of that row, key(row) =
//     (row >> 1) & 7: the XOR swizzle is applied on the global side.  Rows past M / N are cut off by
//     the buffer descriptor's size (the hardware returns zeros), chunks past K
//     by pointing the lane's offset outside the descriptor.
//   - Two LDS stages of 64 KB.  The loads of step k+2 are issued in the middle
//     of step k, right after the barrier that retires step k's stage, and are
//     waited for in the middle of step k+1: a full step (2048 cycles at peak)
//     of latency cover.
//   - LDS -> registers in K halves: a 32x32x64 MFMA takes 32 rows x 64 bytes,
//     lane l supplying chunks {h, h+2} (h = l/32) of the half for row l%32.
//     Both operands use the same assignment.  A 64-lane 128-bit LDS read is
//     served as two halves of 32 lanes, and within a half each of the 16 bank
//     groups (16 bytes wide, 256-byte wrap) may be hit twice: with key(row) =
//     (row >> 1) & 7 the 32 rows of a fragment give every (row parity, chunk
//     slot) pair exactly twice, so the reads run at the full 256 B/clk
//     (key = row & 7 measures at half of that).
//     Two register sets alternate: while the matrix cores work on one K half,
//     the fragments of the next half are read.
//   - The B tile is the first MFMA operand, A the second: a lane's accumulators
//     belong to one output row m.  B rows are dealt to the MFMA row index i as
//     n = 16*((i/4)%2) + 4*(i/8) + i%4, which makes the 16 accumulators of a
//     lane 16 consecutive n.  The epilogue scales, rounds to bfloat16, parks the
//     quadrant in LDS and writes whole 256-byte rows (scattered 32-byte pieces
//     straight from registers cost ~20 us per tile, ~3 us this way).
//   - Workgroup ids are dealt round-robin to the 8 XCDs by the hardware; each
//     XCD gets one contiguous range of tiles walked in groups of tile rows, so
//     concurrently running tiles share operand panels in that XCD's L2.
#include "fp8_device.hpp"
#include "launchers.hpp"
#include <cstdlib>
#include <type_traits>

namespace fp8k {

typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef unsigned v4u_t __attribute__((ext_vector_type(4)));
typedef int v8i_t __attribute__((ext_vector_type(8)));
typedef float v16f_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

namespace pl {
constexpr int BM = 256, BN = 256, BK = 128;
constexpr int NT = 256;                  // four wavefronts, 2 x 2
constexpr int WM = 128, WN = 128;
constexpr int STAGE = (BM + BN) * BK;    // 64 KB
constexpr int GROUP_M = 4;
constexpr int NUM_XCD = 8;
}  // namespace pl

__device__ __forceinline__ uint32_t pack_bf16_rne(float a, float b) {
    f32x2_t v = {a, b};
    bf16x2_t h = __builtin_convertvector(v, bf16x2_t);
    uint32_t r;
    __builtin_memcpy(&r, &h, 4);
    return r;
}

// 16 bytes per lane from a raw buffer straight into LDS at lds_addr + lane * 16
// (lds_addr wave-uniform).  Out-of-range lanes deliver zeros.
__device__ __forceinline__ void lds_dma16(v4i_t rsrc, uint32_t lds_addr, uint32_t voffset) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voffset), "s"(rsrc)
                 : "memory", "m0");
}
__device__ __forceinline__ void wait_all_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

template <int FA, int FB, bool OUT_F32>
__global__ __launch_bounds__(pl::NT) void gemm_fp8_pipelined_kernel(
    const uint8_t* __restrict__ A, int64_t lda, const uint8_t* __restrict__ B, int64_t ldb,
    const float* __restrict__ scale_a, int row_a, const float* __restrict__ scale_b, int row_b, int M, int N,
    int K, void* __restrict__ out, int64_t ld_out, int tiles_m, int tiles_n) {
    using namespace pl;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    
    // ---- workgroup -> tile (XCD-aware)
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

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: LDS-DMA bases live in M0
    const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;

    // ---- buffer descriptors of this tile's operand panels (raw buffers, sizes in bytes)
    const int rows_a = M - m0 < BM ? M - m0 : BM, rows_b = N - n0 < BN ? N - n0 : BN;
    const uint64_t pa = reinterpret_cast<uint64_t>(A + (int64_t)m0 * lda);
    const uint64_t pb = reinterpret_cast<uint64_t>(B + (int64_t)n0 * ldb);
    const v4i_t rsrc_a = {(int)(uint32_t)pa, (int)(uint32_t)(pa >> 32), (int)((int64_t)(rows_a - 1) * lda + K), 0x00020000};
    const v4i_t rsrc_b = {(int)(uint32_t)pb, (int)(uint32_t)(pb >> 32), (int)((int64_t)(rows_b - 1) * ldb + K), 0x00020000};

    // wave w fills row groups w, w+4, ... (8 rows each) of both operand tiles
    const int lrow = lane >> 3;                         // row inside the 8-row group
    // logical chunk this lane fetches: slot ^ key(row), key(row) = (row >> 1) & 7 with
    // row = 8 * (4 * i + wave) + lrow, i.e. 4 * (wave & 1) + lrow / 2 for every i
    const int lchunk = (lane & 7) ^ (4 * (wave & 1) + (lrow >> 1));
    const uint32_t va0 = (uint32_t)((wave * 8 + lrow) * (int)lda + lchunk * 16);
    const uint32_t vb0 = (uint32_t)((wave * 8 + lrow) * (int)ldb + lchunk * 16);
    const uint32_t va_step = (uint32_t)(32 * (int)lda), vb_step = (uint32_t)(32 * (int)ldb);
    const uint32_t lds_base = (uint32_t)(size_t)smem + (uint32_t)wave * 1024u;

    // The loads are inline assembly on purpose: the compiler must not know that
    // they write LDS, or it would drain them (vmcnt 0) before every LDS read and
    // undo the prefetch.  They are waited for explicitly before the barrier that
    // publishes a stage.  A panel offset never reaches 2^31 (checked on the
    // host), so adding 2^31 puts a lane outside its descriptor: zeros arrive.
    auto issue_loads = [&](int stage, int k0) {
        const uint32_t koff = (k0 + lchunk * 16 < K) ? (uint32_t)k0 : 0x80000000u;
        const uint32_t la = lds_base + (uint32_t)(stage * STAGE), lb = la + BM * BK;
#pragma unroll
        for (int i = 0; i < 8; ++i) lds_dma16(rsrc_a, la + i * 4096, va0 + (uint32_t)i * va_step + koff);
#pragma unroll
        for (int i = 0; i < 8; ++i) lds_dma16(rsrc_b, lb + i * 4096, vb0 + (uint32_t)i * vb_step + koff);
    };

    // ---- LDS -> fragments
    const int l32 = lane & 31, h = lane >> 5;
    const int perm = 16 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3);   // B row for MFMA row index l32
    const int a_row_off = (wm0 + l32) * BK, b_row_off = (wn0 + perm) * BK;
    const int key_a = (l32 >> 1) & 7, key_b = (perm >> 1) & 7;
    // chunk offsets for K half 0: {h, h+2}; half 1 adds 4 to the logical chunk
    int offa[2][2], offb[2][2];
#pragma unroll
    for (int kh = 0; kh < 2; ++kh)
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            offa[kh][c] = a_row_off + (((4 * kh + h + 2 * c) ^ key_a) << 4);
            offb[kh][c] = BM * BK + b_row_off + (((4 * kh + h + 2 * c) ^ key_b) << 4);
        }

    v8i_t af[2][4], bf[2][4];
    // one fragment = two 128-bit reads; `which` 0..3 = A fragments, 4..7 = B fragments
    auto read_frag = [&](const uint8_t* s, int kh, int set, int which) {
        if (which < 4) {
            const uint4 a0 = *reinterpret_cast<const uint4*>(s + offa[kh][0] + which * 32 * BK);
            const uint4 a1 = *reinterpret_cast<const uint4*>(s + offa[kh][1] + which * 32 * BK);
            af[set][which] = v8i_t{(int)a0.x, (int)a0.y, (int)a0.z, (int)a0.w, (int)a1.x, (int)a1.y, (int)a1.z, (int)a1.w};
        } else {
            const int f = which - 4;
            const uint4 b0 = *reinterpret_cast<const uint4*>(s + offb[kh][0] + f * 32 * BK);
            const uint4 b1 = *reinterpret_cast<const uint4*>(s + offb[kh][1] + f * 32 * BK);
            bf[set][f] = v8i_t{(int)b0.x, (int)b0.y, (int)b0.z, (int)b0.w, (int)b1.x, (int)b1.y, (int)b1.z, (int)b1.w};
        }
    };

    v16f_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // The 16 MFMAs of a K half are issued in 2 x 2 blocks of (A fragment, B
    // fragment) pairs, and the fragments of the next half are read in the order
    // in which those blocks will need them.  Every slot = one MFMA (64 cycles
    // of matrix core time) plus at most one fragment read and one LDS-DMA load,
    // pinned with scheduling barriers so the issue work hides under the MFMAs.
    constexpr int MI[16] = {0, 0, 1, 1, 0, 0, 1, 1, 2, 2, 3, 3, 2, 2, 3, 3};
    constexpr int MJ[16] = {0, 1, 0, 1, 2, 3, 2, 3, 0, 1, 0, 1, 2, 3, 2, 3};
    constexpr int RD[8] = {0, 4, 5, 1, 6, 7, 2, 3};   // read order: a0 b0 b1 a1 b2 b3 a2 a3

    const int ksteps = (K + BK - 1) / BK;
    if (ksteps > 0) {
        issue_loads(0, 0);
        wait_all_vmem();
        __syncthreads();                       // stage 0 landed for every wave
        if (ksteps > 1) issue_loads(1, BK);
#pragma unroll
        for (int q = 0; q < 8; ++q) read_frag(smem, 0, 0, RD[q]);
        __builtin_amdgcn_sched_barrier(0);
        // one K step; WITH_DMA = refill the retired stage with step k+2
        auto k_step = [&](auto with_dma, int k) {
            const int cur = k & 1;
            const uint8_t* s_cur = smem + cur * STAGE;
            const uint8_t* s_nxt = smem + (cur ^ 1) * STAGE;
            // ---- first K half: MFMAs on set 0, read the second half into set 1
#pragma unroll
            for (int t = 0; t < 16; ++t) {
                acc[MI[t]][MJ[t]] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bf[0][MJ[t]], af[0][MI[t]],
                                                                                     acc[MI[t]][MJ[t]], FB, FA, 0, 0, 0, 0);
                if (t < 8) read_frag(s_cur, 1, 1, RD[t]);
                __builtin_amdgcn_sched_barrier(0);
            }
            wait_all_vmem();                   // my part of step k+1 has landed
            __syncthreads();                   // ... and everyone's; everyone is done reading stage cur
            __builtin_amdgcn_sched_barrier(0);
            // ---- second K half: MFMAs on set 1; refill stage cur with step k+2,
            //      read the first half of step k+1 into set 0 (after the last step
            //      that read fetches a stage nobody uses: no branch in the slots)
            const uint32_t koff = ((k + 2) * BK + lchunk * 16 < K) ? (uint32_t)((k + 2) * BK) : 0x80000000u;
            const uint32_t la = lds_base + (uint32_t)(cur * STAGE), lb = la + BM * BK;
#pragma unroll
            for (int t = 0; t < 16; ++t) {
                acc[MI[t]][MJ[t]] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bf[1][MJ[t]], af[1][MI[t]],
                                                                                     acc[MI[t]][MJ[t]], FB, FA, 0, 0, 0, 0);
                if constexpr (decltype(with_dma)::value) {
                    if (t < 8) lds_dma16(rsrc_a, la + t * 4096, va0 + (uint32_t)t * va_step + koff);
                    else       lds_dma16(rsrc_b, lb + (t - 8) * 4096, vb0 + (uint32_t)(t - 8) * vb_step + koff);
                }
                if (t < 8) read_frag(s_nxt, 0, 0, RD[t]);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        int k = 0;
        for (; k + 2 < ksteps; ++k) k_step(std::true_type{}, k);
        for (; k < ksteps; ++k) k_step(std::false_type{}, k);      // nothing left to prefetch
    }

    // ---- epilogue.  Lane holds output row m = .. + l32 and, per B fragment j,
    //      the 16 consecutive columns n = 32*j + 16*h + r (accumulator r is MFMA
    //      row 8*(r/4) + 4*h + r%4, which the B row permutation maps to n offset r).
    //      The reciprocal scales of the tile's 256 rows and 256 columns are
    //      computed once (one correctly rounded divide per thread) into LDS.
    float* inv_tab = reinterpret_cast<float*>(smem + 2 * STAGE);       // [0,256): 1/sa, [256,512): 1/sb
    {
        const int m = m0 + tid, n = n0 + tid;
        inv_tab[tid] = row_a ? (m < M ? 1.0f / scale_a[m] : 0.f) : 1.0f / scale_a[0];
        inv_tab[256 + tid] = row_b ? (n < N ? 1.0f / scale_b[n] : 0.f) : 1.0f / scale_b[0];
    }
    __syncthreads();   // tables visible; every wave is past its last LDS read of the stages

    if constexpr (OUT_F32) {
        // fp32 output: straight from registers, 64 contiguous bytes per lane
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int nl = wn0 + 32 * j + 16 * h, nb = n0 + nl;
            float inv_b[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) inv_b[e] = inv_tab[256 + nl + e];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int ml = wm0 + 32 * i + l32, m = m0 + ml;
                if (m >= M || nb >= N) continue;
                const float inv_a = inv_tab[ml];
                float* dst = static_cast<float*>(out) + (int64_t)m * ld_out + nb;
                float v[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) v[r] = (acc[i][j][r] * inv_a) * inv_b[r];
                if (nb + 16 <= N) {
#pragma unroll
                    for (int e = 0; e < 16; e += 4)
                        *reinterpret_cast<float4*>(dst + e) = make_float4(v[e], v[e + 1], v[e + 2], v[e + 3]);
                } else {
                    for (int e = 0; nb + e < N; ++e) dst[e] = v[e];
                }
            }
        }
    } else {
        // bfloat16 output: each wave parks its 128 x 128 quadrant in its own 32 KB
        // of LDS (row = 256 bytes = 16 chunks, chunk c stored at c ^ (row & 15):
        // conflict-free both ways) and streams it out as whole rows, 16 lanes x
        // 16 bytes = 256 contiguous bytes per row.
        uint8_t* q = smem + wave * 32768;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int nl = wn0 + 32 * j + 16 * h;
            float inv_b[16];
#pragma unroll
            for (int e = 0; e < 16; e += 4) {
                const float4 t4 = *reinterpret_cast<const float4*>(inv_tab + 256 + nl + e);
                inv_b[e] = t4.x; inv_b[e + 1] = t4.y; inv_b[e + 2] = t4.z; inv_b[e + 3] = t4.w;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r_loc = 32 * i + l32;
                const float inv_a = inv_tab[wm0 + r_loc];
                uint32_t p[8];
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    p[e] = pack_bf16_rne((acc[i][j][2 * e] * inv_a) * inv_b[2 * e], (acc[i][j][2 * e + 1] * inv_a) * inv_b[2 * e + 1]);
                const int c = 4 * j + 2 * h;
                uint8_t* row = q + r_loc * 256;
                *reinterpret_cast<uint4*>(row + (((c) ^ (r_loc & 15)) << 4)) = make_uint4(p[0], p[1], p[2], p[3]);
                *reinterpret_cast<uint4*>(row + (((c + 1) ^ (r_loc & 15)) << 4)) = make_uint4(p[4], p[5], p[6], p[7]);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int c = lane & 15;
        const int n = n0 + wn0 + c * 8;
        uint16_t* obase = static_cast<uint16_t*>(out) + n;
#pragma unroll 8
        for (int it = 0; it < 32; ++it) {
            const int r_loc = it * 4 + (lane >> 4);
            const int m = m0 + wm0 + r_loc;
            const uint4 v = *reinterpret_cast<const uint4*>(q + r_loc * 256 + ((c ^ (r_loc & 15)) << 4));
            if (m < M && n < N) {
                uint16_t* dst = obase + (int64_t)m * ld_out;
                if (n + 8 <= N) {
                    // streaming store: the output is not read again by this kernel and
                    // should not push the operand panels out of L2
                    __builtin_nontemporal_store(v4u_t{v.x, v.y, v.z, v.w}, reinterpret_cast<v4u_t*>(dst));
                } else {
                    const uint32_t w4[4] = {v.x, v.y, v.z, v.w};
                    for (int e = 0; n + e < N; ++e) dst[e] = (uint16_t)(w4[e >> 1] >> ((e & 1) * 16));
                }
            }
        }
    }
}

template <int FA, int FB, bool OUT_F32>
static hipError_t launch_pl(const uint8_t* a, int64_t lda, const float* sa, int row_a, const uint8_t* b, int64_t ldb,
                            const float* sb, int row_b, int M, int N, int K, void* out, int64_t ld_out,
                            hipStream_t st) {
    using namespace pl;
    auto kern = gemm_fp8_pipelined_kernel<FA, FB, OUT_F32>;
    constexpr int lds = 2 * STAGE + 2048;   // two stages + the reciprocal-scale tables of the epilogue
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int64_t ntiles = (int64_t)tiles_m * tiles_n;
    const int64_t grid = (ntiles + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
    if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
    kern<<<dim3((unsigned)grid), dim3(NT), lds, st>>>(a, lda, b, ldb, sa, row_a, sb, row_b, M, N, K, out, ld_out,
                                                      tiles_m, tiles_n);
    return hipGetLastError();
}

// The panel offsets are 32-bit: a 256-row panel must stay below 4 GiB.
bool gemm_fp8_pipelined_supported(int64_t lda, int64_t ldb) {
    return lda < (1 << 23) && ldb < (1 << 23);
}

hipError_t launch_gemm_fp8_pipelined(const uint8_t* a, int64_t lda, int fmt_a, const float* scale_a, int row_a,
                                     const uint8_t* b, int64_t ldb, int fmt_b, const float* scale_b, int row_b,
                                     int64_t M, int64_t N, int64_t K, void* out, int64_t ld_out, int out_f32,
                                     hipStream_t st) {
    if (M == 0 || N == 0) return hipSuccess;
    const int m = (int)M, n = (int)N, k = (int)K;
#define FP8K_PL(FA_, FB_)                                                                                  \
    if (fmt_a == FA_ && fmt_b == FB_)                                                                      \
        return out_f32 ? launch_pl<FA_, FB_, true>(a, lda, scale_a, row_a, b, ldb, scale_b, row_b, m, n, k, out, ld_out, st) \
                       : launch_pl<FA_, FB_, false>(a, lda, scale_a, row_a, b, ldb, scale_b, row_b, m, n, k, out, ld_out, st)
    FP8K_PL(FMT_E4M3FN, FMT_E4M3FN);
    FP8K_PL(FMT_E5M2, FMT_E4M3FN);
    FP8K_PL(FMT_E4M3FN, FMT_E5M2);
    FP8K_PL(FMT_E5M2, FMT_E5M2);
#undef FP8K_PL
    return hipErrorInvalidValue;
}

}  // namespace fp8k
