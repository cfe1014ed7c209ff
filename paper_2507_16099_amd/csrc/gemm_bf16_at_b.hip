// bfloat16 GEMM with the contraction axis on the ROWS of both operands:
//     out[i, j] = sum_c a[c, i] * b[c, j]        (a [C, I], b [C, J] row-major, fp32 accumulate, bf16 out)
// This is the weight gradient dW = dY^T X of a linear layer computed from the
// unquantized tensors, which the rowwise_gw_hp recipe keeps in high precision
// (Appendix A: the grad_weight GEMM is the one most sensitive to low precision):
// a = dY [M, N], b = X [M, K], out = dW [N, K], contraction over the M tokens.
//
// v_mfma_f32_16x16x32_bf16 wants, per lane, 8 consecutive contraction elements
// of one operand row, but here the contraction index is the slow axis of both
// operands in memory.  The transposition is done on the way into LDS: a thread
// loads an 8 (c) x 8 (i) block with eight 128-bit loads (a wavefront reads two
// 512-byte runs per load), transposes it in registers with 32 v_perm_b32 and
// writes eight 16-byte pieces, one per operand row, so that LDS holds the
// operands as rows of 64 contraction elements (128 bytes) like the FP8 kernels
// do.  From there on it is the register-staged scheme of gemm_fp8.hip: 256 x 256
// tile, 8 wavefronts (2 x 4) of 128 x 64, two LDS stages of 64 KB, the next step's
// global loads in flight while the matrix cores work on the current one.
//
// LDS layout.  Row r of an operand tile lives at physical row
// (r & ~7) | ((r & 7) ^ ((r >> 4) & 7)); chunk c (16 bytes = 8 contraction
// elements) at position c ^ ((physical row >> 1) & 7).  The first permutation
// makes the transposed 128-bit writes of a wavefront (same element index e in
// every lane, rows 8 apart) hit every bank group twice per half-wavefront
// instead of 16 times; the second is the conflict-free read pattern of the FP8
// kernels (a 16-row fragment is a permutation of 16 consecutive physical rows).
#include "fp8_device.hpp"
#include "launchers.hpp"
#include "tuning.hpp"


namespace fp8k {

typedef __bf16 v8bf_t __attribute__((ext_vector_type(8)));
typedef float v4f_b __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_b __attribute__((ext_vector_type(2)));
typedef float f32x2_b __attribute__((ext_vector_type(2)));

namespace bt {
constexpr int BI = 256, BJ = 256, BC = 64;   // output tile and contraction elements per step
constexpr int NT = 512;                      // 8 wavefronts, 2 (i) x 4 (j)
constexpr int WI = 128, WJ = 64;
constexpr int FI = WI / 16, FJ = WJ / 16;    // fragments per wavefront
constexpr int ROWB = BC * 2;                 // bytes per LDS row
constexpr int STAGE = (BI + BJ) * ROWB;      // 64 KB
constexpr int GROUP_I = 4, NUM_XCD = 8;
}  // namespace bt

__device__ __forceinline__ uint32_t bt_pack_bf16(float a, float b) {
    f32x2_b v = {a, b};
    bf16x2_b h = __builtin_convertvector(v, bf16x2_b);
    uint32_t r;
    __builtin_memcpy(&r, &h, 4);
    return r;
}
__device__ __forceinline__ int bt_phys_row(int r) { return (r & ~7) | ((r & 7) ^ ((r >> 4) & 7)); }

__global__ __launch_bounds__(bt::NT) void gemm_bf16_at_b_kernel(const uint16_t* __restrict__ A, int64_t lda,
                                                                 const uint16_t* __restrict__ B, int64_t ldb, int I, int J,
                                                                 int C, uint16_t* __restrict__ out, int64_t ld_out,
                                                                 int tiles_i, int tiles_j) {
    using namespace bt;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // ---- workgroup -> tile (XCD-aware, as in the FP8 kernels)
    const int ntiles = tiles_i * tiles_j;
    const int per_xcd = gridDim.x / NUM_XCD;
    const int logical = (blockIdx.x % NUM_XCD) * per_xcd + blockIdx.x / NUM_XCD;
    if (logical >= ntiles) return;
    const int in_group = GROUP_I * tiles_j;
    const int first_i = (logical / in_group) * GROUP_I;
    const int gsize = tiles_i - first_i < GROUP_I ? tiles_i - first_i : GROUP_I;
    const int ti = first_i + (logical % in_group) % gsize;
    const int tj = (logical % in_group) / gsize;
    const int i0 = ti * BI, j0 = tj * BJ;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wi0 = (wave >> 2) * WI, wj0 = (wave & 3) * WJ;

    // ---- global -> registers: thread owns the 8 (c) x 8 (column) block (cblk, xblk) of a (threads
    //      0..255) or of b (256..511)
    const int which = tid >> 8, blk = tid & 255;
    const int xblk = blk & 31, cblk = blk >> 5;
    const uint16_t* src = which ? B : A;
    const int64_t ld = which ? ldb : lda;
    const int x0 = (which ? j0 : i0) + xblk * 8;
    const bool x_ok = x0 < (which ? J : I);          // I and J are multiples of 8: a block column is in or out
    const uint16_t* gp = src + (int64_t)(cblk * 8) * ld + x0;
    uint4 r[8];
    auto gload = [&](int c0) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const bool ok = x_ok && c0 + cblk * 8 + j < C;
            r[j] = ok ? *reinterpret_cast<const uint4*>(gp + (int64_t)(c0 + j) * ld) : make_uint4(0, 0, 0, 0);
        }
    };
    // transposed block -> LDS: element e of the block's columns becomes operand row xblk*8 + e,
    // its 8 contraction elements the 16-byte chunk cblk of that row
    int st_off[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int p = bt_phys_row(xblk * 8 + e);
        st_off[e] = which * (BI * ROWB) + p * ROWB + ((cblk ^ ((p >> 1) & 7)) << 4);
    }
    auto lstore = [&](int stage) {
        uint8_t* base = smem + stage * STAGE;
        const uint32_t w[8][4] = {{r[0].x, r[0].y, r[0].z, r[0].w}, {r[1].x, r[1].y, r[1].z, r[1].w},
                                  {r[2].x, r[2].y, r[2].z, r[2].w}, {r[3].x, r[3].y, r[3].z, r[3].w},
                                  {r[4].x, r[4].y, r[4].z, r[4].w}, {r[5].x, r[5].y, r[5].z, r[5].w},
                                  {r[6].x, r[6].y, r[6].z, r[6].w}, {r[7].x, r[7].y, r[7].z, r[7].w}};
#pragma unroll
        for (int q = 0; q < 4; ++q) {       // dword q of the loaded rows holds columns 2q, 2q+1
            uint32_t lo[4], hi[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) {   // rows 2p, 2p+1
                lo[p] = __builtin_amdgcn_perm(w[2 * p + 1][q], w[2 * p][q], 0x05040100u);
                hi[p] = __builtin_amdgcn_perm(w[2 * p + 1][q], w[2 * p][q], 0x07060302u);
            }
            *reinterpret_cast<uint4*>(base + st_off[2 * q]) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
            *reinterpret_cast<uint4*>(base + st_off[2 * q + 1]) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
        }
    };

    // ---- LDS -> MFMA operands: lane (l % 16, g = l / 16) reads chunk g (first 32 contraction
    //      elements) and chunk g + 4 (the other 32) of operand row l % 16 of a fragment
    const int li = lane & 15, g = lane >> 4;
    int offa[FI], offb[FJ];
#pragma unroll
    for (int f = 0; f < FI; ++f) {
        const int p = bt_phys_row(wi0 + 16 * f + li);
        offa[f] = p * ROWB + ((g ^ ((p >> 1) & 7)) << 4);
    }
#pragma unroll
    for (int f = 0; f < FJ; ++f) {
        const int p = bt_phys_row(wj0 + 16 * f + li);
        offb[f] = BI * ROWB + p * ROWB + ((g ^ ((p >> 1) & 7)) << 4);
    }

    v4f_b acc[FI][FJ];
#pragma unroll
    for (int a = 0; a < FI; ++a)
#pragma unroll
        for (int b = 0; b < FJ; ++b) acc[a][b] = v4f_b{0.f, 0.f, 0.f, 0.f};

    auto compute = [&](int stage) {
        const uint8_t* base = smem + stage * STAGE;
#pragma unroll
        for (int s = 0; s < 2; ++s) {       // chunk g + 4 s sits at position (g ^ key) ^ 4
            v8bf_t bf[FJ];
#pragma unroll
            for (int f = 0; f < FJ; ++f) bf[f] = *reinterpret_cast<const v8bf_t*>(base + (offb[f] ^ (s << 6)));
#pragma unroll
            for (int a = 0; a < FI; ++a) {
                const v8bf_t af = *reinterpret_cast<const v8bf_t*>(base + (offa[a] ^ (s << 6)));
#pragma unroll
                for (int b = 0; b < FJ; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bf[b], af, acc[a][b], 0, 0, 0);
            }
        }
    };

    // ---- main loop, two LDS stages
    const int csteps = (C + BC - 1) / BC;
    if (csteps > 0) {
        gload(0);
        lstore(0);
        __syncthreads();
        for (int ct = 0; ct < csteps; ++ct) {
            const bool more = ct + 1 < csteps;
            if (more) gload((ct + 1) * BC);
            compute(ct & 1);
            if (more) lstore((ct + 1) & 1);
            __syncthreads();
        }
    }

    // ---- epilogue: lane holds out[i0 + wi0 + 16 a + l % 16][j0 + wj0 + 16 b + 4 g + r], r = 0..3
#pragma unroll
    for (int a = 0; a < FI; ++a) {
        const int i = i0 + wi0 + 16 * a + li;
        if (i >= I) continue;
        uint16_t* orow = out + (int64_t)i * ld_out;
#pragma unroll
        for (int b = 0; b < FJ; ++b) {
            const int j = j0 + wj0 + 16 * b + 4 * g;
            if (j >= J) continue;          // J is a multiple of 8: the 4 columns are in or out together
            *reinterpret_cast<uint2*>(orow + j) =
                make_uint2(bt_pack_bf16(acc[a][b][0], acc[a][b][1]), bt_pack_bf16(acc[a][b][2], acc[a][b][3]));
        }
    }
}

// out[I, J] = a[C, I]^T b[C, J]; I, J multiples of 8, lda / ldb / ld_out multiples of 8 elements,
// 16-byte aligned pointers (checked by the caller)
hipError_t launch_gemm_bf16_at_b(const void* a, int64_t lda, const void* b, int64_t ldb, int64_t I, int64_t J, int64_t C,
                                 void* out, int64_t ld_out, hipStream_t st) {
    using namespace bt;
    if (I == 0 || J == 0) return hipSuccess;
    {
        // more than 64 tiles: the LDS-DMA kernel (FP8MI355_BF16_VARIANT=0 / 1 forces one of the two)
        const int64_t tiles = ((I + BI - 1) / BI) * ((J + BJ - 1) / BJ);
        const int forced = knob(KNOB_BF16_VARIANT);
        const bool want = forced >= 0 ? forced != 0 : tiles > 64;
        if (want && gemm_bf16_at_b_snake_fits(lda, ldb, I, J, C))
            return launch_gemm_bf16_at_b_snake(a, lda, b, ldb, I, J, C, out, ld_out, st);
    }
    constexpr int lds = 2 * STAGE;
    static DynamicLdsOnce attr;
    if (hipError_t e = attr.ensure(reinterpret_cast<const void*>(gemm_bf16_at_b_kernel), lds); e != hipSuccess) return e;
    const int tiles_i = (int)((I + BI - 1) / BI), tiles_j = (int)((J + BJ - 1) / BJ);
    const int64_t ntiles = (int64_t)tiles_i * tiles_j;
    const int64_t grid = (ntiles + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
    if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
    gemm_bf16_at_b_kernel<<<dim3((unsigned)grid), dim3(NT), lds, st>>>(
        static_cast<const uint16_t*>(a), lda, static_cast<const uint16_t*>(b), ldb, (int)I, (int)J, (int)C,
        static_cast<uint16_t*>(out), ld_out, tiles_i, tiles_j);
    return hipGetLastError();
}

}  // namespace fp8k
