// Linear layer for a few tokens against a weight quantized once, in ONE launch:
//     y[M, N] = (q(X)[M, K] . Wq[N, K]^T) / (s_x * s_w),   q(X) = fp8(X * s_x),  s_x = FMAX / amax(X)
// (Section 3 of the paper: dynamic activation quantization in front of a
// pre-quantized weight, at decode batch sizes).  The two-launch form quantizes X
// in a kernel of its own; at these sizes that launch costs as much as streaming
// a third of the weight.  Here every workgroup quantizes X itself, into LDS.
//
// The product is the LDS-DMA few-row kernel of gemm_fp8_skinny.hip: a wavefront owns NW column
// tiles of 16 weight rows and a part of K; the weight streams through a private ring of LDS slots,
// R steps of 128 bytes ahead, no barriers in the main loop.  What differs:
//  * a workgroup is eight wavefronts (one per CU: X is read and converted once per CU) where that makes one
//    round of workgroups over most CUs, else four (two per CU);
//  * before the main loop the workgroup reads all of X (at most 32768 elements: 8 or 16 loads of 16 bytes
//    per lane, requested ahead of the first ring fill and waited for by count, so they arrive while the
//    weight's first bytes are still on their way), reduces the row maxima (lane maxima folded within rows
//    of 16 lanes by DPP rotations, then through scalar registers, then one LDS word per row), derives the
//    scales with the row quantizer's arithmetic, converts the registers it still holds and leaves the
//    codes in LDS, one padded row per token;
//  * in the main loop the A operand is two 16-byte LDS reads from those codes (lanes of rows past M read
//    zeros); nothing of X is fetched again.
// Same codes, scales and order of sums as the two-launch form: the results are bit-identical.
#include "fp8_device.hpp"
#include "launchers.hpp"
#include "tuning.hpp"

namespace fp8k {

typedef int v8i_q __attribute__((ext_vector_type(8)));
typedef int v4i_q __attribute__((ext_vector_type(4)));
typedef float v4f_q __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_q __attribute__((ext_vector_type(2)));
typedef float f32x2_q __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t skf_pack_bf16(float a, float b) {
    f32x2_q v = {a, b};
    bf16x2_q h = __builtin_convertvector(v, bf16x2_q);
    uint32_t r;
    __builtin_memcpy(&r, &h, 4);
    return r;
}

// 16 bytes per lane from a raw buffer into LDS at lds_addr + lane * 16 (the wavefront's own LDS reads of
// the slot were issued before, in program order, and are waited for here)
__device__ __forceinline__ void skf_lds_dma16(v4i_q rsrc, uint32_t lds_addr, uint32_t voffset) {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voffset), "s"(rsrc)
                 : "memory", "m0");
}
// 16 bytes per lane from a raw buffer into registers; the data is there after skf_wait_x.  Assembly, like
// the wait: the compiler's own count of loads in flight knows nothing of the LDS-DMA loads issued behind these.
__device__ __forceinline__ void skf_load16(v4i_q& dst, v4i_q rsrc, uint32_t voffset) {
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(dst) : "v"(voffset), "s"(rsrc) : "memory");
}
// wait until at most N_ loads are in flight; the registers are operands so that no use of them moves above the wait
template <int N_, int U>
__device__ __forceinline__ void skf_wait_x(v4i_q (&x)[U]) {
    static_assert(U == 8 || U == 16, "8 or 16 register sets");
    if constexpr (U == 8) {
        asm volatile("s_waitcnt vmcnt(%8)"
                     : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7])
                     : "n"(N_)
                     : "memory");
    } else {
        asm volatile("s_waitcnt vmcnt(%16)"
                     : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]),
                       "+v"(x[8]), "+v"(x[9]), "+v"(x[10]), "+v"(x[11]), "+v"(x[12]), "+v"(x[13]), "+v"(x[14]), "+v"(x[15])
                     : "n"(N_)
                     : "memory");
    }
}
template <int N_>
__device__ __forceinline__ void skf_wait_vmem() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N_) : "memory"); }

namespace skf {
constexpr int MAX_X = 32768;       // elements of X a workgroup holds in registers: 8 (16) loads of 8 per lane of its 512 (256) threads
constexpr int ROW_PAD = 64;        // bytes between the rows of codes in LDS beyond K: consecutive rows start 16 banks apart
}  // namespace skf

template <int FX, int FB, int KS, int NW, int WAVES, int R>
__global__ __launch_bounds__(64 * WAVES) void gemm_fp8_skinny_fused_kernel(
    const uint16_t* __restrict__ X, int64_t ldx, int row_x, int flags, const uint8_t* __restrict__ B, int64_t ldb,
    const float* __restrict__ scale_b, int row_b, int M, int N, int K, uint16_t* __restrict__ out, int64_t ld_out) {
    using namespace skf;
    constexpr int NTW = WAVES / KS;
    constexpr int SLOT = NW * 2048;              // weight bytes of one K step of this wavefront
    constexpr int LB = 2 * NW;                   // LDS-DMA loads per step
    static_assert((R - 1) * LB <= 63 && R * LB <= 63, "vmcnt range");
    // dynamic LDS: WAVES rings of R slots; then the codes of X, row r at r * (K + ROW_PAD); then 128 bytes of zeros
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    __shared__ uint32_t amax_bits[8];
    __shared__ float scale_x[8];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 15, g = lane >> 4;
    const int n0 = (blockIdx.x * NTW + wave / KS) * (16 * NW);
    const int kp = wave % KS;
    const int ksteps = K / 128;                  // K is a multiple of 512
    const int per = (ksteps + KS - 1) / KS;
    const int s_begin = kp * per;
    const int s_end = s_begin + per < ksteps ? s_begin + per : ksteps;
    uint8_t* codes = smem + WAVES * R * SLOT;
    const int row_bytes = K + ROW_PAD;
    uint8_t* zeros = codes + M * row_bytes;

    if (tid < 8) amax_bits[tid] = 0;
    if (tid < 8) *reinterpret_cast<uint4*>(zeros + tid * 16) = make_uint4(0, 0, 0, 0);

    float sc_b[NW][4];
#pragma unroll
    for (int w = 0; w < NW; ++w)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int n = n0 + 16 * w + 4 * g + r;
            sc_b[w][r] = scale_b[row_b ? (n < N ? n : N - 1) : 0];
        }

    // buffer descriptors: this wavefront's rows of the weight (zeros past N), all of X
    const int rows_b = n0 < N ? (N - n0 < 16 * NW ? N - n0 : 16 * NW) : 0;
    const uint64_t pb = reinterpret_cast<uint64_t>(B + (int64_t)(n0 < N ? n0 : 0) * ldb);
    const uint64_t px = reinterpret_cast<uint64_t>(X);
    const v4i_q rsrc_b = {(int)(uint32_t)pb, (int)(uint32_t)(pb >> 32), rows_b > 0 ? (int)((int64_t)(rows_b - 1) * ldb + K) : 0, 0x00020000};
    const v4i_q rsrc_x = {(int)(uint32_t)px, (int)(uint32_t)(px >> 32), (int)(((int64_t)(M - 1) * ldx + K) * 2), 0x00020000};
    constexpr uint32_t OOB = 0x80000000u;

    // ---- X: wavefront w takes the pieces w, w + 8, ... of 512 elements (piece q = 512 elements from column
    //      512 (q % cpr) of row q / cpr); a piece past the end is not fetched (zeros)
    constexpr int U = 64 / WAVES;                // pieces per wavefront: 8 or 16 loads of 16 bytes per lane
    const int cpr = K / 512, pieces = M * cpr;
    v4i_q xv[U];
    int prow[U], pcol[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int q = wave + WAVES * u;
        prow[u] = q / cpr;
        pcol[u] = q - prow[u] * cpr;
        skf_load16(xv[u], rsrc_x, q < pieces ? (uint32_t)((prow[u] * (int)ldx + pcol[u] * 512 + lane * 8) * 2) : OOB);
    }

    // ---- weight: load j of a 16-row tile fetches rows 8 j + lane / 8; lane's chunk slot lane % 8 receives chunk slot ^ key(row)
    const int lrow = lane >> 3;
    const int c0 = (lane & 7) ^ ((lrow >> 1) & 7);
    const int c1 = (lane & 7) ^ ((4 + (lrow >> 1)) & 7);
    const uint32_t vb0 = (uint32_t)(lrow * (int)ldb + c0 * 16), vb1 = (uint32_t)((8 + lrow) * (int)ldb + c1 * 16);
    const uint32_t ring = (uint32_t)(size_t)smem + (uint32_t)wave * (uint32_t)(R * SLOT);
    auto issue_b = [&](int slot, int s) {        // K step s into ring slot `slot` (out of range, i.e. no access, past s_end)
        const uint32_t k0 = s < s_end ? (uint32_t)(s * 128) : OOB;
        const uint32_t dst = ring + (uint32_t)(slot * SLOT);
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            skf_lds_dma16(rsrc_b, dst + w * 2048, vb0 + (uint32_t)(16 * w * (int)ldb) + k0);
            skf_lds_dma16(rsrc_b, dst + w * 2048 + 1024, vb1 + (uint32_t)(16 * w * (int)ldb) + k0);
        }
    };
#pragma unroll
    for (int r = 0; r < R; ++r) issue_b(r, s_begin + r);

    // ---- amax per row, scales, codes into LDS
    __syncthreads();                              // amax_bits and zeros are set
    skf_wait_x<R * LB, U>(xv);                       // X is there; the first ring fill may still be under way
    auto as_u4 = [](const v4i_q& a) { return make_uint4((uint32_t)a[0], (uint32_t)a[1], (uint32_t)a[2], (uint32_t)a[3]); };
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (wave + WAVES * u < pieces) {
            const uint32_t m = wave_max_u32<64>(pk_fold(pk_absmax4(0u, as_u4(xv[u]))));
            if (lane == 0) atomicMax(&amax_bits[prow[u]], m);
        }
    }
    __syncthreads();
    if (tid < M) {
        uint32_t mag = amax_bits[tid];
        if (!row_x)
            for (int m = 0; m < M; ++m) mag = amax_bits[m] > mag ? amax_bits[m] : mag;
        scale_x[tid] = scale_from_amax(mag_to_float(mag), FX, flags);
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (wave + WAVES * u < pieces)
            *reinterpret_cast<uint2*>(codes + prow[u] * row_bytes + pcol[u] * 512 + lane * 8) = cast8<FX>(as_u4(xv[u]), scale_x[prow[u]]);
    }
    __syncthreads();

    v4f_q acc[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) acc[w] = v4f_q{0.f, 0.f, 0.f, 0.f};

    // weight fragment: chunks g and g + 4 of row i of a tile; A fragment: the same chunks of row i of the codes
    const int key = (i >> 1) & 7;
    const int f_lo = i * 128 + ((g ^ key) << 4), f_hi = i * 128 + (((g + 4) ^ key) << 4);
    auto frag = [&](const uint8_t* tile) {
        const uint4 lo = *reinterpret_cast<const uint4*>(tile + f_lo);
        const uint4 hi = *reinterpret_cast<const uint4*>(tile + f_hi);
        return v8i_q{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
    };
    const uint8_t* a_row = i < M ? codes + i * row_bytes + 16 * g : zeros + 16 * g;
    const int a_step = i < M ? 128 : 0;

    int slot = 0;
    for (int s = s_begin; s < s_end; ++s) {
        skf_wait_vmem<(R - 1) * LB>();            // all but the R - 1 younger slots have landed
        const uint8_t* base = smem + wave * (R * SLOT) + slot * SLOT;
        v8i_q bf[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) bf[w] = frag(base + w * 2048);
        const uint8_t* ap = a_row + s * a_step;
        const uint4 lo = *reinterpret_cast<const uint4*>(ap), hi = *reinterpret_cast<const uint4*>(ap + 64);
        const v8i_q af = {(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
#pragma unroll
        for (int w = 0; w < NW; ++w)
            acc[w] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bf[w], af, acc[w], FB, FX, 0, 0, 0, 0);
        issue_b(slot, s + R);
        slot = slot + 1 == R ? 0 : slot + 1;
    }
    skf_wait_vmem<0>();       // trailing (out-of-range) refills must land before the LDS is reused or handed back

    // ---- sum the K parts of a column group through LDS (the rings are free now)
    if constexpr (KS > 1) {
        __syncthreads();
        v4f_q* part = reinterpret_cast<v4f_q*>(smem);      // [NTW][KS - 1][NW][64]
        const int grp = wave / KS;
        if (kp > 0) {
#pragma unroll
            for (int w = 0; w < NW; ++w) part[((grp * (KS - 1) + kp - 1) * NW + w) * 64 + lane] = acc[w];
        }
        __syncthreads();
        if (kp > 0) return;
#pragma unroll
        for (int p = 0; p < KS - 1; ++p)
#pragma unroll
            for (int w = 0; w < NW; ++w) acc[w] += part[((grp * (KS - 1) + p) * NW + w) * 64 + lane];
    }

    // ---- epilogue: lane holds y[i][n0 + 16 w + 4 g + r], r = 0..3
    if (i >= M) return;
    const float inv_a = 1.0f / scale_x[i];
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const int nb = n0 + 16 * w + 4 * g;
        if (nb >= N) continue;
        float v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = (acc[w][r] * inv_a) * (1.0f / sc_b[w][r]);
        uint16_t* dst = out + (int64_t)i * ld_out + nb;
        const uint32_t p0 = skf_pack_bf16(v[0], v[1]), p1 = skf_pack_bf16(v[2], v[3]);
        if (nb + 4 <= N) {
            *reinterpret_cast<uint2*>(dst) = make_uint2(p0, p1);
        } else {
            const uint32_t w2[2] = {p0, p1};
            for (int r = 0; nb + r < N; ++r) dst[r] = (uint16_t)(w2[r >> 1] >> ((r & 1) * 16));
        }
    }
}

template <int FX, int FB, int KS, int NW, int WAVES>
static hipError_t launch_skf(const uint16_t* x, int64_t ldx, int row_x, int flags, const uint8_t* b, int64_t ldb,
                             const float* sb, int row_b, int M, int N, int K, uint16_t* out, int64_t ld_out, int64_t grid,
                             hipStream_t st) {
    using namespace skf;
    // eight wavefronts: 96 KB of rings, one workgroup per CU with the codes of X (33 KB at most); four: 40 or 48 KB
    constexpr int R = WAVES == 8 ? (NW == 1 ? 6 : 3) : (NW == 1 ? 5 : 3);
    const int lds = WAVES * R * NW * 2048 + M * (K + ROW_PAD) + 128;
    auto kern = gemm_fp8_skinny_fused_kernel<FX, FB, KS, NW, WAVES, R>;
    static DynamicLdsOnce attr;
    if (hipError_t e = attr.ensure(reinterpret_cast<const void*>(kern), WAVES * R * NW * 2048 + MAX_X + 8 * ROW_PAD + 128); e != hipSuccess) return e;
    kern<<<dim3((unsigned)grid), dim3(64 * WAVES), lds, st>>>(x, ldx, row_x, flags, b, ldb, sb, row_b, M, N, K, out, ld_out);
    return hipGetLastError();
}

// hipErrorNotSupported (nothing launched) where the one-launch form does not apply (more than 8 tokens or more
// than 32768 activations - what a workgroup holds in registers between the amax and the conversion -, activations
// to e5m2, K not a multiple of 512, operands beyond the reach of 32-bit buffer offsets) or does not pay: every
// workgroup reads and converts all of X before its first product, 16 to 128 elements per lane, and that time
// grows with M while the launch it saves (2-3 us) does not.  Measured against the two-launch form on the
// Llama-3 projections, calls replayed from a graph: one token 13-21 % faster on the 8B shapes (2-4 % on the
// 70B ones), two tokens 4-16 %, four tokens 0-9 %, eight tokens 3 % faster on the 14336 x 4096 weight and
// 12-13 % slower on the 4096 x 4096 and 6144 x 4096 ones.  Default therefore: one token, or up to four with
// M * K <= 16384.  The switch DECODE_FUSED: 0 = never, 2 = wherever the kernel applies.
hipError_t launch_linear_skinny_fused(const void* x, int64_t ldx, int fmt_x, int row_x, int flags, const uint8_t* b,
                                      int64_t ldb, int fmt_b, const float* scale_b, int row_b, int64_t M, int64_t N,
                                      int64_t K, void* out, int64_t ld_out, hipStream_t st) {
    using namespace skf;
    const int mode = knob(KNOB_DECODE_FUSED);
    if (mode == 0 || M < 1 || M > 8 || N < 1 || K < 512 || K % 512 != 0 || M * K > MAX_X) return hipErrorNotSupported;
    if (mode != 2 && M != 1 && (M > 4 || M * K > 16384)) return hipErrorNotSupported;
    if (fmt_x != FMT_E4M3FN) return hipErrorNotSupported;
    if (ldb >= (1 << 23) || ((M - 1) * ldx + K) * 2 >= (int64_t)1 << 31 || (int64_t)16 * 4 * ldb + K >= (int64_t)1 << 31)
        return hipErrorNotSupported;
    int nw = N >= 6144 ? 2 : 1;
    if (const int v = knob(KNOB_SKINNY_NW); v == 1 || v == 2) nw = v;
    const int64_t groups = (N + 16 * nw - 1) / (16 * nw);
    int ks = 1;
    while (ks < 4 && groups * ks < 2048 && K / (ks * 2) >= 512) ks *= 2;
    // eight wavefronts per workgroup where that makes one round of workgroups over at least three quarters of the CUs;
    // fewer would leave CUs idle, and with more than one round a CU streams nothing while its only workgroup
    // quantizes X and waits for its first ring fill (two workgroups of four wavefronts cover for each other)
    const int cus = compute_units() > 0 ? compute_units() : 256;
    const int64_t grid8 = (groups * ks + 7) / 8;
    const int waves = grid8 * 4 >= (int64_t)cus * 3 && grid8 <= cus ? 8 : 4;
    const int ntw = waves / ks;
    const int64_t grid = (groups + ntw - 1) / ntw;
    if (grid > 0x7FFFFFFF) return hipErrorNotSupported;
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    uint16_t* op = static_cast<uint16_t*>(out);
    const int m = (int)M, n = (int)N, k = (int)K;
#define FP8K_SKF(FB_, KS_, NW_, W_)                                  \
    if (fmt_b == FB_ && ks == KS_ && nw == NW_ && waves == W_)       \
        return launch_skf<FMT_E4M3FN, FB_, KS_, NW_, W_>(xp, ldx, row_x, flags, b, ldb, scale_b, row_b, m, n, k, op, ld_out, grid, st)
#define FP8K_SKF6(FB_, W_) \
    FP8K_SKF(FB_, 1, 1, W_); FP8K_SKF(FB_, 2, 1, W_); FP8K_SKF(FB_, 4, 1, W_); FP8K_SKF(FB_, 1, 2, W_); FP8K_SKF(FB_, 2, 2, W_); FP8K_SKF(FB_, 4, 2, W_)
    FP8K_SKF6(FMT_E4M3FN, 8);
    FP8K_SKF6(FMT_E4M3FN, 4);
    FP8K_SKF6(FMT_E5M2, 8);
    FP8K_SKF6(FMT_E5M2, 4);
#undef FP8K_SKF6
#undef FP8K_SKF
    return hipErrorNotSupported;
}

}  // namespace fp8k
