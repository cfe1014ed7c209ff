// Linear layer for up to 8 tokens against a weight quantized once, in ONE launch:
//     y[M, N] = (q(X)[M, K] . Wq[N, K]^T) / (s_x * s_w),   q(X) = fp8(X * s_x),  s_x = FMAX / amax(X)
// (Section 3 of the paper: dynamic activation quantization in front of a
// pre-quantized weight, at decode batch sizes).  The two-launch form quantizes X
// in a kernel of its own; at these sizes that launch costs as much as streaming
// a third of the weight.  Here every workgroup derives the scales of X itself
// and converts the bfloat16 activations to fp8 on their way into the matrix cores.
//
// The product is the LDS-DMA few-row kernel of gemm_fp8_skinny.hip: a wavefront owns NW column
// tiles of 16 weight rows and a part of K; the weight streams through a private ring of LDS slots,
// R steps of 128 bytes ahead.  What differs:
//  * the amax of X: all wavefronts of the workgroup read X once (M * K bfloat16, from L2 after the
//    first workgroups), 512 elements per wavefront and load, and fold the maxima into one LDS word per row;
//    the loads are issued behind the first ring fill, so they travel while the weight's first bytes do;
//  * the A operand: per K step the wavefront loads the M x 128 activations of the step densely (lane l the
//    elements 2 l and 2 l + 1 of every row: MB dwords, R steps ahead like the ring), converts them when the
//    step is due (multiply by s_x, clamp, round to nearest even: the arithmetic of the row quantizer, so
//    the codes are the ones it would have written), parks the codes in a 16 x 128 byte LDS tile of its own
//    and reads its MFMA operand from there.  Converting in the operand's own layout would have every lane
//    convert 32 elements of some row, present or not: as many conversions as the weight has bytes.
// Register loads and LDS-DMA loads complete in the order of issue; a step issues first its ring loads, then its
// A loads, so "step s is there" is one wait on the number of younger loads.  The A loads are assembly for that
// reason: the compiler's own bookkeeping of loads in flight knows nothing of the LDS-DMA loads between them.
#include "fp8_device.hpp"
#include "launchers.hpp"
#include "tuning.hpp"

namespace fp8k {

typedef int v8i_q __attribute__((ext_vector_type(8)));
typedef int v4i_q __attribute__((ext_vector_type(4)));
typedef float v4f_q __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_q __attribute__((ext_vector_type(2)));
typedef float f32x2_q __attribute__((ext_vector_type(2)));
typedef uint16_t __attribute__((may_alias)) u16_any;      // the codes of X are written as halfwords and read back as 16-byte operands

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
// one dword per lane from a raw buffer into a register; the data is there after skf_wait
__device__ __forceinline__ void skf_load4(int& dst, v4i_q rsrc, uint32_t voffset) {
    asm volatile("buffer_load_dword %0, %1, %2, 0 offen" : "=v"(dst) : "v"(voffset), "s"(rsrc) : "memory");
}
// wait until at most N_ loads are in flight; the registers are operands so that no use of them moves above the wait
template <int N_, int MB>
__device__ __forceinline__ void skf_wait(int (&a)[MB]) {
    if constexpr (MB == 1) asm volatile("s_waitcnt vmcnt(%1)" : "+v"(a[0]) : "n"(N_) : "memory");
    if constexpr (MB == 2) asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a[0]), "+v"(a[1]) : "n"(N_) : "memory");
    if constexpr (MB == 4)
        asm volatile("s_waitcnt vmcnt(%4)" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]) : "n"(N_) : "memory");
    if constexpr (MB == 8)
        asm volatile("s_waitcnt vmcnt(%8)"
                     : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7])
                     : "n"(N_)
                     : "memory");
}
__device__ __forceinline__ void skf_wait_all() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// MB: rows of X the kernel is built for (M <= MB; 1, 2, 4 or 8)
template <int FX, int FB, int KS, int NW, int MB, int R>
__global__ __launch_bounds__(256) void gemm_fp8_skinny_fused_kernel(
    const uint16_t* __restrict__ X, int64_t ldx, int row_x, int flags, const uint8_t* __restrict__ B, int64_t ldb,
    const float* __restrict__ scale_b, int row_b, int M, int N, int K, uint16_t* __restrict__ out, int64_t ld_out) {
    constexpr int NTW = 4 / KS;
    constexpr int SLOT = NW * 2048;              // weight bytes of one K step of this wavefront
    constexpr int LB = 2 * NW, LA = MB;          // loads per step: LDS-DMA (weight), registers (activations)
    static_assert((R - 1) * (LB + LA) <= 63, "vmcnt range");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];     // 4 rings of R slots, then 4 tiles of 16 x 128 codes of X
    __shared__ uint32_t amax_bits[8];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 15, g = lane >> 4;
    const int n0 = (blockIdx.x * NTW + wave / KS) * (16 * NW);
    const int kp = wave % KS;
    const int ksteps = K / 128;                  // K is a multiple of 512
    const int per = (ksteps + KS - 1) / KS;
    const int s_begin = kp * per;
    const int s_end = s_begin + per < ksteps ? s_begin + per : ksteps;

    if (tid < 8) amax_bits[tid] = 0;
    // this wavefront's tile of codes: rows M..15 stay zero for good
    uint8_t* codes = smem + 4 * R * SLOT + wave * 2048;
    *reinterpret_cast<uint4*>(codes + lane * 32) = make_uint4(0, 0, 0, 0);
    *reinterpret_cast<uint4*>(codes + lane * 32 + 16) = make_uint4(0, 0, 0, 0);
    __syncthreads();

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

    // weight: load j of a 16-row tile fetches rows 8 j + lane / 8; lane's chunk slot lane % 8 receives chunk slot ^ key(row)
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
    // activations: lane l takes elements 2 l, 2 l + 1 of the step of every row (rows past M and steps past
    // the end point outside the buffer: no access, zeros - but the same number of loads every time)
    auto load_a = [&](int (&dst)[MB], int s) {
#pragma unroll
        for (int r = 0; r < MB; ++r)
            skf_load4(dst[r], rsrc_x, (r < M && s < ksteps) ? (uint32_t)((r * (int)ldx + s * 128 + 2 * lane) * 2) : OOB);
    };

    int araw[R][MB];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        issue_b(r, s_begin + r);
        load_a(araw[r], s_begin + r);
    }

    // ---- amax of every row of X: wavefront w takes pieces w, w + 4, ... of 512 elements
    {
        const int cpr = K / 512, pieces = M * cpr;
        constexpr int U = 16;
        for (int q0 = wave; q0 < pieces; q0 += 4 * U) {
            uint4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {       // all requested before the first is used (a piece past the end repeats the last one)
                const int q = q0 + 4 * u < pieces ? q0 + 4 * u : pieces - 1;
                v[u] = *reinterpret_cast<const uint4*>(X + (int64_t)(q / cpr) * ldx + (q % cpr) * 512 + lane * 8);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int q = q0 + 4 * u;
                if (q < pieces) {
                    const uint32_t m = wave_max_u32<64>(pk_fold(pk_absmax4(0u, v[u])));
                    if (lane == 0) atomicMax(&amax_bits[q / cpr], m);
                }
            }
        }
    }
    __syncthreads();
    float sx[MB];
    if (row_x) {
#pragma unroll
        for (int r = 0; r < MB; ++r) sx[r] = scale_from_amax(mag_to_float(amax_bits[r < M ? r : M - 1]), FX, flags);
    } else {
        uint32_t mag = 0;
        for (int m = 0; m < M; ++m) mag = amax_bits[m] > mag ? amax_bits[m] : mag;
        const float s1 = scale_from_amax(mag_to_float(mag), FX, flags);
#pragma unroll
        for (int r = 0; r < MB; ++r) sx[r] = s1;
    }

    v4f_q acc[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) acc[w] = v4f_q{0.f, 0.f, 0.f, 0.f};

    // weight fragment: chunks g and g + 4 of row i of a tile
    const int key = (i >> 1) & 7;
    const int f_lo = i * 128 + ((g ^ key) << 4), f_hi = i * 128 + (((g + 4) ^ key) << 4);
    auto frag = [&](const uint8_t* tile) {
        const uint4 lo = *reinterpret_cast<const uint4*>(tile + f_lo);
        const uint4 hi = *reinterpret_cast<const uint4*>(tile + f_hi);
        return v8i_q{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
    };
    // the same chunks of row i of the codes of X (plain layout)
    const uint8_t* a_lo = codes + i * 128 + 16 * g;

    for (int s0 = s_begin; s0 < s_end; s0 += R) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int s = s0 + r;
            if (s < s_end) {
                skf_wait<(R - 1) * (LB + LA), MB>(araw[r]);   // step s has landed
#pragma unroll
                for (int m = 0; m < MB; ++m) {
                    const uint32_t w2 = (uint32_t)araw[r][m];
                    *reinterpret_cast<u16_any*>(codes + m * 128 + 2 * lane) =
                        (uint16_t)cvt2<FX>(bf16_lo(w2) * sx[m], bf16_hi(w2) * sx[m]);
                }
                const uint8_t* base = smem + wave * (R * SLOT) + r * SLOT;
                v8i_q bf[NW];
#pragma unroll
                for (int w = 0; w < NW; ++w) bf[w] = frag(base + w * 2048);
                const uint4 lo = *reinterpret_cast<const uint4*>(a_lo), hi = *reinterpret_cast<const uint4*>(a_lo + 64);
                const v8i_q af = {(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
#pragma unroll
                for (int w = 0; w < NW; ++w)
                    acc[w] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bf[w], af, acc[w], FB, FX, 0, 0, 0, 0);
                issue_b(r, s + R);
                load_a(araw[r], s + R);
            }
        }
    }
    skf_wait_all();           // trailing loads must land before the registers die and the LDS is reused or handed back

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
    float sxi = sx[0];
#pragma unroll
    for (int r = 1; r < MB; ++r) sxi = i == r ? sx[r] : sxi;
    const float inv_a = 1.0f / sxi;
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

template <int FX, int FB, int KS, int NW, int MB>
static hipError_t launch_skf(const uint16_t* x, int64_t ldx, int row_x, int flags, const uint8_t* b, int64_t ldb,
                             const float* sb, int row_b, int M, int N, int K, uint16_t* out, int64_t ld_out, int64_t grid,
                             hipStream_t st) {
    constexpr int R = NW == 1 ? 6 : 4;      // 56 KB or 72 KB of LDS with the tiles of codes: two workgroups per CU
    constexpr int lds = 4 * R * NW * 2048 + 4 * 2048;
    auto kern = gemm_fp8_skinny_fused_kernel<FX, FB, KS, NW, MB, R>;
    static DynamicLdsOnce attr;
    if (hipError_t e = attr.ensure(reinterpret_cast<const void*>(kern), lds); e != hipSuccess) return e;
    kern<<<dim3((unsigned)grid), dim3(256), lds, st>>>(x, ldx, row_x, flags, b, ldb, sb, row_b, M, N, K, out, ld_out);
    return hipGetLastError();
}

// hipErrorNotSupported (nothing launched) where the one-launch form does not apply (more than 8 tokens,
// activations to e5m2, K not a multiple of 512, operands beyond the reach of 32-bit buffer offsets) or does not
// pay.  Every workgroup reads all of X for the amax and every wavefront its K part of X for the product, and all
// of them want the same lines at the same time: each further token costs 1-2 us on the Llama-3-8B projections
// (more on larger weights), where the launch that is saved costs 2-3 us.  Measured against the two-launch form,
// calls replayed from a graph: one token 6-17 % faster on the 8B shapes (1-6 % on the 70B ones), two tokens
// 2-11 % faster at K = 4096 and 6-10 % slower beyond, four tokens slower nearly everywhere.  Default
// therefore: one token, or M * K <= 8192.  The switch DECODE_FUSED: 0 = never, 2 = wherever the kernel applies.
hipError_t launch_linear_skinny_fused(const void* x, int64_t ldx, int fmt_x, int row_x, int flags, const uint8_t* b,
                                      int64_t ldb, int fmt_b, const float* scale_b, int row_b, int64_t M, int64_t N,
                                      int64_t K, void* out, int64_t ld_out, hipStream_t st) {
    const int mode = knob(KNOB_DECODE_FUSED);
    if (mode == 0 || M < 1 || M > 8 || N < 1 || K < 512 || K % 512 != 0) return hipErrorNotSupported;
    if (mode != 2 && M != 1 && M * K > 8192) return hipErrorNotSupported;
    if (fmt_x != FMT_E4M3FN) return hipErrorNotSupported;
    if (ldb >= (1 << 23) || ((M - 1) * ldx + K) * 2 >= (int64_t)1 << 31 || (int64_t)16 * 4 * ldb + K >= (int64_t)1 << 31)
        return hipErrorNotSupported;
    int nw = N >= 6144 ? 2 : 1;
    if (const int v = knob(KNOB_SKINNY_NW); v == 1 || v == 2) nw = v;
    const int64_t groups = (N + 16 * nw - 1) / (16 * nw);
    int ks = 1;
    while (ks < 4 && groups * ks < 2048 && K / (ks * 2) >= 512) ks *= 2;
    const int64_t grid = (groups + (4 / ks) - 1) / (4 / ks);
    if (grid > 0x7FFFFFFF) return hipErrorNotSupported;
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    uint16_t* op = static_cast<uint16_t*>(out);
    const int m = (int)M, n = (int)N, k = (int)K;
    const int mb = m == 1 ? 1 : (m == 2 ? 2 : (m <= 4 ? 4 : 8));
#define FP8K_SKF(FB_, KS_, NW_, MB_)                                  \
    if (fmt_b == FB_ && ks == KS_ && nw == NW_ && mb == MB_)          \
        return launch_skf<FMT_E4M3FN, FB_, KS_, NW_, MB_>(xp, ldx, row_x, flags, b, ldb, scale_b, row_b, m, n, k, op, ld_out, grid, st)
#define FP8K_SKF4(FB_, KS_, NW_) \
    FP8K_SKF(FB_, KS_, NW_, 1); FP8K_SKF(FB_, KS_, NW_, 2); FP8K_SKF(FB_, KS_, NW_, 4); FP8K_SKF(FB_, KS_, NW_, 8)
#define FP8K_SKF6(FB_) \
    FP8K_SKF4(FB_, 1, 1); FP8K_SKF4(FB_, 2, 1); FP8K_SKF4(FB_, 4, 1); FP8K_SKF4(FB_, 1, 2); FP8K_SKF4(FB_, 2, 2); FP8K_SKF4(FB_, 4, 2)
    FP8K_SKF6(FMT_E4M3FN);
    FP8K_SKF6(FMT_E5M2);
#undef FP8K_SKF6
#undef FP8K_SKF4
#undef FP8K_SKF
    return hipErrorNotSupported;
}

}  // namespace fp8k
