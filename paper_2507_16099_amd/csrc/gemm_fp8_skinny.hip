// Scaled FP8 GEMM for few rows of A (M <= 64): out[M,N] = (A[M,K] . B[N,K]^T) / (sa * sb).
// This is the shape of inference with pre-quantized weights (Section 3 of the
// paper: dynamic activation + weight FP8 quantization) at decode batch sizes:
// B (the weight) is read once and the kernel is bound by that HBM stream, N*K
// bytes, not by the matrix cores.
//
// Two forms.  The first (below) is used for 33..64 rows and for leading
// dimensions beyond the reach of 32-bit buffer offsets; the second, further
// down, brings the operands in by LDS-DMA and is 10-25 % faster on the
// large weight shapes (4.2-5.7 TB/s of weight bytes against 3.6-5.0).
//
// First form: no LDS staging and no barriers in the main loop.  A wavefront owns 16 rows
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
#include "tuning.hpp"


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

// ---------------------------------------------------------------------------------
// The same product with the operands brought in by LDS-DMA (buffer_load ... lds).
// The loads of the kernel above touch 16 rows x 64 bytes per instruction and are
// limited by the address path of the L1 cache; here an instruction fetches 8 rows
// x 128 bytes (whole lines) straight into LDS, and the MFMA operands are read from
// there with the conflict-free swizzle of the tiled kernels (chunk c of row r sits
// at position c ^ ((r >> 1) & 7); lane (l % 16, g) reads chunks g and g + 4).
// Every wavefront still works alone: it owns NW column tiles and a part of K, and
// a private ring of R LDS slots (one K step each: NW + MT tiles of 2 KB); the ring
// is refilled R steps ahead, and "step s has landed" is a wait on the number of
// younger loads (they complete in order).  No barriers in the main loop.
typedef int v4i_k __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void sk_lds_dma16(v4i_k rsrc, uint32_t lds_addr, uint32_t voffset) {
    // LDS reads of this wavefront that still use the slot have been issued before (program order)
    // and are waited for here, so the refill cannot overtake them
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voffset), "s"(rsrc)
                 : "memory", "m0");
}
template <int N_>
__device__ __forceinline__ void sk_wait_vmem() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N_) : "memory"); }

template <int FA, int FB, int MT, int KS, int NW, int R>
__global__ __launch_bounds__(256) void gemm_fp8_skinny_dma_kernel(
    const uint8_t* __restrict__ A, int64_t lda, const uint8_t* __restrict__ B, int64_t ldb,
    const float* __restrict__ scale_a, int row_a, const float* __restrict__ scale_b, int row_b, int M, int N,
    int K, void* __restrict__ out, int64_t ld_out, int out_f32) {
    constexpr int NTW = 4 / KS;
    constexpr int SLOT = (NW + MT) * 2048;       // bytes of one K step of this wavefront
    constexpr int LOADS = 2 * (NW + MT);         // LDS-DMA instructions per slot
    static_assert((R - 1) * LOADS <= 63, "vmcnt range");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 15, g = lane >> 4;
    const int n0 = (blockIdx.x * NTW + wave / KS) * (16 * NW);
    const int kp = wave % KS;
    const int ksteps = (K + 127) / 128;
    const int per = (ksteps + KS - 1) / KS;
    const int s_begin = kp * per;
    const int s_end = s_begin + per < ksteps ? s_begin + per : ksteps;

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

    // buffer descriptors: this wavefront's rows of B (zeros past N), all of A (zeros past M)
    const int rows_b = n0 < N ? (N - n0 < 16 * NW ? N - n0 : 16 * NW) : 0;
    const uint64_t pb = reinterpret_cast<uint64_t>(B + (int64_t)(n0 < N ? n0 : 0) * ldb);
    const uint64_t pa = reinterpret_cast<uint64_t>(A);
    const v4i_k rsrc_b = {(int)(uint32_t)pb, (int)(uint32_t)(pb >> 32), rows_b > 0 ? (int)((int64_t)(rows_b - 1) * ldb + K) : 0, 0x00020000};
    const v4i_k rsrc_a = {(int)(uint32_t)pa, (int)(uint32_t)(pa >> 32), (int)((int64_t)(M - 1) * lda + K), 0x00020000};
    constexpr uint32_t OOB = 0x80000000u;

    // load j of a 16-row tile fetches rows 8 j + lane / 8; lane's chunk slot lane % 8 receives chunk slot ^ key(row)
    const int lrow = lane >> 3;
    const int c0 = (lane & 7) ^ ((lrow >> 1) & 7);            // rows 0..7:  key = (row >> 1) & 7
    const int c1 = (lane & 7) ^ ((4 + (lrow >> 1)) & 7);      // rows 8..15
    const uint32_t vb0 = (uint32_t)(lrow * (int)ldb + c0 * 16), vb1 = (uint32_t)((8 + lrow) * (int)ldb + c1 * 16);
    const uint32_t va0 = (uint32_t)(lrow * (int)lda + c0 * 16), va1 = (uint32_t)((8 + lrow) * (int)lda + c1 * 16);
    const uint32_t ring = (uint32_t)(size_t)smem + (uint32_t)wave * (uint32_t)(R * SLOT);

    auto issue = [&](int slot, int s) {         // K step s into ring slot `slot` (everything out of range past s_end)
        const int k0 = s * 128;
        const bool in = s < s_end;
        const uint32_t k_0 = (in && k0 + c0 * 16 < K) ? (uint32_t)k0 : OOB;
        const uint32_t k_1 = (in && k0 + c1 * 16 < K) ? (uint32_t)k0 : OOB;
        const uint32_t dst = ring + (uint32_t)(slot * SLOT);
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            sk_lds_dma16(rsrc_b, dst + w * 2048, vb0 + (uint32_t)(16 * w * (int)ldb) + k_0);
            sk_lds_dma16(rsrc_b, dst + w * 2048 + 1024, vb1 + (uint32_t)(16 * w * (int)ldb) + k_1);
        }
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            sk_lds_dma16(rsrc_a, dst + (NW + t) * 2048, va0 + (uint32_t)(16 * t * (int)lda) + k_0);
            sk_lds_dma16(rsrc_a, dst + (NW + t) * 2048 + 1024, va1 + (uint32_t)(16 * t * (int)lda) + k_1);
        }
    };

    v4f_k acc[NW][MT];
#pragma unroll
    for (int w = 0; w < NW; ++w)
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[w][t] = v4f_k{0.f, 0.f, 0.f, 0.f};

    // fragment: chunks g and g + 4 of row i of a tile
    const int key = (i >> 1) & 7;
    const int f_lo = i * 128 + ((g ^ key) << 4), f_hi = i * 128 + (((g + 4) ^ key) << 4);
    auto frag = [&](const uint8_t* tile) {
        const uint4 lo = *reinterpret_cast<const uint4*>(tile + f_lo);
        const uint4 hi = *reinterpret_cast<const uint4*>(tile + f_hi);
        return v8i_k{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
    };

#pragma unroll
    for (int r = 0; r < R; ++r) issue(r, s_begin + r);
    int slot = 0;
    for (int s = s_begin; s < s_end; ++s) {
        sk_wait_vmem<(R - 1) * LOADS>();          // all but the R - 1 younger slots have landed
        const uint8_t* base = smem + wave * (R * SLOT) + slot * SLOT;
        v8i_k bf[NW], af[MT];
#pragma unroll
        for (int w = 0; w < NW; ++w) bf[w] = frag(base + w * 2048);
#pragma unroll
        for (int t = 0; t < MT; ++t) af[t] = frag(base + (NW + t) * 2048);
#pragma unroll
        for (int w = 0; w < NW; ++w)
#pragma unroll
            for (int t = 0; t < MT; ++t)
                acc[w][t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bf[w], af[t], acc[w][t], FB, FA, 0, 0, 0, 0);
        issue(slot, s + R);
        slot = slot + 1 == R ? 0 : slot + 1;
    }
    sk_wait_vmem<0>();        // trailing (out-of-range) refills must land before the LDS is reused or handed back

    // ---- sum the K parts of a column group through LDS (the rings are free now)
    if constexpr (KS > 1) {
        __syncthreads();
        v4f_k* part = reinterpret_cast<v4f_k*>(smem);      // [NTW][KS - 1][NW * MT][64]
        const int grp = wave / KS;
        if (kp > 0) {
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int t = 0; t < MT; ++t) part[((grp * (KS - 1) + kp - 1) * (NW * MT) + w * MT + t) * 64 + lane] = acc[w][t];
        }
        __syncthreads();
        if (kp > 0) return;
#pragma unroll
        for (int p = 0; p < KS - 1; ++p)
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    const v4f_k o = part[((grp * (KS - 1) + p) * (NW * MT) + w * MT + t) * 64 + lane];
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

template <int FA, int FB, int MT, int KS, int NW>
static hipError_t launch_sk_dma(const uint8_t* a, int64_t lda, const float* sa, int row_a, const uint8_t* b, int64_t ldb,
                                const float* sb, int row_b, int M, int N, int K, void* out, int64_t ld_out, int out_f32,
                                int64_t grid, hipStream_t st) {
    constexpr int SLOT = (NW + MT) * 2048;
    constexpr int R = SLOT <= 4096 ? 5 : (SLOT <= 6144 ? 3 : 2);     // about 20 KB of ring per wavefront: two workgroups per CU
    constexpr int lds = 4 * R * SLOT;
    auto kern = gemm_fp8_skinny_dma_kernel<FA, FB, MT, KS, NW, R>;
    static DynamicLdsOnce attr;
    if (hipError_t e = attr.ensure(reinterpret_cast<const void*>(kern), lds); e != hipSuccess) return e;
    kern<<<dim3((unsigned)grid), dim3(256), lds, st>>>(a, lda, b, ldb, sa, row_a, sb, row_b, M, N, K, out, ld_out, out_f32);
    return hipGetLastError();
}

template <int FA, int FB>
static hipError_t launch_sk(const uint8_t* a, int64_t lda, const float* sa, int row_a, const uint8_t* b, int64_t ldb,
                            const float* sb, int row_b, int M, int N, int K, void* out, int64_t ld_out, int out_f32,
                            hipStream_t st) {
    const int mt = (M + 15) / 16;                 // 1..4
    // columns per wavefront: 16 or 32 (64 through the override).  Wider groups reuse every fragment of A
    // for two or four MFMAs but shorten the ring of K steps in flight, narrower ones give more wavefronts;
    // measured: 32 wins or ties from N = 6144 on, 64 never beats 32 (28672 x 8192: 5 % slower)
    int nw = N >= 6144 ? 2 : 1;
    if (const int v = knob(KNOB_SKINNY_NW); v == 1 || v == 2 || v == 4) nw = v;     // tuning override
    const int64_t groups = ((int64_t)N + 16 * nw - 1) / (16 * nw);
    // split K over the wavefronts of a workgroup until about 2048 wavefronts stream B
    int ks = 1;
    while (ks < 4 && groups * ks < 2048 && K / (ks * 2) >= 512) ks *= 2;
    const int64_t grid = (groups + (4 / ks) - 1) / (4 / ks);
    if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
    // LDS-DMA form for up to 32 rows when the 32-bit buffer offsets suffice (FP8MI355_SKINNY_DMA=0 / 1 overrides)
    const bool fits = lda < (1 << 23) && ldb < (1 << 23) && mt <= 2;
    if (fits && knob(KNOB_SKINNY_DMA) != 0) {
#define FP8K_SKD(MT_, KS_, NW_)                                                                               \
    if (mt == MT_ && ks == KS_ && nw == NW_)                                                                  \
        return launch_sk_dma<FA, FB, MT_, KS_, NW_>(a, lda, sa, row_a, b, ldb, sb, row_b, M, N, K, out, ld_out, out_f32, grid, st)
#define FP8K_SKD3(MT_) \
    FP8K_SKD(MT_, 1, 1); FP8K_SKD(MT_, 2, 1); FP8K_SKD(MT_, 4, 1); FP8K_SKD(MT_, 1, 2); FP8K_SKD(MT_, 2, 2); FP8K_SKD(MT_, 4, 2); \
    FP8K_SKD(MT_, 1, 4); FP8K_SKD(MT_, 2, 4); FP8K_SKD(MT_, 4, 4)
        FP8K_SKD3(1); FP8K_SKD3(2);
#undef FP8K_SKD3
#undef FP8K_SKD
    }
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
