// MX (microscaling) FP8 GEMM for gfx950, the block-scaled form of the "snake"
// kernel of gemm_fp8_snake.hip (same 256 x 256 tile, four wavefronts of 128 x 128,
// LDS-DMA loads, four-phase schedule, LDS layout and swizzle keys; see there).
//     out[m, n] = sum_blk 2^(ea[m,blk]-127) 2^(eb[n,blk]-127) sum_{k in blk} dec(a[m,k]) dec(b[n,k])
// with one E8M0 byte per row and block of 32 K-bytes (OCP MX specification v1.0).
// What is added: v_mfma_scale_f32_16x16x128_f8f6f4 takes, in lane (l % 16, g = l / 16),
// the scale byte of block g of operand row l % 16 (the 128 K-bytes of a step are 4
// blocks; the hardware routes each scale to the lanes that hold its block's bytes,
// which in this layout are chunks g and g + 4 of lanes ...).  Every K step therefore
// also brings one dword of scales per tile row into LDS (two extra LDS-DMA loads
// per wavefront: 64 A rows and 64 B rows), and every fragment read is followed by a
// one-byte LDS read of its scale.  The epilogue has no scaling left to do.
#include "fp8_device.hpp"
#include "launchers.hpp"
#include "tuning.hpp"

#include <type_traits>

namespace fp8k {

typedef int v4i_x __attribute__((ext_vector_type(4)));
typedef unsigned v4u_x __attribute__((ext_vector_type(4)));
typedef int v8i_x __attribute__((ext_vector_type(8)));
typedef float v4f_x __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_x __attribute__((ext_vector_type(2)));
typedef float f32x2_x __attribute__((ext_vector_type(2)));

namespace msn {
constexpr int BM = 256, BN = 256, BK = 128;
constexpr int NT = 256;
constexpr int WM = 128, WN = 128;
constexpr int TILE = (BM + BN) * BK;     // 64 KB of codes
constexpr int STAGE = TILE + (BM + BN) * 4;   // + one dword of scales per row
constexpr int SCBUF = (BM + BN) * 16;         // scales of four K steps, 16 bytes per row (SC16 mode)
constexpr int GROUP_M = 4;
constexpr int NUM_XCD = 8;
}  // namespace msn

__device__ __forceinline__ uint32_t msn_pack_bf16(float a, float b) {
    f32x2_x v = {a, b};
    bf16x2_x h = __builtin_convertvector(v, bf16x2_x);
    uint32_t r;
    __builtin_memcpy(&r, &h, 4);
    return r;
}

// 16 bytes per lane from a raw buffer straight into LDS at lds_addr + lane * 16
// (lds_addr wave-uniform).  Out-of-range lanes deliver zeros.  Inline assembly
// on purpose: the compiler must not know that these loads write LDS, or it
// would drain them before every LDS read and undo the prefetch.
__device__ __forceinline__ void msn_lds_dma16(v4i_x rsrc, uint32_t lds_addr, uint32_t voffset) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voffset), "s"(rsrc)
                 : "memory", "m0");
}
// 4 bytes per lane into LDS at lds_addr + lane * 4 (the scales of 64 rows)
__device__ __forceinline__ void msn_lds_dma4(v4i_x rsrc, uint32_t lds_addr, uint32_t voffset) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voffset), "s"(rsrc)
                 : "memory", "m0");
}
__device__ __forceinline__ void msn_wait_all_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// workgroup barrier behind the wave's own LDS reads (no wait for loads in flight)
__device__ __forceinline__ void msn_barrier_lds() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}
// wait until at most the five youngest loads are in flight (loads complete in issue order), own LDS reads done, barrier
__device__ __forceinline__ void msn_wait_vmem_but5_barrier() {
    asm volatile("s_waitcnt vmcnt(5) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// SC16 (K a multiple of 512): the scale bytes are fetched 16 per row at a time (four K steps, two buffers
// behind the stages) instead of 4 per row and K step.  A scale load touches one cache line per lane
// whatever its width; one dword per lane and step doubled the kernel's cache-line traffic and cost 20 %.
template <int FA, int FB, bool OUT_F32, bool SC16>
__global__ __launch_bounds__(msn::NT) void gemm_mxfp8_snake_kernel(
    const uint8_t* __restrict__ A, int64_t lda, const uint8_t* __restrict__ EA, int64_t ld_ea,
    const uint8_t* __restrict__ B, int64_t ldb, const uint8_t* __restrict__ EB, int64_t ld_eb, int M, int N,
    int K, void* __restrict__ out, int64_t ld_out, int tiles_m, int tiles_n) {
    using namespace msn;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // ---- workgroup -> tile (XCD-aware: ids are dealt round-robin to the 8 XCDs;
    //      each XCD gets a contiguous range of tiles walked in groups of tile rows)
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
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;

    // ---- buffer descriptors of this tile's operand panels (raw buffers, sizes in bytes)
    const int rows_a = M - m0 < BM ? M - m0 : BM, rows_b = N - n0 < BN ? N - n0 : BN;
    const uint64_t pa = reinterpret_cast<uint64_t>(A + (int64_t)m0 * lda);
    const uint64_t pb = reinterpret_cast<uint64_t>(B + (int64_t)n0 * ldb);
    const v4i_x rsrc_a = {(int)(uint32_t)pa, (int)(uint32_t)(pa >> 32), (int)((int64_t)(rows_a - 1) * lda + K), 0x00020000};
    const v4i_x rsrc_b = {(int)(uint32_t)pb, (int)(uint32_t)(pb >> 32), (int)((int64_t)(rows_b - 1) * ldb + K), 0x00020000};

    // scale panels: rows m0.. of EA, n0.. of EB, K / 32 bytes per row; wave w fetches rows 64 w + lane.
    // A negative leading dimension (SC16 only) means slabs of sixteen blocks, [K / 512][-ld rows][16 bytes]: the
    // 256 pieces a tile needs for four K steps are 4 KB in a row (8 cache lines per wave load instead of 64).
    // Rows past the operand's end then read the next slab's first rows instead of zeros: their products only
    // reach output rows / columns that are never stored.  The descriptor ends with the buffer.
    const bool slab_a = ld_ea < 0, slab_b = ld_eb < 0;
    const int64_t gsa = slab_a ? -ld_ea * 16 : 16, gsb = slab_b ? -ld_eb * 16 : 16;     // bytes from one group of four K steps to the next
    const uint64_t pea = reinterpret_cast<uint64_t>(EA + (int64_t)m0 * (slab_a ? 16 : ld_ea));
    const uint64_t peb = reinterpret_cast<uint64_t>(EB + (int64_t)n0 * (slab_b ? 16 : ld_eb));
    const int64_t nrec_a = slab_a ? (int64_t)(K / 512) * gsa - (int64_t)m0 * 16 : (int64_t)(rows_a - 1) * ld_ea + K / 32;
    const int64_t nrec_b = slab_b ? (int64_t)(K / 512) * gsb - (int64_t)n0 * 16 : (int64_t)(rows_b - 1) * ld_eb + K / 32;
    const v4i_x rsrc_ea = {(int)(uint32_t)pea, (int)(uint32_t)(pea >> 32), (int)nrec_a, 0x00020000};
    const v4i_x rsrc_eb = {(int)(uint32_t)peb, (int)(uint32_t)(peb >> 32), (int)nrec_b, 0x00020000};
    const uint32_t vea0 = (uint32_t)((wave * 64 + lane) * (slab_a ? 16 : (int)ld_ea)), veb0 = (uint32_t)((wave * 64 + lane) * (slab_b ? 16 : (int)ld_eb));
    const uint32_t gsa32 = (uint32_t)gsa, gsb32 = (uint32_t)gsb;
    const uint32_t lds_sc = (uint32_t)(size_t)smem + (uint32_t)TILE + (uint32_t)wave * 256u;   // + BM * 4 for B
    const uint32_t lds_sc16 = (uint32_t)(size_t)smem + (uint32_t)(2 * STAGE) + (uint32_t)wave * 1024u;   // + SCBUF per buffer, + BM * 16 for B

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
#pragma unroll
        for (int i = 0; i < 8; ++i) msn_lds_dma16(rsrc_a, la + i * 4096, va0 + (uint32_t)i * va_step + ka);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            msn_lds_dma16(rsrc_b, lb + i * 4096, ((i & 1) ? vb0_o + ko : vb0_e + ke) + (uint32_t)i * vb_step);
        if constexpr (SC16) {
            if (k0 == 0) {   // scales of steps 0..3 into scale buffer 0
                msn_lds_dma16(rsrc_ea, lds_sc16, vea0);
                msn_lds_dma16(rsrc_eb, lds_sc16 + BM * 16, veb0);
            }
        } else {
            const uint32_t ks = k0 < K ? (uint32_t)(k0 >> 5) : OOB;      // byte offset of this step's 4 blocks in a scale row
            msn_lds_dma4(rsrc_ea, lds_sc + (uint32_t)(stage * STAGE), vea0 + ks);
            msn_lds_dma4(rsrc_eb, lds_sc + (uint32_t)(stage * STAGE) + BM * 4, veb0 + ks);
        }
    };

    // ---- LDS -> fragments
    const int r16 = lane & 15, g = lane >> 4;
    const int key_a = (r16 >> 1) & 7;
    const int key_b = ((r16 >> 1) & 1) | ((r16 >> 2) << 1);
    int offa[2], offb[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        offa[c] = (wm0 + r16) * BK + (((g + 4 * c) ^ key_a) << 4);
        offb[c] = BM * BK + (wn0 + 16 * (r16 >> 2) + (r16 & 3)) * BK + (((g + 4 * c) ^ key_b) << 4);
    }
    constexpr int RS = SC16 ? 16 : 4;       // bytes per row in the scale area
    const int offsa = (SC16 ? 0 : TILE) + (wm0 + r16) * RS + g;                                     // scale byte of block g of this lane's A row
    const int offsb = (SC16 ? 0 : TILE) + BM * RS + (wn0 + 16 * (r16 >> 2) + (r16 & 3)) * RS + g;   // ... B row
    v8i_x af[2][4], bf[2][4];   // [half][fragment in half]
    int sa[2], sb[2];           // their scale bytes: byte f of sa[half] belongs to fragment f (selected by op_sel)
    auto read_a = [&](const uint8_t* s, int half, int f) {
        const int row_off = (half * 4 + f) * 16 * BK;
        const uint4 x0 = *reinterpret_cast<const uint4*>(s + offa[0] + row_off);
        const uint4 x1 = *reinterpret_cast<const uint4*>(s + offa[1] + row_off);
        af[half][f] = v8i_x{(int)x0.x, (int)x0.y, (int)x0.z, (int)x0.w, (int)x1.x, (int)x1.y, (int)x1.z, (int)x1.w};
    };
    // the four scale bytes of a fragment half, packed into one register
    // (read and packing are separate steps so that the main loop can put MFMAs between them:
    // packed right after the reads, every packing waited out the LDS latency)
    auto scales_a_read = [&](const uint8_t* s, int half, uint32_t (&raw)[4]) {
        const int o = offsa + half * (64 * RS);
        raw[0] = s[o]; raw[1] = s[o + 16 * RS]; raw[2] = s[o + 32 * RS]; raw[3] = s[o + 48 * RS];
    };
    auto scales_b_read = [&](const uint8_t* s, int half, uint32_t (&raw)[4]) {
        const int o = offsb + half * (64 * RS);
        raw[0] = s[o]; raw[1] = s[o + 4 * RS]; raw[2] = s[o + 8 * RS]; raw[3] = s[o + 12 * RS];
    };
    auto scales_pack = [&](const uint32_t (&raw)[4]) { return (int)(raw[0] | (raw[1] << 8) | (raw[2] << 16) | (raw[3] << 24)); };
    auto scales_a = [&](const uint8_t* s, int half) { uint32_t raw[4]; scales_a_read(s, half, raw); return scales_pack(raw); };
    auto scales_b = [&](const uint8_t* s, int half) { uint32_t raw[4]; scales_b_read(s, half, raw); return scales_pack(raw); };
    auto read_b = [&](const uint8_t* s, int half, int f) {
        const int row_off = (half * 64 + f * 4) * BK;   // group `half`, fragment t = f
        const uint4 x0 = *reinterpret_cast<const uint4*>(s + offb[0] + row_off);
        const uint4 x1 = *reinterpret_cast<const uint4*>(s + offb[1] + row_off);
        bf[half][f] = v8i_x{(int)x0.x, (int)x0.y, (int)x0.z, (int)x0.w, (int)x1.x, (int)x1.y, (int)x1.z, (int)x1.w};
    };

    v4f_x acc[8][8];   // [A fragment][B fragment]
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = v4f_x{0.f, 0.f, 0.f, 0.f};

    // MFMA number t of a phase pairs A fragment t / 4 with B fragment t % 4: the byte selectors of the
    // two packed scale registers are immediates.  Written as inline assembly with the accumulator
    // tied to the destination: through the builtin the compiler gives the scaled MFMA a destination
    // different from its accumulator input and copies every accumulator back (three extra moves per
    // MFMA in this loop).  The instructions around it are far enough apart for its result and operand
    // hazards: an accumulator is touched once per 16 MFMAs and read by other instructions only after
    // the loop's last barrier; the scale registers are packed at least one phase before their use.
#define MSN_CASE(T, SEL, FMT)                                                                                  \
    case T:                                                                                                    \
        asm volatile("v_mfma_scale_f32_16x16x128_f8f6f4 %0, %1, %2, %0, %3, %4 " SEL FMT                       \
                     : "+a"(c)                                                                                 \
                     : "v"(b), "v"(a), "v"(sbp), "v"(sap));                                                    \
        break;
#define MSN_ALL(FMT)                                                                                           \
    switch (t) {                                                                                               \
            MSN_CASE(0, "op_sel:[0,0,0] op_sel_hi:[0,0,0]", FMT) \
            MSN_CASE(1, "op_sel:[1,0,0] op_sel_hi:[0,0,0]", FMT) \
            MSN_CASE(2, "op_sel:[0,0,0] op_sel_hi:[1,0,0]", FMT) \
            MSN_CASE(3, "op_sel:[1,0,0] op_sel_hi:[1,0,0]", FMT) \
            MSN_CASE(4, "op_sel:[0,1,0] op_sel_hi:[0,0,0]", FMT) \
            MSN_CASE(5, "op_sel:[1,1,0] op_sel_hi:[0,0,0]", FMT) \
            MSN_CASE(6, "op_sel:[0,1,0] op_sel_hi:[1,0,0]", FMT) \
            MSN_CASE(7, "op_sel:[1,1,0] op_sel_hi:[1,0,0]", FMT) \
            MSN_CASE(8, "op_sel:[0,0,0] op_sel_hi:[0,1,0]", FMT) \
            MSN_CASE(9, "op_sel:[1,0,0] op_sel_hi:[0,1,0]", FMT) \
            MSN_CASE(10, "op_sel:[0,0,0] op_sel_hi:[1,1,0]", FMT) \
            MSN_CASE(11, "op_sel:[1,0,0] op_sel_hi:[1,1,0]", FMT) \
            MSN_CASE(12, "op_sel:[0,1,0] op_sel_hi:[0,1,0]", FMT) \
            MSN_CASE(13, "op_sel:[1,1,0] op_sel_hi:[0,1,0]", FMT) \
            MSN_CASE(14, "op_sel:[0,1,0] op_sel_hi:[1,1,0]", FMT) \
            MSN_CASE(15, "op_sel:[1,1,0] op_sel_hi:[1,1,0]", FMT)                                             \
    }
    auto mfma_sel = [&](int t, const v8i_x& b, const v8i_x& a, v4f_x c, int sbp, int sap) -> v4f_x {
        if constexpr (FB == 0 && FA == 0) { MSN_ALL("") }
        if constexpr (FB == 1 && FA == 0) { MSN_ALL(" cbsz:1") }
        if constexpr (FB == 0 && FA == 1) { MSN_ALL(" blgp:1") }
        if constexpr (FB == 1 && FA == 1) { MSN_ALL(" cbsz:1 blgp:1") }
        return c;
    };
#undef MSN_ALL
#undef MSN_CASE

    // one phase: 16 MFMAs of A half AH x B half BH; in its slots, optionally the
    // reads of one fragment half (RD_A: 1 = A half RH, 0 = B half RH, -1 = none)
    // from stage `rs`, CNT of the step's sixteen LDS-DMA refill loads from number L0 on (0-7: the B part,
    // 8-15: the A part), and the refill of one operand's scales (SCD: 0 = A, 1 = B, -1 = none).
    auto phase = [&](auto ah_t, auto bh_t, auto rda_t, auto rh_t, auto l0_t, auto cnt_t, auto scd_t, const uint8_t* rs, uint32_t la, uint32_t lb,
                     uint32_t ka, uint32_t ke, uint32_t ko, uint32_t lsc, uint32_t ks, const uint8_t* rsc, bool sc_issue) {
        constexpr int AH = decltype(ah_t)::value, BH = decltype(bh_t)::value, RDA = decltype(rda_t)::value,
                      RH = decltype(rh_t)::value, L0 = decltype(l0_t)::value, CNT = decltype(cnt_t)::value,
                      DMA = decltype(scd_t)::value;
        uint32_t raw[4] = {0, 0, 0, 0};
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            const int i = t >> 2, j = (i & 1) ? 3 - (t & 3) : (t & 3);   // boustrophedon: one operand stays between neighbours
            acc[AH * 4 + i][BH * 4 + j] = mfma_sel(4 * i + j, bf[BH][j], af[AH][i], acc[AH * 4 + i][BH * 4 + j], sb[BH], sa[AH]);
            if constexpr (RDA == 1) { if (t % 2 == 0 && t < 8) read_a(rs, RH, t / 2); }
            if constexpr (RDA == 0) { if (t % 2 == 0 && t < 8) read_b(rs, RH, t / 2); }
            if (t % 2 == 1 && t / 2 < CNT) {
                const int q = L0 + t / 2;
                if (q < 8) msn_lds_dma16(rsrc_b, lb + q * 4096, ((q & 1) ? vb0_o + ko : vb0_e + ke) + (uint32_t)q * vb_step);
                else msn_lds_dma16(rsrc_a, la + (q - 8) * 4096, va0 + (uint32_t)(q - 8) * va_step + ka);
            }
            // scales of the half that was read in slots 0..6, packed (the half is not in use in this phase)
            if constexpr (RDA == 1) { if (t == 9) scales_a_read(rsc, RH, raw); if (t == 14) sa[RH] = scales_pack(raw); }
            if constexpr (RDA == 0) { if (t == 9) scales_b_read(rsc, RH, raw); if (t == 14) sb[RH] = scales_pack(raw); }
            // the refill of the scales rides in a slot that has neither a read nor a data load
            if constexpr (SC16) {
                // (lsc, ks: scale buffer and number of the next group of four steps)
                if constexpr (DMA == 0) { if (t == 8 && sc_issue) msn_lds_dma16(rsrc_ea, lsc, vea0 + ks * gsa32); }
                if constexpr (DMA == 1) { if (t == 8 && sc_issue) msn_lds_dma16(rsrc_eb, lsc + BM * 16, veb0 + ks * gsb32); }
            } else {
                if constexpr (DMA == 0) { if (t == 8) msn_lds_dma4(rsrc_ea, lsc, vea0 + ks); }
                if constexpr (DMA == 1) { if (t == 8) msn_lds_dma4(rsrc_eb, lsc + BM * 4, veb0 + ks); }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using IN = std::integral_constant<int, -1>;
    using I5 = std::integral_constant<int, 5>;
    using I6 = std::integral_constant<int, 6>;
    using I11 = std::integral_constant<int, 11>;

    // K steps are processed in pairs (the B halves swap roles every step); an odd
    // number of steps gets one phantom step whose loads are all out of range (zeros).
    const int ksteps = (K + BK - 1) / BK;
    const int kpairs = (ksteps + 1) / 2;
    if (ksteps > 0) issue_loads(0, 0);
    if (ksteps > 0) {
        msn_wait_all_vmem();
        __syncthreads();                       // stage 0 landed for every wave
        issue_loads(1, BK);                    // (out of range if there is no step 1)
#pragma unroll
        for (int f = 0; f < 4; ++f) { read_a(smem, 0, f); read_b(smem, 0, f); }
        sa[0] = scales_a(SC16 ? smem + 2 * STAGE : smem, 0);
        sb[0] = scales_b(SC16 ? smem + 2 * STAGE : smem, 0);
        sa[1] = sb[1] = 0;
        __builtin_amdgcn_sched_barrier(0);

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
                // SC16: the scales of step kk sit in buffer (kk / 4) % 2 at byte 4 * (kk % 4) of their row; the group
                // of steps 4q+4.. is fetched during step 4q+1 into the buffer that steps 4q-4.. have left
                const int q1 = (k >> 2) + 1;
                const bool sc_issue = SC16 && (k & 3) == 1 && q1 * 512 < K;
                const uint32_t lsc = SC16 ? lds_sc16 + (uint32_t)((q1 & 1) * SCBUF) : lds_sc + (uint32_t)(par * STAGE);
                const uint32_t ks = SC16 ? (uint32_t)q1 : (k2 < K ? (uint32_t)(k2 >> 5) : OOB);   // SC16: the group's number
                const uint8_t* c_cur = SC16 ? smem + 2 * STAGE + ((k >> 2) & 1) * SCBUF + (k & 3) * 4 : s_cur;
                const uint8_t* c_nxt = SC16 ? smem + 2 * STAGE + (((k + 1) >> 2) & 1) * SCBUF + ((k + 1) & 3) * 4 : s_nxt;
                // The sixteen data loads of the refill are spread over phases 2-4 (B part first: it is read out after
                // phase 1; the A part after phase 2); the scale loads stay behind the wait in the middle of the step, so
                // that the five youngest loads at that wait are always phase 2's.
                if (par == 0) {
                    // even step: B order 0,1,1,0.  Holds A0, B0 of this step.
                    phase(I0{}, I0{}, I0{}, I1{}, I0{}, I0{}, IN{}, s_cur, la, lb, ka, ke, ko, lsc, ks, c_cur, sc_issue);    // (A0,B0) | read B1 of this step
                    msn_barrier_lds();                 // this step's B part is read out by everyone
                    phase(I0{}, I1{}, I1{}, I1{}, I0{}, I5{}, IN{}, s_cur, la, lb, ka, ke, ko, lsc, ks, c_cur, sc_issue);    // (A0,B1) | read A1 of this step, refill B 0-4
                    msn_wait_vmem_but5_barrier();      // step k+1 has landed for everyone; this step's A part and scales are read out
                    phase(I1{}, I1{}, I1{}, I0{}, I5{}, I6{}, I0{}, s_nxt, la, lb, ka, ke, ko, lsc, ks, c_nxt, sc_issue);    // (A1,B1) | read A0 of step k+1, refill B 5-7, A 0-2, A scales
                    phase(I1{}, I0{}, I0{}, I1{}, I11{}, I5{}, I1{}, s_nxt, la, lb, ka, ke, ko, lsc, ks, c_nxt, sc_issue);   // (A1,B0) | read B1 of step k+1, refill A 3-7, B scales
                } else {
                    // odd step: B order 1,0,0,1.  Holds A0, B1 of this step.
                    phase(I0{}, I1{}, I0{}, I0{}, I0{}, I0{}, IN{}, s_cur, la, lb, ka, ke, ko, lsc, ks, c_cur, sc_issue);    // (A0,B1) | read B0 of this step
                    msn_barrier_lds();
                    phase(I0{}, I0{}, I1{}, I1{}, I0{}, I5{}, IN{}, s_cur, la, lb, ka, ke, ko, lsc, ks, c_cur, sc_issue);    // (A0,B0) | read A1 of this step, refill B 0-4
                    msn_wait_vmem_but5_barrier();
                    phase(I1{}, I0{}, I1{}, I0{}, I5{}, I6{}, I0{}, s_nxt, la, lb, ka, ke, ko, lsc, ks, c_nxt, sc_issue);    // (A1,B0) | read A0 of step k+1, refill B 5-7, A 0-2, A scales
                    phase(I1{}, I1{}, I0{}, I0{}, I11{}, I5{}, I1{}, s_nxt, la, lb, ka, ke, ko, lsc, ks, c_nxt, sc_issue);   // (A1,B1) | read B0 of step k+1, refill A 3-7, B scales
                }
            }
        }
        msn_wait_all_vmem();    // trailing (out-of-range) refills must not land in the epilogue's LDS
    }

    // ---- epilogue.  Lane holds output row m = 16*fi + l%16 and, per 64-wide B group,
    //      the 16 consecutive columns 16*g + 4*t + r (fragment t, accumulator r).
    __syncthreads();   // nobody's trailing refill can land in the staging rows below

    if constexpr (OUT_F32) {
#pragma unroll
        for (int fi = 0; fi < 8; ++fi) {
            const int r_loc = 16 * fi + r16;               // row inside the wave's quadrant
            const int m = m0 + wm0 + r_loc;
#pragma unroll
            for (int grp = 0; grp < 2; ++grp) {
                float v[16];
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[4 * t + r] = acc[fi][grp * 4 + t][r];
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
        uint16_t* orow = static_cast<uint16_t*>(out) + (int64_t)(m0 + wm0 + (lane >> 4)) * ld_out + n_rd;
#pragma unroll
        for (int fi = 0; fi < 8; ++fi) {
            const int r_loc = 16 * fi + r16;
            uint8_t* row = q + r_loc * 256;
#pragma unroll
            for (int grp = 0; grp < 2; ++grp) {
                uint32_t p[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int e0 = 2 * e, e1 = 2 * e + 1;
                    p[e] = msn_pack_bf16(acc[fi][grp * 4 + (e0 >> 2)][e0 & 3], acc[fi][grp * 4 + (e1 >> 2)][e1 & 3]);
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
                const int rr = 16 * fi + 4 * it + (lane >> 4);      // row in the quadrant
                const uint4 v = *reinterpret_cast<const uint4*>(q + rr * 256 + ((c_rd ^ (rr & 15)) << 4));
                uint16_t* dst = orow + (int64_t)(16 * fi + 4 * it) * ld_out;
                if (interior) {
                    // streaming store: the output is not read again by this kernel and
                    // should not push the operand panels out of L2
                    __builtin_nontemporal_store(v4u_x{v.x, v.y, v.z, v.w}, reinterpret_cast<v4u_x*>(dst));
                } else if (m0 + wm0 + rr < M && n_rd < N) {
                    if (n_rd + 8 <= N) {
                        __builtin_nontemporal_store(v4u_x{v.x, v.y, v.z, v.w}, reinterpret_cast<v4u_x*>(dst));
                    } else {
                        const uint32_t w4[4] = {v.x, v.y, v.z, v.w};
                        for (int e = 0; n_rd + e < N; ++e) dst[e] = (uint16_t)(w4[e >> 1] >> ((e & 1) * 16));
                    }
                }
            }
        }
    }
}

template <int FA, int FB, bool OUT_F32, bool SC16>
static hipError_t launch_msn(const uint8_t* a, int64_t lda, const uint8_t* ea, int64_t ld_ea, const uint8_t* b, int64_t ldb,
                             const uint8_t* eb, int64_t ld_eb, int M, int N, int K, void* out, int64_t ld_out,
                             hipStream_t st) {
    using namespace msn;
    auto kern = gemm_mxfp8_snake_kernel<FA, FB, OUT_F32, SC16>;
    constexpr int lds = 2 * STAGE + (SC16 ? 2 * SCBUF : 0);
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

// same contract as launch_gemm_mxfp8; additionally lda, ldb < 2^23 and ld_ea, ld_eb < 2^23
// (buffer offsets are 32-bit)
hipError_t launch_gemm_mxfp8_snake(const uint8_t* a, int64_t lda, int fmt_a, const uint8_t* ea, int64_t ld_ea,
                                   const uint8_t* b, int64_t ldb, int fmt_b, const uint8_t* eb, int64_t ld_eb, int64_t M,
                                   int64_t N, int64_t K, void* out, int64_t ld_out, int out_f32, hipStream_t st) {
    if (M == 0 || N == 0) return hipSuccess;
    const int m = (int)M, n = (int)N, k = (int)K;
    const bool sc16 = K > 0 && K % 512 == 0;   // whole 16-byte scale chunks per row
#define FP8K_MSN(FA_, FB_)                                                                                  \
    if (fmt_a == FA_ && fmt_b == FB_)                                                                       \
        return sc16 ? (out_f32 ? launch_msn<FA_, FB_, true, true>(a, lda, ea, ld_ea, b, ldb, eb, ld_eb, m, n, k, out, ld_out, st)   \
                               : launch_msn<FA_, FB_, false, true>(a, lda, ea, ld_ea, b, ldb, eb, ld_eb, m, n, k, out, ld_out, st)) \
                    : (out_f32 ? launch_msn<FA_, FB_, true, false>(a, lda, ea, ld_ea, b, ldb, eb, ld_eb, m, n, k, out, ld_out, st)  \
                               : launch_msn<FA_, FB_, false, false>(a, lda, ea, ld_ea, b, ldb, eb, ld_eb, m, n, k, out, ld_out, st))
    FP8K_MSN(FMT_E4M3FN, FMT_E4M3FN);
    FP8K_MSN(FMT_E5M2, FMT_E4M3FN);
    FP8K_MSN(FMT_E4M3FN, FMT_E5M2);
    FP8K_MSN(FMT_E5M2, FMT_E5M2);
#undef FP8K_MSN
    return hipErrorInvalidValue;
}

}  // namespace fp8k
