// bfloat16 GEMM with the contraction axis on the ROWS of both operands,
//     out[i, j] = sum_c a[c, i] * b[c, j]        (a [C, I], b [C, J] row-major, fp32 accumulate, bf16 out),
// the weight gradient dW = dY^T X of the rowwise_gw_hp recipe (Appendix A of the
// paper keeps that product in high precision), for large problems.
//
// Same skeleton as the FP8 "snake" kernel (gemm_fp8_snake.hip): 256 x 256 tile,
// four wavefronts of 128 x 128, two LDS stages of 64 KB filled by LDS-DMA
// (buffer_load_dwordx4 ... lds), the four-phase schedule in which every phase
// pairs one half of the A fragments with one half of the B fragments and reads
// exactly one new half.  What differs is where the transposition happens: the
// operand tiles go into LDS exactly as they lie in memory, as rows of the
// contraction index c (64 per K step) holding 256 consecutive i (512 bytes), and
// the MFMA operands are read with ds_read_b64_tr_b16, gfx950's transposing LDS
// read: the 16 lanes of a group fetch 8-byte pieces (input lane 4e + q: row e,
// elements 4q..4q+3) and output lane j receives element j of rows e = 0..3.
// So a lane ends up with 4 consecutive c of one i per read, and two reads make
// the 8 contraction elements that v_mfma_f32_16x16x32_bf16 takes per lane
// (lane (i, g): c = 8g..8g+7 of the 32 of one instruction; any assignment works
// as long as both operands use the same one).  A former FP8 MFMA slot
// (16x16x128, 32 cycles) becomes two bf16 MFMAs (2 x 16 cycles), a former
// 2 x 128-bit fragment read becomes 4 transposing 64-bit reads: the schedule
// carries over unchanged.
//
// LDS bank layout: row c holds 32 chunks of 16 bytes; chunk pair p (32 bytes =
// the 16 i of one fragment) is stored at pair p ^ key(c), key(c) = (c & 3) |
// (((c >> 3) & 1) << 2).  A transposing read touches rows 8g + e (+ const): the
// 16 rows of lanes 0..31 have 8 distinct keys, i.e. 8 distinct 32-byte bank
// groups, each hit by the 4 lanes of a row with different 8-byte pieces.  The
// swizzle is applied on the global side of the LDS-DMA (lane fetches chunk
// slot ^ (key << 1)).
#include "fp8_device.hpp"
#include "launchers.hpp"
#include "tuning.hpp"

#include <type_traits>

namespace fp8k {

typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef unsigned v4u_tt __attribute__((ext_vector_type(4)));
typedef short v4s_t __attribute__((ext_vector_type(4)));
typedef short v8s_t __attribute__((ext_vector_type(8)));
typedef __bf16 v8bf_s __attribute__((ext_vector_type(8)));
typedef float v4f_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

namespace bts {
constexpr int BI = 256, BJ = 256, BC = 64;
constexpr int NT = 256;
constexpr int WI = 128, WJ = 128;
constexpr int ROWB = 512;                    // bytes of one c row of an operand tile
constexpr int PART = BC * ROWB;              // 32 KB per operand
constexpr int STAGE = 2 * PART;              // 64 KB
constexpr int GROUP_I = 4;
constexpr int NUM_XCD = 8;
}  // namespace bts

__device__ __forceinline__ uint32_t bts_pack_bf16(float a, float b) {
    f32x2_t v = {a, b};
    bf16x2_t h = __builtin_convertvector(v, bf16x2_t);
    uint32_t r;
    __builtin_memcpy(&r, &h, 4);
    return r;
}

// see gemm_fp8_snake.hip: inline assembly so that the compiler does not drain these loads before LDS reads
__device__ __forceinline__ void bts_lds_dma16(v4i_t rsrc, uint32_t lds_addr, uint32_t voffset) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voffset), "s"(rsrc)
                 : "memory", "m0");
}
__device__ __forceinline__ void bts_wait_all_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// workgroup barrier behind the wave's own LDS reads (no wait for loads in flight)
__device__ __forceinline__ void bts_barrier_lds() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}
// wait until at most the five youngest loads are in flight (loads complete in issue order), own LDS reads done, barrier
__device__ __forceinline__ void bts_wait_vmem_but5_barrier() {
    asm volatile("s_waitcnt vmcnt(5) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// HALF: a workgroup computes half a tile, the rows (i) of ONE A half of every wave's quadrant against the
// whole width, as in the FP8 kernel: the launcher runs the tiles of a last round that would fill at most half
// of the CUs this way (this kernel is bound by the LDS, not by power: a partly filled round costs a whole
// one - 3.25 to 4 rounds of tiles all took 1.50-1.57 ms).  A launch covers `units` units from tile
// `tile_first`: whole tiles, or with HALF the two halves of each tile.  Two phases per K step:
// (A,B0) | read B1, barrier, (A,B1) | read A and B0 of the next step, refill (the A loads skip the other
// half's columns: their lanes point past the end and nothing is fetched).
template <bool HALF>
__global__ __launch_bounds__(bts::NT) void gemm_bf16_at_b_snake_kernel(
    const uint16_t* __restrict__ A, int64_t lda, const uint16_t* __restrict__ B, int64_t ldb, int I, int J, int C,
    uint16_t* __restrict__ out, int64_t ld_out, int tiles_i, int tiles_j, int tile_first, int units) {
    using namespace bts;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // ---- workgroup -> tile (XCD-aware, as in the FP8 kernel)
    const int per_xcd = gridDim.x / NUM_XCD;
    const int unit = (blockIdx.x % NUM_XCD) * per_xcd + blockIdx.x / NUM_XCD;
    if (unit >= units) return;
    const int logical = tile_first + (HALF ? unit >> 1 : unit);
    const int ah = HALF ? __builtin_amdgcn_readfirstlane(unit & 1) : 0;
    const int in_group = GROUP_I * tiles_j;
    const int first_i = (logical / in_group) * GROUP_I;
    const int gsize = tiles_i - first_i < GROUP_I ? tiles_i - first_i : GROUP_I;
    const int ti = first_i + (logical % in_group) % gsize;
    const int tj = (logical % in_group) / gsize;
    const int i0 = ti * BI, j0 = tj * BJ;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wi0 = (wave >> 1) * WI, wj0 = (wave & 1) * WJ;

    // ---- buffer descriptors: the tile's column panel of each operand, all C rows (sizes in bytes).
    //      Rows past C lie beyond the end and arrive as zeros.
    const int cols_a = I - i0 < BI ? I - i0 : BI, cols_b = J - j0 < BJ ? J - j0 : BJ;
    const uint64_t pa = reinterpret_cast<uint64_t>(A + i0);
    const uint64_t pb = reinterpret_cast<uint64_t>(B + j0);
    const v4i_t rsrc_a = {(int)(uint32_t)pa, (int)(uint32_t)(pa >> 32), (int)(((int64_t)(C - 1) * lda + cols_a) * 2), 0x00020000};
    const v4i_t rsrc_b = {(int)(uint32_t)pb, (int)(uint32_t)(pb >> 32), (int)(((int64_t)(C - 1) * ldb + cols_b) * 2), 0x00020000};

    // ---- global -> LDS.  One instruction fills 1 KB = rows 2n, 2n + 1 of a part; wave w takes
    //      n = 4 * i + w for load i = 0..7: row = 8 * i + 2 * w + lane / 32, lane % 32 = chunk slot,
    //      which receives logical chunk slot ^ (key(row) << 1); key's high bit is the parity of i.
    constexpr uint32_t OOB = 0x80000000u;   // offsets stay below 2^31 (checked on the host)
    const int lrow = 2 * wave + (lane >> 5);
    const int slot = lane & 31;
    const int ch_e = slot ^ ((lrow & 3) << 1), ch_o = slot ^ (((lrow & 3) | 4) << 1);
    // HALF: only the 64 columns of this A half in each quadrant (chunks with (chunk / 8) % 2 == ah) are fetched
    const bool use_e = !HALF || ((ch_e >> 3) & 1) == ah, use_o = !HALF || ((ch_o >> 3) & 1) == ah;
    const uint32_t va_e = (uint32_t)(lrow * (int)lda * 2 + ch_e * 16) + ((ch_e * 8 < cols_a && use_e) ? 0u : OOB);
    const uint32_t va_o = (uint32_t)(lrow * (int)lda * 2 + ch_o * 16) + ((ch_o * 8 < cols_a && use_o) ? 0u : OOB);
    const uint32_t vb_e = (uint32_t)(lrow * (int)ldb * 2 + ch_e * 16) + (ch_e * 8 < cols_b ? 0u : OOB);
    const uint32_t vb_o = (uint32_t)(lrow * (int)ldb * 2 + ch_o * 16) + (ch_o * 8 < cols_b ? 0u : OOB);
    const uint32_t va_row8 = (uint32_t)(8 * (int)lda * 2), vb_row8 = (uint32_t)(8 * (int)ldb * 2);
    const uint32_t lds_base = (uint32_t)(size_t)smem + (uint32_t)wave * 1024u;
    // load i of a part: LDS offset i * 4096 (+ wave * 1024), global rows 8 i + lrow
    auto dma_a = [&](uint32_t la, int i, uint32_t step_off) {
        bts_lds_dma16(rsrc_a, la + i * 4096, ((i & 1) ? va_o : va_e) + (uint32_t)i * va_row8 + step_off);
    };
    auto dma_b = [&](uint32_t lb, int i, uint32_t step_off) {
        bts_lds_dma16(rsrc_b, lb + i * 4096, ((i & 1) ? vb_o : vb_e) + (uint32_t)i * vb_row8 + step_off);
    };
    const uint32_t a_step = (uint32_t)(BC * (int)lda * 2), b_step = (uint32_t)(BC * (int)ldb * 2);
    auto issue_loads = [&](int stage, int step) {
        const uint32_t la = lds_base + (uint32_t)(stage * STAGE), lb = la + PART;
#pragma unroll
        for (int i = 0; i < 8; ++i) dma_a(la, i, (uint32_t)step * a_step);
#pragma unroll
        for (int i = 0; i < 8; ++i) dma_b(lb, i, (uint32_t)step * b_step);
    };

    // ---- LDS -> fragments (transposing reads).  Input lane (g, e, q) = (lane / 16, (lane % 16) / 4, lane % 4)
    //      points at row 32 s + 8 g + 4 h + e, chunk pair (fragment index ^ key), piece q.
    const int r16 = lane & 15, g = lane >> 4;
    const int e_in = r16 >> 2, q_in = r16 & 3;
    const int key = e_in | ((g & 1) << 2);
    const int lane_off = (8 * g + e_in) * ROWB + q_in * 8;
    // fragment f of the wave's quadrant: chunk pair ((quadrant / 16) | (f ^ key)); computed per read
    // (one xor-add) rather than kept in 16 registers
    const int key5 = key << 5;
    const int base_a = lane_off + ((wi0 >> 4) << 5), base_b = PART + lane_off + ((wj0 >> 4) << 5);
    typedef __attribute__((address_space(3))) v4s_t lds_v4s;
    auto read_frag = [&](const uint8_t* s, int off, v8bf_s (&dst)[2]) {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const v4s_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s*)(s + off + sub * 32 * ROWB));
            const v4s_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s*)(s + off + sub * 32 * ROWB + 4 * ROWB));
            const v8s_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            dst[sub] = __builtin_bit_cast(v8bf_s, both);
        }
    };
    v8bf_s af[2][4][2], bf[2][4][2];   // [half][fragment in half][k sub-step]
    auto read_a = [&](const uint8_t* s, int half, int f) { read_frag(s, base_a + (key5 ^ ((half * 4 + f) << 5)), af[half][f]); };
    // HALF: fragment f of this workgroup's A half into fragment set `dst`
    const int ah4 = ah << 7;                 // (4 * ah) << 5
    auto read_ah = [&](const uint8_t* s, auto dst_t, int f) {
        read_frag(s, base_a + (key5 ^ (ah4 | (f << 5))), af[decltype(dst_t)::value][f]);
    };
    auto read_b = [&](const uint8_t* s, int half, int f) { read_frag(s, base_b + (key5 ^ ((half * 4 + f) << 5)), bf[half][f]); };

    v4f_t acc[8][8];   // [A fragment][B fragment]
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = v4f_t{0.f, 0.f, 0.f, 0.f};

    // The MFMA as inline assembly with the accumulator tied to the destination: through the builtin
    // the compiler does not accumulate in place here (it rotates the accumulators through other
    // registers with copies in the main loop).
    auto mfma = [&](v4f_t& c, const v8bf_s& first, const v8bf_s& second) {
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(first), "v"(second));
    };
    // one phase: 32 MFMA slots (A half AH x B half BH: the 16 tile pairs with the first 32 contraction
    // elements, then the same 16 with the second 32, so that an accumulator is reused only after 16
    // instructions); in its slots the reads of one fragment half (RDA: 1 = A half RH, 0 = B half RH)
    // from stage `rs`, and CNT of the step's sixteen LDS-DMA refill loads, from number L0 on
    // (0-7: the B part, 8-15: the A part)
    auto phase = [&](auto ah_t, auto bh_t, auto rda_t, auto rh_t, auto l0_t, auto cnt_t, const uint8_t* rs, uint32_t la, uint32_t lb,
                     uint32_t sa_off, uint32_t sb_off) {
        constexpr int AH = decltype(ah_t)::value, BH = decltype(bh_t)::value, RDA = decltype(rda_t)::value,
                      RH = decltype(rh_t)::value, L0 = decltype(l0_t)::value, CNT = decltype(cnt_t)::value;
#pragma unroll
        for (int t = 0; t < 32; ++t) {
            const int sub = t >> 4, i = (t & 15) >> 2, j = (i & 1) ? 3 - (t & 3) : (t & 3);   // boustrophedon inside a pass
            mfma(acc[AH * 4 + i][BH * 4 + j], bf[BH][j][sub], af[AH][i][sub]);
            if constexpr (RDA == 1) { if (t % 4 == 0 && t < 16) read_a(rs, RH, t / 4); }
            if constexpr (RDA == 0) { if (t % 4 == 0 && t < 16) read_b(rs, RH, t / 4); }
            if (t % 4 == 2 && t / 4 < CNT) {
                const int q = L0 + t / 4;
                if (q < 8) dma_b(lb, q, sb_off); else dma_a(la, q - 8, sa_off);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I5 = std::integral_constant<int, 5>;
    using I6 = std::integral_constant<int, 6>;
    using I11 = std::integral_constant<int, 11>;

    // K steps in pairs (the B halves swap roles every step); an odd count gets one phantom
    // step whose loads are all past the end (zeros)
    const int ksteps = (C + BC - 1) / BC;
    const int kpairs = (ksteps + 1) / 2;
    if (ksteps > 0) {
        issue_loads(0, 0);
        bts_wait_all_vmem();
        __syncthreads();
        issue_loads(1, 1);
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            if constexpr (HALF) read_ah(smem, I0{}, f); else read_a(smem, 0, f);
            read_b(smem, 0, f);
        }
        __builtin_amdgcn_sched_barrier(0);

        if constexpr (HALF) {
            auto hstep = [&](auto par_t, int k) {
                constexpr int PAR = decltype(par_t)::value;
                using PN = std::integral_constant<int, PAR ^ 1>;
                const uint8_t* s_cur = smem + PAR * STAGE;
                const uint8_t* s_nxt = smem + (PAR ^ 1) * STAGE;
                const uint32_t sa_off = (uint32_t)(k + 2) * a_step, sb_off = (uint32_t)(k + 2) * b_step;
                const uint32_t la = lds_base + (uint32_t)(PAR * STAGE), lb = la + PART;
#pragma unroll
                for (int t = 0; t < 32; ++t) {               // (A, B0) | read B1 of this step
                    const int sub = t >> 4, i = (t & 15) >> 2, j = t & 3;
                    mfma(acc[i][j], bf[0][j][sub], af[PAR][i][sub]);
                    if (t % 4 == 0 && t < 16) read_b(s_cur, 1, t / 4);
                    __builtin_amdgcn_sched_barrier(0);
                }
                bts_wait_all_vmem();
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < 32; ++t) {               // (A, B1) | read A, B0 of step k+1, refill both parts
                    const int sub = t >> 4, i = (t & 15) >> 2, j = t & 3;
                    mfma(acc[i][4 + j], bf[1][j][sub], af[PAR][i][sub]);
                    if (t % 4 == 0 && t < 16) read_ah(s_nxt, PN{}, t / 4);
                    if (t % 4 == 1 && t < 16) read_b(s_nxt, 0, t / 4);
                    if (t % 4 == 2) dma_a(la, t / 4, sa_off);
                    if (t % 4 == 3) dma_b(lb, t / 4, sb_off);
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
                const uint32_t sa_off = (uint32_t)(k + 2) * a_step, sb_off = (uint32_t)(k + 2) * b_step;   // refill with step k + 2
                const uint32_t la = lds_base + (uint32_t)(par * STAGE), lb = la + PART;
                // the sixteen refill loads of this step's buffer are spread over phases 2-4 (the LDS is the
                // kernel's limit: no phase should carry more of them than another): the B part is read out
                // after phase 1, the A part after phase 2
                if (par == 0) {
                    phase(I0{}, I0{}, I0{}, I1{}, I0{}, I0{}, s_cur, la, lb, sa_off, sb_off);    // (A0,B0) | read B1 of this step
                    bts_barrier_lds();
                    phase(I0{}, I1{}, I1{}, I1{}, I0{}, I5{}, s_cur, la, lb, sa_off, sb_off);    // (A0,B1) | read A1 of this step, refill B 0-4
                    bts_wait_vmem_but5_barrier();      // step k+1 has landed for everyone; this step's A part is read out
                    phase(I1{}, I1{}, I1{}, I0{}, I5{}, I6{}, s_nxt, la, lb, sa_off, sb_off);    // (A1,B1) | read A0 of step k+1, refill B 5-7, A 0-2
                    phase(I1{}, I0{}, I0{}, I1{}, I11{}, I5{}, s_nxt, la, lb, sa_off, sb_off);   // (A1,B0) | read B1 of step k+1, refill A 3-7
                } else {
                    phase(I0{}, I1{}, I0{}, I0{}, I0{}, I0{}, s_cur, la, lb, sa_off, sb_off);    // (A0,B1) | read B0 of this step
                    bts_barrier_lds();
                    phase(I0{}, I0{}, I1{}, I1{}, I0{}, I5{}, s_cur, la, lb, sa_off, sb_off);    // (A0,B0) | read A1 of this step, refill B 0-4
                    bts_wait_vmem_but5_barrier();
                    phase(I1{}, I0{}, I1{}, I0{}, I5{}, I6{}, s_nxt, la, lb, sa_off, sb_off);    // (A1,B0) | read A0 of step k+1, refill B 5-7, A 0-2
                    phase(I1{}, I1{}, I0{}, I0{}, I11{}, I5{}, s_nxt, la, lb, sa_off, sb_off);   // (A1,B1) | read B0 of step k+1, refill A 3-7
                }
            }
        }
        bts_wait_all_vmem();    // trailing (out-of-range) refills must not land in the epilogue's LDS
    }

    // ---- epilogue.  Lane holds output row i = 16 * fi + l % 16 and, per B fragment t, the 4
    //      consecutive columns 16 t + 4 g + r.  16 rows at a time are rounded to bfloat16, parked
    //      in this wave's own 32 KB of LDS (row = 256 bytes, chunk c stored at c ^ (row & 15)) and
    //      streamed out as whole 256-byte rows.
    __syncthreads();
    uint8_t* q = smem + wave * 32768;
    const int c_rd = lane & 15;
    const int n_rd = j0 + wj0 + c_rd * 8;
    const bool interior = i0 + BI <= I && j0 + BJ <= J;
    uint16_t* orow = out + (int64_t)(i0 + wi0 + 64 * ah + (lane >> 4)) * ld_out + n_rd;
#pragma unroll
    for (int fi = 0; fi < (HALF ? 4 : 8); ++fi) {
        const int r_loc = 64 * ah + 16 * fi + r16;
        uint8_t* row = q + r_loc * 256;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const uint2 p = make_uint2(bts_pack_bf16(acc[fi][t][0], acc[fi][t][1]), bts_pack_bf16(acc[fi][t][2], acc[fi][t][3]));
            const int c = 2 * t + (g >> 1);
            *reinterpret_cast<uint2*>(row + ((c ^ r16) << 4) + (g & 1) * 8) = p;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int rr = 64 * ah + 16 * fi + 4 * it + (lane >> 4);
            const uint4 v = *reinterpret_cast<const uint4*>(q + rr * 256 + ((c_rd ^ (rr & 15)) << 4));
            uint16_t* dst = orow + (int64_t)(16 * fi + 4 * it) * ld_out;
            if (interior) {
                __builtin_nontemporal_store(v4u_tt{v.x, v.y, v.z, v.w}, reinterpret_cast<v4u_tt*>(dst));
            } else if (i0 + wi0 + rr < I && n_rd < J) {     // J % 8 == 0: a chunk is inside or outside
                __builtin_nontemporal_store(v4u_tt{v.x, v.y, v.z, v.w}, reinterpret_cast<v4u_tt*>(dst));
            }
        }
    }
}

// large problems only; the caller falls back to the register-staged kernel otherwise.
// Requires I, J multiples of 8, every byte offset of a panel below 2^31.
bool gemm_bf16_at_b_snake_fits(int64_t lda, int64_t ldb, int64_t I, int64_t J, int64_t C) {
    using namespace bts;
    const int64_t lim = (int64_t)1 << 31;
    return I % 8 == 0 && J % 8 == 0 && C > 0 && (C + 4 * BC) * lda * 2 + 2 * ROWB < lim && (C + 4 * BC) * ldb * 2 + 2 * ROWB < lim;
}

template <bool HALF>
static hipError_t bts_launch_part(const uint16_t* a, int64_t lda, const uint16_t* b, int64_t ldb, int I, int J, int C,
                                  uint16_t* out, int64_t ld_out, int tiles_i, int tiles_j, int tile_first, int64_t units,
                                  hipStream_t st) {
    using namespace bts;
    constexpr int lds = 2 * STAGE;
    static DynamicLdsOnce attr;
    if (hipError_t e = attr.ensure(reinterpret_cast<const void*>(gemm_bf16_at_b_snake_kernel<HALF>), lds); e != hipSuccess) return e;
    const int64_t grid = (units + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
    if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
    gemm_bf16_at_b_snake_kernel<HALF><<<dim3((unsigned)grid), dim3(NT), lds, st>>>(a, lda, b, ldb, I, J, C, out, ld_out, tiles_i,
                                                                              tiles_j, tile_first, (int)units);
    return hipGetLastError();
}

hipError_t launch_gemm_bf16_at_b_snake(const void* a, int64_t lda, const void* b, int64_t ldb, int64_t I, int64_t J,
                                       int64_t C, void* out, int64_t ld_out, hipStream_t st) {
    using namespace bts;
    if (I == 0 || J == 0) return hipSuccess;
    if (!gemm_bf16_at_b_snake_fits(lda, ldb, I, J, C)) return hipErrorInvalidValue;
    const int tiles_i = (int)((I + BI - 1) / BI), tiles_j = (int)((J + BJ - 1) / BJ);
    const int64_t ntiles = (int64_t)tiles_i * tiles_j;
    if (ntiles > 0x3FFFFFFF) return hipErrorInvalidValue;
    const uint16_t* ap = static_cast<const uint16_t*>(a);
    const uint16_t* bp = static_cast<const uint16_t*>(b);
    uint16_t* op = static_cast<uint16_t*>(out);
    // a last round that would fill at most half of the CUs runs as half tiles (FP8MI355_SNAKE_HALF=0: whole tiles)
    const int cus = compute_units();
    const int64_t rest = cus > 0 ? ntiles % cus : 0;
    if (knob(KNOB_SNAKE_HALF) != 0 && cus >= 16 && cus % NUM_XCD == 0 && rest > 0 && 2 * rest <= cus) {
        const int64_t full = ntiles - rest;
        if (full > 0) {
            hipError_t err = bts_launch_part<false>(ap, lda, bp, ldb, (int)I, (int)J, (int)C, op, ld_out, tiles_i, tiles_j, 0, full, st);
            if (err != hipSuccess) return err;
        }
        return bts_launch_part<true>(ap, lda, bp, ldb, (int)I, (int)J, (int)C, op, ld_out, tiles_i, tiles_j, (int)full, 2 * rest, st);
    }
    return bts_launch_part<false>(ap, lda, bp, ldb, (int)I, (int)J, (int)C, op, ld_out, tiles_i, tiles_j, 0, ntiles, st);
}

}  // namespace fp8k
