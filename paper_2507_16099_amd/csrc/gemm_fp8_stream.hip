// Scaled FP8 GEMM for gfx950, persistent form of the 16x16x128 "snake" kernel of gemm_fp8_snake.hip
// (same 256 x 256 tile, LDS layout, swizzles and four-phase K step; see there).
// out[M,N] = bfloat16( (A[M,K] . B[N,K]^T) / (sa * sb) ).
//
// What is different.  One workgroup per CU walks a list of tiles and the tile boundary disappears from the
// matrix cores' point of view:
//   * the refill slots of a tile's last two K steps fetch steps 0 and 1 of the workgroup's NEXT tile, and the
//     fragment reads of the last step pick up the next tile's first fragments: no load latency at a tile start;
//   * the epilogue is drained quadrant by quadrant INSIDE the K steps around the boundary.  A wave's accumulators
//     are four quadrants (A half x B half); quadrant q is final after its phase of the tile's last step and is
//     needed again (overwritten with C = 0) by a phase of the next tile's first step.  In between, the vector
//     ALU reads it out (v_accvgpr_read), scales it by the reciprocal scales, rounds to bfloat16 and stores it,
//     in the issue slots between the MFMAs of the phases that run meanwhile:
//         last step  (odd):  P1 (A0,B1)  P2 (A0,B0)  P3 (A1,B0) | drain (A0,B0)   P4 (A1,B1) | drain (A0,B1)
//         first step (even): P1 (A0,B0) | drain (A1,B1)   P2 (A0,B1)   P3 (A1,B1) | drain (A1,B0)   P4 (A1,B0)
//     so the stores and their write traffic overlap the next tile's products instead of idling the matrix cores;
//   * no staging through LDS: a lane holds 16 consecutive bfloat16 of one output row (32 bytes); two lane-row
//     swaps (v_permlane16_swap, v_permlane32_swap) regroup the four lanes of a row so that each store
//     instruction writes 64 contiguous bytes per row.  Stores are raw buffer stores whose descriptor ends at the
//     last valid output row; a lane whose columns lie past N gets an out-of-range offset.  Every store
//     instruction is therefore ISSUED whatever the tile, which the wait counts below rely on.
// Loads and stores share one counter (vmcnt) and complete in issue order.  A wait for "step k+1 has landed" names
// the number of operations issued after that step's last load: the five refill loads of phase 2 and, around a tile
// boundary, the stores issued since (counted exactly; their positions in the slot sequence are fixed).
//
// Tile height.  The A half of a wave is two groups of fragments, A0 (four fragments, 64 rows) and A1 (AF1 = four,
// three or two fragments): tiles of 256, 224 or 192 rows x 256 columns.  A lower tile does (4 + AF1) / 8 of the work
// of a full one in as much less time, so the launcher picks the height whose tile count fills whole rounds of
// workgroups best (the weight gradient of the benchmark, 14336 x 4096: 896 tiles of 256 rows are 3.5 rounds on 256
// CUs, 1024 tiles of 224 rows are exactly 4 rounds of 7/8 the length).
//
// Restrictions (the launcher falls back to the non-persistent kernel otherwise): bfloat16 output, N a multiple
// of 8, at least four K steps, leading dimensions below 2^23.
#include "fp8_device.hpp"
#include "launchers.hpp"
#include "tuning.hpp"

#include <type_traits>

namespace fp8k {

typedef int v4i_t2 __attribute__((ext_vector_type(4)));
typedef unsigned v4u_t2 __attribute__((ext_vector_type(4)));
typedef unsigned v2u_t2 __attribute__((ext_vector_type(2)));
typedef int v8i_t2 __attribute__((ext_vector_type(8)));
typedef float v4f_t2 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t2 __attribute__((ext_vector_type(2)));
typedef float f32x2_t2 __attribute__((ext_vector_type(2)));

namespace st {
constexpr int BM = 256, BN = 256, BK = 128;
constexpr int NT = 256;
constexpr int WM = 128, WN = 128;
constexpr int STAGE = (BM + BN) * BK;    // 64 KB
constexpr int TAB = 2048;                // reciprocal scales of one tile: 256 rows + 256 columns
constexpr int LDS_BYTES = 2 * STAGE + 2 * TAB;
constexpr int GROUP_M = 4;
constexpr int NUM_XCD = 8;
}  // namespace st

__device__ __forceinline__ uint32_t st_pack_bf16(float a, float b) {
    f32x2_t2 v = {a, b};
    bf16x2_t2 h = __builtin_convertvector(v, bf16x2_t2);
    uint32_t r;
    __builtin_memcpy(&r, &h, 4);
    return r;
}

// 16 bytes per lane from a raw buffer straight into LDS at lds_addr + lane * 16 (lds_addr wave-uniform);
// out-of-range lanes deliver zeros.  Inline assembly: the compiler must not know that these loads write LDS.
__device__ __forceinline__ void st_lds_dma16(v4i_t2 rsrc, uint32_t lds_addr, uint32_t voffset) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voffset), "s"(rsrc)
                 : "memory", "m0");
}
__device__ __forceinline__ void st_wait_all_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void st_barrier_lds() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}
// everything but the N youngest vector-memory operations has completed (they complete in issue order), own LDS reads done, barrier
// The matrix instruction as assembly with the accumulator tied to the destination (FA / FB: 0 = e4m3, 1 = e5m2; the B
// fragment is the first operand).  Through the builtin the compiler keeps the accumulation in place inside the K loop,
// but around the tile boundary - where the drain reads the accumulators a phase or two after their last update - it
// sent the last updates to other registers and copied them out right behind the instruction (a matrix-core latency
// of stall each, and 64 copies back per tile: 158 instructions more in the last two K steps).  With the accumulator
// fixed in its register the reads happen where the drain is scheduled (+0.5 %).  The compiler inserts no wait states
// for assembly: the drain schedule keeps at least two matrix instructions between an accumulator's last update and
// its first read, and between its last read and the next tile's first write.
template <int FA, int FB>
__device__ __forceinline__ void st_mfma(v4f_t2& c, const v8i_t2& b, const v8i_t2& a) {
    if constexpr (FB == 0 && FA == 0) asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0" : "+a"(c) : "v"(b), "v"(a));
    else if constexpr (FB == 1 && FA == 0) asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0 cbsz:1" : "+a"(c) : "v"(b), "v"(a));
    else if constexpr (FB == 0 && FA == 1) asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0 blgp:1" : "+a"(c) : "v"(b), "v"(a));
    else asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0 cbsz:1 blgp:1" : "+a"(c) : "v"(b), "v"(a));
}
// the same starting from C = 0 (the first K step of a tile: nothing is cleared beforehand)
template <int FA, int FB>
__device__ __forceinline__ void st_mfma_zero(v4f_t2& c, const v8i_t2& b, const v8i_t2& a) {
    if constexpr (FB == 0 && FA == 0) asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, 0" : "=a"(c) : "v"(b), "v"(a));
    else if constexpr (FB == 1 && FA == 0) asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, 0 cbsz:1" : "=a"(c) : "v"(b), "v"(a));
    else if constexpr (FB == 0 && FA == 1) asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, 0 blgp:1" : "=a"(c) : "v"(b), "v"(a));
    else asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, 0 cbsz:1 blgp:1" : "=a"(c) : "v"(b), "v"(a));
}

template <int N>
__device__ __forceinline__ void st_wait_vmem_but_barrier() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// operand panels of one tile
struct StTile {
    v4i_t2 rsrc_a, rsrc_b;
    int m0, n0;
    int valid;
};

enum { ST_FIRST = 0, ST_FIRST_DRAIN = 1, ST_MIDDLE = 2, ST_LAST = 3 };

// One accumulator-drain job: A fragment U of quadrant (A half AH, B half BH).  none(AF1): the fragment does not
// exist in a tile whose A1 group has AF1 fragments.
template <int AH_, int BH_, int U_>
struct StJob {
    static constexpr int AH = AH_, BH = BH_, U = U_;
    static constexpr bool none(int af1) { return AH == 1 && U >= af1; }
};
struct StNoJob {
    static constexpr int AH = 0, BH = 0, U = 0;
    static constexpr bool none(int) { return true; }
};
// Up to three jobs ride on the sixteen issue slots of a phase: job n takes slots 5n .. 5n+5 (its scale loads in
// slot 5n, four packing slots, swaps + its two stores in slot 5n+5, which it shares with the next job's loads).
template <class J0_, class J1_, class J2_>
struct StJobs {
    using J0 = J0_; using J1 = J1_; using J2 = J2_;
    // stores issued by the phase (two per job), and those of its slots 10 and 15 alone
    static constexpr int stores(int af1) { return 2 * ((J0::none(af1) ? 0 : 1) + (J1::none(af1) ? 0 : 1) + (J2::none(af1) ? 0 : 1)); }
    static constexpr int late_stores(int af1) { return 2 * ((J1::none(af1) ? 0 : 1) + (J2::none(af1) ? 0 : 1)); }
};
using StNoJobs = StJobs<StNoJob, StNoJob, StNoJob>;
// The schedule around a tile boundary (L = last step of a tile, odd; F = first step of the next, even).  A quadrant
// is final after the phase that last adds to it and must be gone before the phase of F that restarts it:
//   (A0,B1) final after L.P1, restarted by F.P2      (A0,B0) final after L.P2, restarted by F.P1
//   (A1,B0) final after L.P3, restarted by F.P4      (A1,B1) final after L.P4, restarted by F.P3
using StJobsL2 = StJobs<StJob<0, 1, 0>, StJob<0, 1, 1>, StJob<0, 1, 2>>;
using StJobsL3 = StJobs<StJob<0, 1, 3>, StJob<0, 0, 0>, StJob<0, 0, 1>>;
using StJobsL4 = StJobs<StJob<0, 0, 2>, StJob<0, 0, 3>, StJob<1, 0, 0>>;
using StJobsF1 = StJobs<StJob<1, 1, 0>, StJob<1, 1, 1>, StJob<1, 0, 1>>;
using StJobsF2 = StJobs<StJob<1, 1, 2>, StJob<1, 1, 3>, StJob<1, 0, 2>>;
using StJobsF3 = StJobs<StJob<1, 0, 3>, StNoJob, StNoJob>;
// Vector-memory operations issued after the last refill load of a step's phase 4 (slot 9 at the latest) and before
// the wait in the middle of the next step, beyond the five refill loads of that step's phase 2:
//   wait of L: the stores of L.P2;
//   wait of F (behind a drained tile): the stores of L.P4's slots 10 and 15, those of F.P1 and of F.P2.
constexpr int st_extra_l(int af1) { return StJobsL2::stores(af1); }
constexpr int st_extra_f(int af1) { return StJobsL4::late_stores(af1) + StJobsF1::stores(af1) + StJobsF2::stores(af1); }

template <int FA, int FB, int AF1>
__global__ __launch_bounds__(st::NT) void gemm_fp8_stream_kernel(
    const uint8_t* __restrict__ A, int64_t lda, const uint8_t* __restrict__ B, int64_t ldb,
    const float* __restrict__ scale_a, int row_a, const float* __restrict__ scale_b, int row_b, int M, int N,
    int K, uint16_t* __restrict__ out, int64_t ld_out, int tiles_m, int tiles_n, int units) {
    using namespace st;
    static_assert(AF1 >= 2 && AF1 <= 4, "the A1 group has two to four fragments");
    constexpr int TM = 32 * (4 + AF1);     // tile height: 256, 224 or 192 rows (the LDS layout keeps room for 256)
    constexpr int NLA = TM / 32;           // LDS-DMA loads of the A part per wave and K step
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // ---- this workgroup's tiles.  Workgroup ids are dealt round-robin to the 8 XCDs; each XCD owns a contiguous
    //      range of tiles (walked in groups of tile rows) and its workgroups take them round by round, so the tiles
    //      in flight on an XCD form a patch that shares operand panels in that L2.
    const int slots = gridDim.x / NUM_XCD;
    const int xcd = blockIdx.x % NUM_XCD, slot = blockIdx.x / NUM_XCD;
    const int per_xcd = (units + NUM_XCD - 1) / NUM_XCD;
    const int u_first = xcd * per_xcd + slot;
    const int u_end = (xcd + 1) * per_xcd < units ? (xcd + 1) * per_xcd : units;
    if (u_first >= u_end) return;
    const int my_tiles = (u_end - u_first + slots - 1) / slots;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave >> 1) * (TM / 2), wn0 = (wave & 1) * WN;

    auto tile_of = [&](int j) {
        StTile t;
        const int unit = u_first + j * slots;
        t.valid = (j < my_tiles) ? 1 : 0;
        const int logical = t.valid ? unit : u_first;          // a missing tile aliases a valid one (its loads are forced out of range)
        const int in_group = GROUP_M * tiles_n;
        const int first_m = (logical / in_group) * GROUP_M;
        const int gsize = tiles_m - first_m < GROUP_M ? tiles_m - first_m : GROUP_M;
        const int tm = first_m + (logical % in_group) % gsize;
        const int tn = (logical % in_group) / gsize;
        t.m0 = tm * TM;
        t.n0 = tn * BN;
        const int rows_a = M - t.m0 < TM ? M - t.m0 : TM, rows_b = N - t.n0 < BN ? N - t.n0 : BN;
        const uint64_t pa = reinterpret_cast<uint64_t>(A + (int64_t)t.m0 * lda);
        const uint64_t pb = reinterpret_cast<uint64_t>(B + (int64_t)t.n0 * ldb);
        t.rsrc_a = v4i_t2{(int)(uint32_t)pa, (int)(uint32_t)(pa >> 32), (int)((int64_t)(rows_a - 1) * lda + K), 0x00020000};
        t.rsrc_b = v4i_t2{(int)(uint32_t)pb, (int)(uint32_t)(pb >> 32), (int)((int64_t)(rows_b - 1) * ldb + K), 0x00020000};
        return t;
    };

    // ---- global -> LDS (as in the non-persistent kernel): wave w fills row groups w, w+4, ... (8 rows each) of both
    //      tiles; lane l fills (row l/8, chunk slot l%8) with logical chunk slot ^ key(row).  The A part has TM rows:
    //      NLA loads per wave (rows past TM are never read: the wave halves start at TM / 2).
    const int lrow = lane >> 3;
    const int ca = (lane & 7) ^ ((4 * (wave & 1) + (lrow >> 1)) & 7);
    const int cb_e = (lane & 7) ^ (((lrow >> 1) & 1) | (((wave >> 1) & 3) << 1));
    const int cb_o = (lane & 7) ^ (((lrow >> 1) & 1) | (((2 + (wave >> 1)) & 3) << 1));
    const uint32_t va0 = (uint32_t)((wave * 8 + lrow) * (int)lda + ca * 16);
    const uint32_t vb0_e = (uint32_t)((wave * 8 + lrow) * (int)ldb + cb_e * 16);
    const uint32_t vb0_o = (uint32_t)((wave * 8 + lrow) * (int)ldb + cb_o * 16);
    const uint32_t va_step = (uint32_t)(32 * (int)lda), vb_step = (uint32_t)(32 * (int)ldb);
    const uint32_t lds_base = (uint32_t)(size_t)smem + (uint32_t)wave * 1024u;
    constexpr uint32_t OOB = 0x80000000u;   // no valid offset reaches 2^31: adding it puts a lane outside its descriptor

    // byte offsets of a K position in the three lane classes, forced out of range past K or for a missing tile
    struct KOff { uint32_t a, e, o; };
    auto koff = [&](int k0, int valid) {
        KOff r;
        r.a = (valid && k0 + ca * 16 < K) ? (uint32_t)k0 : OOB;
        r.e = (valid && k0 + cb_e * 16 < K) ? (uint32_t)k0 : OOB;
        r.o = (valid && k0 + cb_o * 16 < K) ? (uint32_t)k0 : OOB;
        return r;
    };
    auto issue_loads = [&](const StTile& t, int stage, int k0) {
        const KOff ko = koff(k0, t.valid);
        const uint32_t la = lds_base + (uint32_t)(stage * STAGE), lb = la + BM * BK;
#pragma unroll
        for (int i = 0; i < NLA; ++i) st_lds_dma16(t.rsrc_a, la + i * 4096, va0 + (uint32_t)i * va_step + ko.a);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            st_lds_dma16(t.rsrc_b, lb + i * 4096, ((i & 1) ? vb0_o + ko.o : vb0_e + ko.e) + (uint32_t)i * vb_step);
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
    v8i_t2 af[2][4], bf[2][4];   // [half][fragment in half]
    auto read_a = [&](const uint8_t* s, int half, int f) {
        const int row_off = (half * 4 + f) * 16 * BK;
        const uint4 x0 = *reinterpret_cast<const uint4*>(s + offa[0] + row_off);
        const uint4 x1 = *reinterpret_cast<const uint4*>(s + offa[1] + row_off);
        af[half][f] = v8i_t2{(int)x0.x, (int)x0.y, (int)x0.z, (int)x0.w, (int)x1.x, (int)x1.y, (int)x1.z, (int)x1.w};
    };
    auto read_b = [&](const uint8_t* s, int half, int f) {
        const int row_off = (half * 64 + f * 4) * BK;
        const uint4 x0 = *reinterpret_cast<const uint4*>(s + offb[0] + row_off);
        const uint4 x1 = *reinterpret_cast<const uint4*>(s + offb[1] + row_off);
        bf[half][f] = v8i_t2{(int)x0.x, (int)x0.y, (int)x0.z, (int)x0.w, (int)x1.x, (int)x1.y, (int)x1.z, (int)x1.w};
    };

    v4f_t2 acc[8][8];   // [A fragment][B fragment]

    // ---- drain.  Lane (g, r16) holds, per A fragment fi, output row 16 fi + r16 of the wave's quadrant and, per B
    //      half, the 16 consecutive columns 64 BH + 16 g + x, x = 4 t + r (B fragment t, accumulator register r).
    //      The output of a tile is addressed through a raw buffer that starts at the tile's first element and ends
    //      with the last valid output row: rows past M are dropped by the bounds check.
    struct Drain {
        __amdgpu_buffer_rsrc_t rsrc;   // output window of the tile
        const float* tab;   // reciprocal scales of that tile: [0,256) rows, [256,512) columns
        int n_left;         // N - n0: columns of the tile that exist
    };
    const uint32_t lane_out = (uint32_t)(((wm0 + r16) * (int)ld_out + wn0 + 8 * g) * 2);   // byte offset of this lane's first piece in a tile
    const int lane_col = wn0 + 8 * g;
    float inv_b[4][4], inv_a = 0.f;     // the job's sixteen column scales and its row scale
    uint32_t pk[8];
    // step S of a job: 0 = fetch its row scale and first column scales; 1..4 = read four accumulators (one B fragment),
    // scale, round, pack, and fetch the next fragment's column scales; 5 = regroup and store
    auto job_step = [&](auto job_t, auto step_t, const Drain& d) {
        using J = decltype(job_t);
        constexpr int S = decltype(step_t)::value;
        if constexpr (!J::none(AF1)) {
            constexpr int AH = J::AH, BH = J::BH, U = J::U;
            if constexpr (S == 0) {
                // all of the job's scales in one go (one wait for LDS per job instead of five; measured neutral)
                inv_a = d.tab[wm0 + 16 * (AH * 4 + U) + r16];
#pragma unroll
                for (int T = 0; T < 4; ++T) {
                    const float4 t4 = *reinterpret_cast<const float4*>(d.tab + 256 + wn0 + 64 * BH + 16 * g + 4 * T);
                    inv_b[T][0] = t4.x; inv_b[T][1] = t4.y; inv_b[T][2] = t4.z; inv_b[T][3] = t4.w;
                }
            } else if constexpr (S <= 4) {
                constexpr int T = S - 1;                                   // B fragment of the half
                const v4f_t2 v = acc[AH * 4 + U][BH * 4 + T];
                pk[2 * T] = st_pack_bf16((v[0] * inv_a) * inv_b[T][0], (v[1] * inv_a) * inv_b[T][1]);
                pk[2 * T + 1] = st_pack_bf16((v[2] * inv_a) * inv_b[T][2], (v[3] * inv_a) * inv_b[T][3]);
            } else {
                // lanes g = 0..3 of a row hold the 16-byte pieces (2g, 2g+1) of its 128 bytes; after the two swaps
                // lane g holds pieces g (lo) and 4 + g (hi): each store writes 64 contiguous bytes per row
                uint32_t lo[4], hi[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const v2u_t2 s1 = __builtin_amdgcn_permlane16_swap(pk[e], pk[4 + e], false, false);
                    const v2u_t2 s2 = __builtin_amdgcn_permlane32_swap(s1[0], s1[1], false, false);
                    lo[e] = s2[0]; hi[e] = s2[1];
                }
                // (offsets formed here, from values the optimizer cannot see through: hoisted out of the tile loop,
                //  the sixteen jobs' offsets would be sixteen more live registers)
                uint32_t lo_base = lane_out;
                int ld32 = (int)ld_out;
                asm volatile("" : "+v"(lo_base), "+s"(ld32));
                const uint32_t off = lo_base + (uint32_t)((16 * (AH * 4 + U) * ld32 + 64 * BH) * 2);
                const uint32_t off_lo = lane_col + 64 * BH < d.n_left ? off : OOB;
                const uint32_t off_hi = lane_col + 64 * BH + 32 < d.n_left ? off + 64u : OOB;
                __builtin_amdgcn_raw_buffer_store_b128(v4u_t2{lo[0], lo[1], lo[2], lo[3]}, d.rsrc, (int)off_lo, 0, 2);   // 2: non-temporal
                __builtin_amdgcn_raw_buffer_store_b128(v4u_t2{hi[0], hi[1], hi[2], hi[3]}, d.rsrc, (int)off_hi, 0, 2);
            }
        }
    };
    // slot t of a phase carrying the jobs JS
    auto jobs_slot = [&](auto jobs_t, auto slot_t, const Drain& d) {
        using JS = decltype(jobs_t);
        constexpr int T = decltype(slot_t)::value;
        if constexpr (T <= 5) job_step(typename JS::J0{}, std::integral_constant<int, T>{}, d);
        if constexpr (T >= 5 && T <= 10) job_step(typename JS::J1{}, std::integral_constant<int, T - 5>{}, d);
        if constexpr (T >= 10) job_step(typename JS::J2{}, std::integral_constant<int, T - 10>{}, d);
    };

    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I5 = std::integral_constant<int, 5>;
    using I6 = std::integral_constant<int, 6>;
    using I11 = std::integral_constant<int, 11>;

    // one phase: 16 MFMAs of A half AH x B half BH (ZERO: starting from C = 0); in its slots, optionally the reads of
    // one fragment half (RDA: 1 = A half RH, 0 = B half RH) from stage `rs`, CNT of the step's sixteen LDS-DMA refill
    // loads from number L0 on (0-7: the B part, 8-15: the A part) out of tile `lt` at K offsets `ko`, and the drain
    // jobs JS of the tile described by `dr`.  Order inside a slot: MFMA, fragment reads, refill load, drain work.
    auto phase = [&](auto ah_t, auto bh_t, auto rda_t, auto rh_t, auto l0_t, auto cnt_t, auto zero_t, auto jobs_t, const uint8_t* rs,
                     uint32_t la, uint32_t lb, const StTile& lt, const KOff& ko, const Drain& dr) {
        constexpr int AH = decltype(ah_t)::value, BH = decltype(bh_t)::value, RDA = decltype(rda_t)::value,
                      RH = decltype(rh_t)::value, L0 = decltype(l0_t)::value, CNT = decltype(cnt_t)::value,
                      ZERO = decltype(zero_t)::value;
        using JS = decltype(jobs_t);
        constexpr bool DRAINS = JS::stores(AF1) > 0;
        [&]<int... TS>(std::integer_sequence<int, TS...>) {
            ([&] {
                constexpr int t = TS;
                constexpr int i = t >> 2, j = (i & 1) ? 3 - (t & 3) : (t & 3);   // boustrophedon: one operand stays between neighbours
                if constexpr (AH == 0 || i < AF1) {        // (a lower tile has no fragment i of the A1 group: the slot stays empty)
                    if constexpr (ZERO) st_mfma_zero<FA, FB>(acc[AH * 4 + i][BH * 4 + j], bf[BH][j], af[AH][i]);
                    else st_mfma<FA, FB>(acc[AH * 4 + i][BH * 4 + j], bf[BH][j], af[AH][i]);
                }
                if constexpr (RDA == 1 && t % 2 == 0 && t < 8 && (RH == 0 || t / 2 < AF1)) read_a(rs, RH, t / 2);
                if constexpr (RDA == 0 && t % 2 == 0 && t < 8) read_b(rs, RH, t / 2);
                if constexpr (t % 2 == 1 && t / 2 < CNT) {
                    constexpr int q = L0 + t / 2;
                    if constexpr (q < 8) st_lds_dma16(lt.rsrc_b, lb + q * 4096, ((q & 1) ? vb0_o + ko.o : vb0_e + ko.e) + (uint32_t)q * vb_step);
                    else if constexpr (q - 8 < NLA) st_lds_dma16(lt.rsrc_a, la + (q - 8) * 4096, va0 + (uint32_t)(q - 8) * va_step + ko.a);
                }
                if constexpr (DRAINS) {
                    __builtin_amdgcn_sched_barrier(0);     // the slot's refill load is issued before its stores (the wait counts rely on it)
                    jobs_slot(JS{}, std::integral_constant<int, t>{}, dr);
                }
                __builtin_amdgcn_sched_barrier(0);
            }(), ...);
        }(std::make_integer_sequence<int, 16>{});
    };

    const int ksteps = (K + BK - 1) / BK;
    const int kpairs = (ksteps + 1) / 2;        // >= 2 (checked by the launcher); an odd count gets one phantom step of zeros
    const int nsteps = 2 * kpairs;

    // reciprocal scales of a tile, one row and one column per thread (correctly rounded divides); the raw scales are
    // fetched by assembly loads so that the compiler's own wait counters never see them (a compiler-placed wait would
    // also wait for the LDS-DMA loads in flight)
    float raw_a = 1.f, raw_b = 1.f;
    auto scale_loads = [&](const StTile& t) {
        const int m = t.m0 + (int)threadIdx.x, n = t.n0 + (int)threadIdx.x;
        const float* pa = scale_a + (row_a ? (m < M ? m : M - 1) : 0);
        const float* pb = scale_b + (row_b ? (n < N ? n : N - 1) : 0);
        asm volatile("global_load_dword %0, %2, off\n\tglobal_load_dword %1, %3, off"
                     : "=&v"(raw_a), "=&v"(raw_b)
                     : "v"(pa), "v"(pb)
                     : "memory");
    };
    auto scale_table = [&](float* tab) {
        // (the loads were issued ahead of a phase 3's refill loads and a wait that lets only younger operations stay in flight has passed)
        asm volatile("" : "+v"(raw_a), "+v"(raw_b));
        tab[threadIdx.x] = 1.0f / raw_a;
        tab[256 + threadIdx.x] = 1.0f / raw_b;
    };
    float* const tab0 = reinterpret_cast<float*>(smem + 2 * STAGE);

    auto drain_of = [&](int m0, int n0, int j) {
        Drain d;
        const int rows = M - m0 < TM ? M - m0 : TM;
        d.n_left = N - n0;
        const int cols = d.n_left < BN ? d.n_left : BN;
        d.rsrc = __builtin_amdgcn_make_buffer_rsrc(out + (int64_t)m0 * ld_out + n0, 0, (int)(((int64_t)(rows - 1) * ld_out + cols) * 2), 0x00020000);
        d.tab = tab0 + (j & 1) * (TAB / 4);
        return d;
    };

    // a pair of K steps (the B halves swap roles every step).  KIND: ST_FIRST(_DRAIN) = steps 0, 1 of a tile (step 0
    // starts the accumulators from zero; with _DRAIN the rest of the previous tile leaves in its phases 1-3; the scale
    // loads of this tile go out in step 0, its table is written in step 1), ST_MIDDLE, ST_LAST = the last two steps
    // (refills fetch steps 0, 1 of tile `lt` = the next tile; the drain of this tile starts in phase 2 of the last step).
    auto pair = [&](auto kind_t, const StTile& cur, const StTile& lt, int k2_even, const Drain& dprev, const Drain& dcur, float* tab_cur) {
        constexpr int KIND = decltype(kind_t)::value;
        constexpr bool FIRST = KIND == ST_FIRST || KIND == ST_FIRST_DRAIN;
        constexpr bool FD = KIND == ST_FIRST_DRAIN, LD = KIND == ST_LAST;
        using Z = std::integral_constant<int, FIRST ? 1 : 0>;
        using NJ = StNoJobs;
        {
            // even step: B order 0,1,1,0.  Holds A0, B0 of this step.
            const uint8_t* s_cur = smem;
            const uint8_t* s_nxt = smem + STAGE;
            const KOff ko = koff(k2_even, lt.valid);
            const uint32_t la = lds_base, lb = la + BM * BK;
            phase(I0{}, I0{}, I0{}, I1{}, I0{}, I0{}, Z{}, std::conditional_t<FD, StJobsF1, NJ>{}, s_cur, la, lb, lt, ko, dprev);   // (A0,B0) | read B1 of this step
            st_barrier_lds();                  // this step's B part is read out by everyone
            phase(I0{}, I1{}, I1{}, I1{}, I0{}, I5{}, Z{}, std::conditional_t<FD, StJobsF2, NJ>{}, s_cur, la, lb, lt, ko, dprev);   // (A0,B1) | read A1 of this step, refill B 0-4
            st_wait_vmem_but_barrier<5 + (FD ? st_extra_f(AF1) : 0)>();   // step k+1 has landed for everyone; this step's A part is read out
            if constexpr (FIRST) scale_loads(cur);   // older than the refill loads below: complete at the next such wait
            phase(I1{}, I1{}, I1{}, I0{}, I5{}, I6{}, Z{}, std::conditional_t<FD, StJobsF3, NJ>{}, s_nxt, la, lb, lt, ko, dprev);   // (A1,B1) | read A0 of step k+1, refill B 5-7, A 0-2
            phase(I1{}, I0{}, I0{}, I1{}, I11{}, I5{}, Z{}, NJ{}, s_nxt, la, lb, lt, ko, dprev);                                    // (A1,B0) | read B1 of step k+1, refill A 3-7
        }
        {
            // odd step: B order 1,0,0,1.  Holds A0, B1 of this step.
            const uint8_t* s_cur = smem + STAGE;
            const uint8_t* s_nxt = smem;
            const KOff ko = koff(k2_even + BK, lt.valid);
            const uint32_t la = lds_base + (uint32_t)STAGE, lb = la + BM * BK;
            phase(I0{}, I1{}, I0{}, I0{}, I0{}, I0{}, I0{}, NJ{}, s_cur, la, lb, lt, ko, dcur);                                     // (A0,B1) | read B0 of this step
            st_barrier_lds();
            phase(I0{}, I0{}, I1{}, I1{}, I0{}, I5{}, I0{}, std::conditional_t<LD, StJobsL2, NJ>{}, s_cur, la, lb, lt, ko, dcur);   // (A0,B0) | read A1 of this step, refill B 0-4
            st_wait_vmem_but_barrier<5 + (LD ? st_extra_l(AF1) : 0)>();
            if constexpr (FIRST) scale_table(tab_cur);
            phase(I1{}, I0{}, I1{}, I0{}, I5{}, I6{}, I0{}, std::conditional_t<LD, StJobsL3, NJ>{}, s_nxt, la, lb, lt, ko, dcur);   // (A1,B0) | read A0 of step k+1, refill B 5-7, A 0-2
            phase(I1{}, I1{}, I0{}, I0{}, I11{}, I5{}, I0{}, std::conditional_t<LD, StJobsL4, NJ>{}, s_nxt, la, lb, lt, ko, dcur);  // (A1,B1) | read B0 of step k+1, refill A 3-7
        }
    };

    // ---- first tile: both stages in flight at once, then the first fragments
    StTile cur = tile_of(0);
    issue_loads(cur, 0, 0);
    issue_loads(cur, 1, BK);
    st_wait_all_vmem();
    __syncthreads();
#pragma unroll
    for (int f = 0; f < 4; ++f) {
        read_a(smem, 0, f);
        read_b(smem, 0, f);
    }
    __builtin_amdgcn_sched_barrier(0);

    int pm0 = cur.m0, pn0 = cur.n0;
    for (int j = 0; j < my_tiles; ++j) {
        float* tab_cur = tab0 + (j & 1) * (TAB / 4);
        {
            const Drain dprev = drain_of(pm0, pn0, j - 1);
            if (j == 0) pair(std::integral_constant<int, ST_FIRST>{}, cur, cur, 2 * BK, dprev, dprev, tab_cur);
            else pair(std::integral_constant<int, ST_FIRST_DRAIN>{}, cur, cur, 2 * BK, dprev, dprev, tab_cur);
        }
        for (int kp = 1; kp < kpairs - 1; ++kp) {
            const Drain none = drain_of(cur.m0, cur.n0, j);
            pair(std::integral_constant<int, ST_MIDDLE>{}, cur, cur, (2 * kp + 2) * BK, none, none, tab_cur);
        }
        const StTile nxt = tile_of(j + 1);
        {
            const Drain dcur = drain_of(cur.m0, cur.n0, j);
            pair(std::integral_constant<int, ST_LAST>{}, cur, nxt, 0, dcur, dcur, tab_cur);
        }
        pm0 = cur.m0; pn0 = cur.n0;
        cur = nxt;
    }
    st_wait_all_vmem();    // the trailing refills (all out of range) have landed

    // ---- what is left of the last tile: the jobs that the next tile's first step would have carried
    {
        const Drain dlast = drain_of(pm0, pn0, my_tiles - 1);
        [&]<int... TS>(std::integer_sequence<int, TS...>) {
            (jobs_slot(StJobsF1{}, std::integral_constant<int, TS>{}, dlast), ...);
            (jobs_slot(StJobsF2{}, std::integral_constant<int, TS>{}, dlast), ...);
            (jobs_slot(StJobsF3{}, std::integral_constant<int, TS>{}, dlast), ...);
        }(std::make_integer_sequence<int, 16>{});
    }
}

template <int FA, int FB, int AF1>
static hipError_t launch_stream_t(const uint8_t* a, int64_t lda, const float* sa, int row_a, const uint8_t* b, int64_t ldb,
                                  const float* sb, int row_b, int M, int N, int K, void* out, int64_t ld_out, int tiles_m,
                                  int tiles_n, int64_t units, hipStream_t st) {
    using namespace st;
    auto kern = gemm_fp8_stream_kernel<FA, FB, AF1>;
    static DynamicLdsOnce attr;
    if (hipError_t e = attr.ensure(reinterpret_cast<const void*>(kern), LDS_BYTES); e != hipSuccess) return e;
    // one workgroup per CU (they do not fit twice), a multiple of the XCD count; the switch GEMM_STREAM >= 8 sets
    // the number of workgroups instead (test aid: few workgroups walk many tiles each, also on small problems)
    int cus = compute_units();
    if (const int forced = knob(KNOB_GEMM_STREAM); forced >= NUM_XCD) cus = forced;
    if (cus < NUM_XCD) cus = NUM_XCD;
    int64_t grid = cus / NUM_XCD * NUM_XCD;
    const int64_t need = (units + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
    if (grid > need) grid = need;
    kern<<<dim3((unsigned)grid), dim3(NT), LDS_BYTES, st>>>(a, lda, b, ldb, sa, row_a, sb, row_b, M, N, K,
                                                           static_cast<uint16_t*>(out), ld_out, tiles_m, tiles_n, (int)units);
    return hipGetLastError();
}

bool gemm_fp8_stream_fits(int64_t lda, int64_t ldb, int64_t ld_out, int64_t N, int64_t K, int out_f32, int act) {
    return !out_f32 && !act && N % 8 == 0 && K > 2 * st::BK && lda < (1 << 23) && ldb < (1 << 23) && ld_out < (1 << 22);
}

// Tile height (256, 224 or 192 rows) for an [M, N] output when the persistent kernel takes every tile: the one
// with the least rounds x height on this device's CUs; 256 when it is no worse (a lower tile moves more operand
// bytes per product).  The switch GEMM_TILE_M forces one.
int gemm_fp8_stream_tile_m(int64_t M, int64_t N) {
    const int forced = knob(KNOB_GEMM_TILE_M);
    if (forced == 256 || forced == 224 || forced == 192) return forced;
    const int64_t cus = compute_units() > 0 ? compute_units() : 256;
    const int64_t tiles_n = (N + st::BN - 1) / st::BN;
    int best = 256;
    int64_t best_cost = 0;
    for (int tm : {256, 224, 192}) {
        const int64_t tiles = (M + tm - 1) / tm * tiles_n;
        const int64_t cost = (tiles + cus - 1) / cus * tm;
        if (tm == 256 || cost < best_cost) { best = tm; best_cost = cost; }
    }
    return best;
}

// tiles [0, units) of the tile order of the non-persistent kernel (tile_m == 256), or every tile of the problem cut
// into tiles of tile_m rows (units == the tile count)
hipError_t launch_gemm_fp8_stream(const uint8_t* a, int64_t lda, int fmt_a, const float* scale_a, int row_a,
                                  const uint8_t* b, int64_t ldb, int fmt_b, const float* scale_b, int row_b,
                                  int64_t M, int64_t N, int64_t K, void* out, int64_t ld_out, int64_t units, int tile_m,
                                  hipStream_t st) {
    using namespace st;
    if (units <= 0) return hipSuccess;
    if (tile_m != 256 && tile_m != 224 && tile_m != 192) return hipErrorInvalidValue;
    const int tiles_m = (int)((M + tile_m - 1) / tile_m), tiles_n = (int)((N + BN - 1) / BN);
    if (units > (int64_t)tiles_m * tiles_n || units > 0x3FFFFFFF) return hipErrorInvalidValue;
    const int m = (int)M, n = (int)N, k = (int)K;
#define FP8K_STREAM(FA_, FB_)                                                                                   \
    if (fmt_a == FA_ && fmt_b == FB_) {                                                                         \
        if (tile_m == 256) return launch_stream_t<FA_, FB_, 4>(a, lda, scale_a, row_a, b, ldb, scale_b, row_b, m, n, k, out, ld_out, tiles_m, tiles_n, units, st); \
        if (tile_m == 224) return launch_stream_t<FA_, FB_, 3>(a, lda, scale_a, row_a, b, ldb, scale_b, row_b, m, n, k, out, ld_out, tiles_m, tiles_n, units, st); \
        return launch_stream_t<FA_, FB_, 2>(a, lda, scale_a, row_a, b, ldb, scale_b, row_b, m, n, k, out, ld_out, tiles_m, tiles_n, units, st); \
    }
    FP8K_STREAM(FMT_E4M3FN, FMT_E4M3FN)
    FP8K_STREAM(FMT_E5M2, FMT_E4M3FN)
    FP8K_STREAM(FMT_E4M3FN, FMT_E5M2)
    FP8K_STREAM(FMT_E5M2, FMT_E5M2)
#undef FP8K_STREAM
    return hipErrorInvalidValue;
}

}  // namespace fp8k
