// Device-side helpers shared by the quantization kernels (gfx950 only).
//
// Numerics (paper Section 2.1: dynamic cast to FP8; the formats are the OCP
// OFP8 E4M3 "fn" and E5M2 encodings, which is what the gfx950 conversion and
// matrix instructions implement):
//   amax    - compared on the 15 magnitude bits of bfloat16 as unsigned
//             integers (same order as the absolute values, exact);
//   scale   - FMAX / max(amax, 1e-12) in binary64, rounded once to binary32,
//             optionally truncated to a power of two;
//   cast    - binary32 product x*s (one rounding), clamp to +-FMAX, then the
//             hardware round-to-nearest-even conversion v_cvt_pk_{fp8,bf8}_f32.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fp8k {

constexpr int FMT_E4M3FN = 0;
constexpr int FMT_E5M2 = 1;
constexpr int GRAN_TENSOR = 0;
constexpr int GRAN_ROW = 1;
constexpr int GRAN_COL = 2;
constexpr int FLAG_POW2 = 1;

typedef unsigned short u16x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float fmt_max(int fmt) { return fmt == FMT_E4M3FN ? 448.0f : 57344.0f; }

// 128-bit / 64-bit accesses with the streaming (non-temporal) hint, for data that
// this kernel touches once: measured 6-12 % faster than plain accesses on the
// casts, and it keeps such data from displacing what later kernels re-read
typedef unsigned v4u_t __attribute__((ext_vector_type(4)));
typedef unsigned v2u_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 load_stream(const void* p) {
    const v4u_t t = __builtin_nontemporal_load(static_cast<const v4u_t*>(p));
    return make_uint4(t[0], t[1], t[2], t[3]);
}
__device__ __forceinline__ void store_stream(void* p, const uint4& v) {
    __builtin_nontemporal_store(v4u_t{v.x, v.y, v.z, v.w}, static_cast<v4u_t*>(p));
}
__device__ __forceinline__ void store_stream(void* p, const uint2& v) {
    __builtin_nontemporal_store(v2u_t{v.x, v.y}, static_cast<v2u_t*>(p));
}

// two bfloat16 packed in a dword -> two binary32 (exact widening)
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// running maximum of the magnitude bits of packed bfloat16 pairs
__device__ __forceinline__ uint32_t pk_absmax(uint32_t acc, uint32_t w) {
    w &= 0x7FFF7FFFu;
    u16x2_t a, b;
    __builtin_memcpy(&a, &acc, 4);
    __builtin_memcpy(&b, &w, 4);
    a = __builtin_elementwise_max(a, b);
    __builtin_memcpy(&acc, &a, 4);
    return acc;
}
__device__ __forceinline__ uint32_t pk_absmax4(uint32_t acc, const uint4& v) {
    acc = pk_absmax(acc, v.x);
    acc = pk_absmax(acc, v.y);
    acc = pk_absmax(acc, v.z);
    return pk_absmax(acc, v.w);
}
// fold the two 16-bit halves: result is the 15-bit magnitude of the maximum
__device__ __forceinline__ uint32_t pk_fold(uint32_t acc) {
    const uint32_t lo = acc & 0xFFFFu, hi = acc >> 16;
    return lo > hi ? lo : hi;
}
__device__ __forceinline__ float mag_to_float(uint32_t mag15) { return __uint_as_float(mag15 << 16); }

// pk_absmax of a register with the same register of the lane OFF away (lane ^ OFF), without a trip through the
// LDS crossbar: neighbours within a quad by DPP quad permutation, 8 away by a DPP rotation of the row of 16,
// 16 and 32 away by the row swaps (v_permlane16_swap / v_permlane32_swap of a register with itself leave, in
// every lane, the lane's own value in one result and its partner's in the other).
template <int OFF>
__device__ __forceinline__ uint32_t pk_absmax_xor(uint32_t v) {
    static_assert(OFF == 1 || OFF == 2 || OFF == 8 || OFF == 16 || OFF == 32, "no register-to-register form for this distance");
    if constexpr (OFF == 1) return pk_absmax(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false));        // quad_perm:[1,0,3,2]
    else if constexpr (OFF == 2) return pk_absmax(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false));   // quad_perm:[2,3,0,1]
    else if constexpr (OFF == 8) return pk_absmax(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x128, 0xF, 0xF, false));  // row_ror:8
    else if constexpr (OFF == 16) {
        const auto s = __builtin_amdgcn_permlane16_swap(v, v, false, false);
        return pk_absmax(s[0] & 0x7FFF7FFFu, s[1]);
    } else {
        const auto s = __builtin_amdgcn_permlane32_swap(v, v, false, false);
        return pk_absmax(s[0] & 0x7FFF7FFFu, s[1]);
    }
}

// maximum over the lanes of a (sub)wavefront of WIDTH lanes (power of two <= 64), the same value in all of them.
// Groups of 16 lanes fold by DPP rotations within their row (register-to-register: four dependent VALU
// operations instead of four round trips through the LDS crossbar); a whole wavefront then combines its
// four rows through scalar registers.
template <int WIDTH>
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
    if constexpr (WIDTH == 16 || WIDTH == 64) {
        uint32_t o;
        o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x121, 0xF, 0xF, false);   // row_ror:1
        v = o > v ? o : v;
        o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x122, 0xF, 0xF, false);   // row_ror:2
        v = o > v ? o : v;
        o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x124, 0xF, 0xF, false);   // row_ror:4
        v = o > v ? o : v;
        o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x128, 0xF, 0xF, false);   // row_ror:8
        v = o > v ? o : v;
        if constexpr (WIDTH == 64) {
            const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)v, 0), b = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
            const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)v, 32), d = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
            const uint32_t ab = a > b ? a : b, cd = c > d ? c : d;
            v = ab > cd ? ab : cd;
        }
        return v;
    } else {
#pragma unroll
        for (int off = WIDTH / 2; off > 0; off >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)v, off, 64);
            v = o > v ? o : v;
        }
        return v;
    }
}

// scale from amax: binary64 quotient rounded once to binary32
__device__ __forceinline__ float scale_from_amax(float amax, int fmt, int flags) {
    double a = (double)amax;
    if (!(a > 1e-12)) a = 1e-12;
    float s = (float)((double)fmt_max(fmt) / a);
    if (flags & FLAG_POW2) s = __uint_as_float(__float_as_uint(s) & 0xFF800000u);
    return s;
}

// clamp to the finite range; NaN stays NaN
template <int FMT>
__device__ __forceinline__ float sat(float v) {
    constexpr float F = FMT == FMT_E4M3FN ? 448.0f : 57344.0f;
    const float c = __builtin_amdgcn_fmed3f(v, -F, F);
    return v != v ? v : c;
}

// two binary32 -> two fp8 codes in the low 16 bits
template <int FMT>
__device__ __forceinline__ uint32_t cvt2(float a, float b) {
    if constexpr (FMT == FMT_E4M3FN)
        return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(sat<FMT>(a), sat<FMT>(b), 0, false) & 0xFFFFu;
    else
        return (uint32_t)__builtin_amdgcn_cvt_pk_bf8_f32(sat<FMT>(a), sat<FMT>(b), 0, false) & 0xFFFFu;
}

// four binary32 -> four fp8 codes packed little-endian in a dword
template <int FMT>
__device__ __forceinline__ uint32_t cvt4(float a, float b, float c, float d) {
    int r;
    if constexpr (FMT == FMT_E4M3FN) {
        r = __builtin_amdgcn_cvt_pk_fp8_f32(sat<FMT>(a), sat<FMT>(b), 0, false);
        r = __builtin_amdgcn_cvt_pk_fp8_f32(sat<FMT>(c), sat<FMT>(d), r, true);
    } else {
        r = __builtin_amdgcn_cvt_pk_bf8_f32(sat<FMT>(a), sat<FMT>(b), 0, false);
        r = __builtin_amdgcn_cvt_pk_bf8_f32(sat<FMT>(c), sat<FMT>(d), r, true);
    }
    return (uint32_t)r;
}

// 8 bfloat16 (one 128-bit load) times 8 scales -> 8 fp8 codes (two dwords)
template <int FMT>
__device__ __forceinline__ uint2 cast8(const uint4& v, const float (&s)[8]) {
    uint2 r;
    r.x = cvt4<FMT>(bf16_lo(v.x) * s[0], bf16_hi(v.x) * s[1], bf16_lo(v.y) * s[2], bf16_hi(v.y) * s[3]);
    r.y = cvt4<FMT>(bf16_lo(v.z) * s[4], bf16_hi(v.z) * s[5], bf16_lo(v.w) * s[6], bf16_hi(v.w) * s[7]);
    return r;
}
template <int FMT>
__device__ __forceinline__ uint2 cast8(const uint4& v, float s) {
    uint2 r;
    r.x = cvt4<FMT>(bf16_lo(v.x) * s, bf16_hi(v.x) * s, bf16_lo(v.y) * s, bf16_hi(v.y) * s);
    r.y = cvt4<FMT>(bf16_lo(v.z) * s, bf16_hi(v.z) * s, bf16_lo(v.w) * s, bf16_hi(v.w) * s);
    return r;
}

// Gradient through a sigmoid whose output y is stored in bfloat16: dz = dy * y * (1 - y), evaluated in
// binary32 one operation at a time, left to right (no contraction), rounded to bfloat16; 8 elements.
__device__ __forceinline__ uint32_t sigmoid_bwd_bf16_bits(float g, float y) {
    const float t = __fmul_rn(__fmul_rn(g, y), __fsub_rn(1.0f, y));
    const uint32_t b = __float_as_uint(t);
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;      // finite inputs: round to nearest even
}
__device__ __forceinline__ uint32_t sigmoid_bwd_pair(uint32_t g2, uint32_t y2) {
    return sigmoid_bwd_bf16_bits(bf16_lo(g2), bf16_lo(y2)) | (sigmoid_bwd_bf16_bits(bf16_hi(g2), bf16_hi(y2)) << 16);
}
__device__ __forceinline__ uint4 sigmoid_bwd8(const uint4& g, const uint4& y) {
    return make_uint4(sigmoid_bwd_pair(g.x, y.x), sigmoid_bwd_pair(g.y, y.y), sigmoid_bwd_pair(g.z, y.z), sigmoid_bwd_pair(g.w, y.w));
}

}  // namespace fp8k
