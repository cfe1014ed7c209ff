// amax / scale / cast / fused quantization kernels for gfx950 (HBM-bound).
//
// Every kernel reads bfloat16 with 128-bit loads laid out so that one
// wavefront instruction touches whole 128-byte lines, and writes fp8 codes
// with 64- or 128-bit stores.  Groups follow the paper's Appendix A: one scale
// per tensor, per row, or per column.
#include "fp8_device.hpp"
#include "launchers.hpp"
#include "tuning.hpp"

namespace fp8k {

// Twin launches.  Several kernels below take a second problem of the same kind after their ordinary arguments
// (x2, rows2, ...): blocks [0, split) work on the first, blocks [split, gridDim.x) on the second.  A linear layer
// quantizes two or three tensors the same way back to back (X and W; dY, W and X); for small layers the ~5 us that
// every dependent launch costs on the stream is what the step costs, so the launchers pair them up.
constexpr int NO_TWIN = 0x7FFFFFFF;


// ---------------------------------------------------------------- fill
__global__ void fill_u32_kernel(uint32_t* p, int64_t n, uint32_t v) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

hipError_t launch_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    fill_u32_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st>>>(p, n, v);
    return hipGetLastError();
}

// ---------------------------------------------------------------- amax
// Atomic max on the bits of a non-negative float.  Thousands of workgroups
// fold into the same few words; same-address atomics serialise in L2, so a
// plain load first drops every contribution that cannot raise the value (the
// stored maximum only grows, hence a stale read is harmless).
__device__ __forceinline__ void atomic_max_bits(uint32_t* addr, uint32_t bits) {
    if (bits > __builtin_nontemporal_load(addr)) atomicMax(addr, bits);
}

// One group of TX threads per row; TY = 256 / TX rows per block.
// single != 0: every row folds into out[0] with an atomic max (tensorwise
// amax of a matrix whose rows are not contiguous in memory).
template <int TX>
__global__ __launch_bounds__(256) void amax_rows_kernel(const uint16_t* __restrict__ x, int64_t rows,
                                                         int64_t cols, int64_t ld,
                                                         float* __restrict__ out, int single) {
    constexpr int TY = 256 / TX;
    const int tx = threadIdx.x % TX, ty = threadIdx.x / TX;
    const int64_t r = (int64_t)blockIdx.x * TY + ty;
    uint32_t acc = 0;
    if (r < rows) {
        const uint16_t* row = x + r * ld;
        const uint4* rv = reinterpret_cast<const uint4*>(row);
        const int64_t nvec = cols >> 3;
#pragma unroll 4
        for (int64_t v = tx; v < nvec; v += TX) acc = pk_absmax4(acc, rv[v]);
        for (int64_t c = (nvec << 3) + tx; c < cols; c += TX) acc = pk_absmax(acc, (uint32_t)row[c]);
    }
    uint32_t m = pk_fold(acc);
    m = wave_max_u32<(TX < 64 ? TX : 64)>(m);
    if constexpr (TX > 64) {
        __shared__ uint32_t part[256 / 64];
        const int wave = threadIdx.x / 64;
        if ((threadIdx.x & 63) == 0) part[wave] = m;
        __syncthreads();
        constexpr int WPR = TX / 64;  // waves per row
        const int w0 = ty * WPR;
        m = part[w0];
#pragma unroll
        for (int i = 1; i < WPR; ++i) m = part[w0 + i] > m ? part[w0 + i] : m;
    }
    if (r < rows && tx == 0) {
        if (single) atomic_max_bits(reinterpret_cast<uint32_t*>(out), m << 16);
        else out[r] = mag_to_float(m);
    }
}

// Tensorwise amax of a contiguous array of n bfloat16.  A block owns a
// contiguous chunk of 256 x 8 vectors; every thread issues its eight 128-bit
// loads back to back (all in flight together), then reduces.  One integer
// atomic max per block (out zeroed beforehand); PART: the block's maximum goes to
// out[blockIdx.x] instead (nothing to zero, the reader combines the gridDim.x values).
// A launch with gridDim.z == 2 serves two tensors: the blocks with blockIdx.z == 1 work on (x2, n2, out2).
template <bool PART>
__global__ __launch_bounds__(256) void amax_flat_kernel(const uint16_t* __restrict__ x, int64_t n,
                                                         float* __restrict__ out,
                                                         const uint16_t* __restrict__ x2 = nullptr, int64_t n2 = 0,
                                                         float* __restrict__ out2 = nullptr) {
    if (blockIdx.z) { x = x2; n = n2; out = out2; }
    const uint4* xv = reinterpret_cast<const uint4*>(x);
    const int64_t nvec = n >> 3;
    uint32_t acc = 0;
    // chunks of 256 x 8 vectors, dealt round-robin to the blocks (a block walks several chunks
    // when the tensor is large)
    for (int64_t chunk = blockIdx.x; chunk * (256 * 8) < nvec; chunk += gridDim.x) {
        const int64_t base = chunk * (256 * 8) + threadIdx.x;
        uint4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int64_t i = base + j * 256;
            v[j] = i < nvec ? load_stream(xv + i) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) acc = pk_absmax4(acc, v[j]);
    }
    if (blockIdx.x == 0)
        for (int64_t c = (nvec << 3) + threadIdx.x; c < n; c += 256) acc = pk_absmax(acc, (uint32_t)x[c]);
    uint32_t m = wave_max_u32<64>(pk_fold(acc));
    __shared__ uint32_t part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x / 64] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        m = part[0];
        for (int i = 1; i < 4; ++i) m = part[i] > m ? part[i] : m;
        if constexpr (PART) reinterpret_cast<uint32_t*>(out)[blockIdx.x] = m << 16;
        else atomic_max_bits(reinterpret_cast<uint32_t*>(out), m << 16);
    }
}

// The tensor's scale from the per-block maxima of amax_flat_kernel<true> (n_part of them, bits of
// non-negative floats): computed by the first wavefront of every block of the cast that follows, so that
// neither a zeroing nor a scale kernel sits between the two passes.  Returns the scale to all threads
// (contains a barrier: call it from uniform control flow).
template <int FMT>
__device__ __forceinline__ float tensor_scale_from_partials(const float* part, int n_part, int sflags, int tid,
                                                            bool writer, float* scale_out) {
    __shared__ float bc;
    if (tid < 64) {
        const uint32_t* pp = reinterpret_cast<const uint32_t*>(part);
        uint32_t m = 0;
        for (int i = tid; i < n_part; i += 64) {
            const uint32_t v = pp[i];
            m = v > m ? v : m;
        }
        m = wave_max_u32<64>(m);
        const float s = scale_from_amax(__uint_as_float(m), FMT, sflags);
        if (tid == 0) {
            bc = s;
            if (writer) scale_out[0] = s;
        }
    }
    __syncthreads();
    return bc;
}

// Column amax: a block of 8 wavefronts owns 512 columns (64 lanes x 8) and
// rows_per_block rows; wavefront w takes rows w, w+8, ...  out must be zeroed
// beforehand.
constexpr int AMAX_COLS_WAVES = 8;
__global__ __launch_bounds__(AMAX_COLS_WAVES * 64) void amax_cols_kernel(const uint16_t* __restrict__ x, int64_t rows,
                                                                          int64_t cols, int64_t ld,
                                                                          float* __restrict__ out,
                                                                          int64_t rows_per_block) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t c0 = (int64_t)blockIdx.x * 512 + lane * 8;
    const int64_t r_begin = (int64_t)blockIdx.y * rows_per_block;
    const int64_t r_end = r_begin + rows_per_block < rows ? r_begin + rows_per_block : rows;
    uint4 acc = make_uint4(0, 0, 0, 0);
    if (c0 < cols) {
        const uint16_t* p = x + c0;
#pragma unroll 8
        for (int64_t r = r_begin + wave; r < r_end; r += AMAX_COLS_WAVES) {
            const uint4 v = *reinterpret_cast<const uint4*>(p + r * ld);
            acc.x = pk_absmax(acc.x, v.x);
            acc.y = pk_absmax(acc.y, v.y);
            acc.z = pk_absmax(acc.z, v.z);
            acc.w = pk_absmax(acc.w, v.w);
        }
    }
    __shared__ uint4 part[AMAX_COLS_WAVES][64];
    part[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && c0 < cols) {
#pragma unroll
        for (int w = 1; w < AMAX_COLS_WAVES; ++w) {
            const uint4 o = part[w][lane];
            acc.x = pk_absmax(acc.x, o.x);
            acc.y = pk_absmax(acc.y, o.y);
            acc.z = pk_absmax(acc.z, o.z);
            acc.w = pk_absmax(acc.w, o.w);
        }
        const uint32_t w4[4] = {acc.x, acc.y, acc.z, acc.w};
        uint32_t* o = reinterpret_cast<uint32_t*>(out) + c0;
        // current maxima of my eight columns in two loads (stale values are fine:
        // they only grow), then atomics only where this block can raise them
        uint32_t cur[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (c0 + 8 <= cols) {
            const uint4 lo = *reinterpret_cast<const uint4*>(o);
            const uint4 hi = *reinterpret_cast<const uint4*>(o + 4);
            cur[0] = lo.x; cur[1] = lo.y; cur[2] = lo.z; cur[3] = lo.w;
            cur[4] = hi.x; cur[5] = hi.y; cur[6] = hi.z; cur[7] = hi.w;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t bits = ((e & 1) ? (w4[e >> 1] >> 16) : (w4[e >> 1] & 0xFFFFu)) << 16;
            if (c0 + e < cols && bits > cur[e]) atomicMax(o + e, bits);
        }
    }
}

// Column maxima, first level, for tall matrices: the matrix is streamed row by
// row exactly like the rowwise kernels do (a block reads whole rows, 128-bit
// loads, full lines), every thread keeps the running packed maxima of its own
// 8 * NV columns, and block b folds rows b, b + G, b + 2G, ...  The result is a
// [G, cols] matrix of bfloat16 magnitudes (same layout as the input rows) that
// the second level reduces with amax_cols_kernel.  This replaces thousands of
// strided 1 KB reads by long sequential ones.
template <int NV>
__global__ __launch_bounds__(256) void colmax_partial_kernel(const uint16_t* __restrict__ x, int64_t rows,
                                                              int64_t cols, int64_t ld,
                                                              uint16_t* __restrict__ part, int64_t ld_part,
                                                              int split = NO_TWIN, const uint16_t* __restrict__ x2 = nullptr,
                                                              int64_t rows2 = 0, int64_t ld2 = 0,
                                                              uint16_t* __restrict__ part2 = nullptr) {
    int bid = blockIdx.x, nb = split == NO_TWIN ? (int)gridDim.x : split;
    if (bid >= split) { bid -= split; nb = (int)gridDim.x - split; x = x2; rows = rows2; ld = ld2; part = part2; }
    const int64_t nvec = cols >> 3;
    const int ntail = (int)(cols & 7);
    uint4 acc[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) acc[j] = make_uint4(0, 0, 0, 0);
    uint32_t tail = 0;
    for (int64_t r = bid; r < rows; r += nb) {
        const uint16_t* row = x + r * ld;
        const uint4* rv = reinterpret_cast<const uint4*>(row);
        uint4 v[NV];
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int64_t vi = threadIdx.x + (int64_t)j * 256;
            v[j] = vi < nvec ? rv[vi] : make_uint4(0, 0, 0, 0);
        }
        if ((int)threadIdx.x < ntail) tail = pk_absmax(tail, (uint32_t)row[(nvec << 3) + threadIdx.x]);
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            acc[j].x = pk_absmax(acc[j].x, v[j].x);
            acc[j].y = pk_absmax(acc[j].y, v[j].y);
            acc[j].z = pk_absmax(acc[j].z, v[j].z);
            acc[j].w = pk_absmax(acc[j].w, v[j].w);
        }
    }
    uint16_t* prow = part + (int64_t)bid * ld_part;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int64_t vi = threadIdx.x + (int64_t)j * 256;
        if (vi < nvec) reinterpret_cast<uint4*>(prow)[vi] = acc[j];
    }
    if ((int)threadIdx.x < ntail) prow[(nvec << 3) + threadIdx.x] = (uint16_t)tail;
}

// Column maxima, second level, and the scales in the same kernel: the [G, cols]
// matrix of first-level magnitudes (G <= 1024) is small, so this is a latency
// problem.  A block of 1024 threads owns CL * 8 columns (CL = 8: 128-byte row
// pieces, twice the blocks of CL = 16); thread (row group t / CL, lane t % CL)
// folds rows t/CL, t/CL + 1024/CL, ... of its 8 columns with all of its loads in
// flight at once; the row groups of a wavefront combine by shuffles, the sixteen
// wavefronts through LDS, and CL threads turn the maxima into scales.  No
// atomics, nothing to zero first.
template <int CL>
__global__ __launch_bounds__(1024) void colmax_final_scale_kernel(const uint16_t* __restrict__ part, int G,
                                                                   int64_t cols, int64_t ld_part, int fmt, int flags,
                                                                   float* __restrict__ scale_out,
                                                                   int split = NO_TWIN, const uint16_t* __restrict__ part2 = nullptr,
                                                                   int G2 = 0, int64_t cols2 = 0, int64_t ld_part2 = 0, int fmt2 = 0,
                                                                   float* __restrict__ scale_out2 = nullptr,
                                                                   int split3 = NO_TWIN, const uint16_t* __restrict__ part3 = nullptr,
                                                                   int G3 = 0, int64_t cols3 = 0, int64_t ld_part3 = 0, int fmt3 = 0,
                                                                   float* __restrict__ scale_out3 = nullptr) {
    constexpr int RG = 1024 / CL;   // row groups
    const int tid = threadIdx.x, cl = tid % CL, rg = tid / CL;
    int bid = blockIdx.x;
    if (bid >= split3) { bid -= split3; part = part3; G = G3; cols = cols3; ld_part = ld_part3; fmt = fmt3; scale_out = scale_out3; }
    else if (bid >= split) { bid -= split; part = part2; G = G2; cols = cols2; ld_part = ld_part2; fmt = fmt2; scale_out = scale_out2; }
    const int64_t c = (int64_t)bid * (CL * 8) + cl * 8;
    uint4 acc = make_uint4(0, 0, 0, 0);
    if (c < cols) {
        const uint16_t* p = part + c;
#pragma unroll 16
        for (int g = rg; g < G; g += RG) {
            const uint4 v = *reinterpret_cast<const uint4*>(p + (int64_t)g * ld_part);
            acc.x = pk_absmax(acc.x, v.x);
            acc.y = pk_absmax(acc.y, v.y);
            acc.z = pk_absmax(acc.z, v.z);
            acc.w = pk_absmax(acc.w, v.w);
        }
    }
    static_assert(CL == 8 || CL == 16, "row pieces of 8 or 16 lanes");
    if constexpr (CL == 8) {
        acc.x = pk_absmax_xor<8>(acc.x); acc.y = pk_absmax_xor<8>(acc.y); acc.z = pk_absmax_xor<8>(acc.z); acc.w = pk_absmax_xor<8>(acc.w);
    }
    acc.x = pk_absmax_xor<16>(acc.x); acc.y = pk_absmax_xor<16>(acc.y); acc.z = pk_absmax_xor<16>(acc.z); acc.w = pk_absmax_xor<16>(acc.w);
    acc.x = pk_absmax_xor<32>(acc.x); acc.y = pk_absmax_xor<32>(acc.y); acc.z = pk_absmax_xor<32>(acc.z); acc.w = pk_absmax_xor<32>(acc.w);
    __shared__ uint4 sm[16][CL];
    if ((tid & 63) < CL) sm[tid >> 6][cl] = acc;
    __syncthreads();
    if (tid < CL && c < cols) {
#pragma unroll
        for (int w = 1; w < 16; ++w) {
            const uint4 o = sm[w][tid];
            acc.x = pk_absmax(acc.x, o.x);
            acc.y = pk_absmax(acc.y, o.y);
            acc.z = pk_absmax(acc.z, o.z);
            acc.w = pk_absmax(acc.w, o.w);
        }
        const uint32_t wds[4] = {acc.x, acc.y, acc.z, acc.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t mag = (wds[e >> 1] >> ((e & 1) * 16)) & 0x7FFFu;
            if (c + e < cols) scale_out[c + e] = scale_from_amax(mag_to_float(mag), fmt, flags);
        }
    }
}

static hipError_t launch_colmax_final_scale(const uint16_t* part, int64_t G, int64_t cols, int64_t ld_part, int fmt,
                                            int flags, float* scale_out, hipStream_t st) {
    // blocks of 64 columns (128-byte row pieces) unless that would be more blocks than the device has units for
    if (cols <= 64 * 256)
        colmax_final_scale_kernel<8><<<dim3((unsigned)((cols + 63) / 64)), dim3(1024), 0, st>>>(part, (int)G, cols, ld_part,
                                                                                            fmt, flags, scale_out);
    else
        colmax_final_scale_kernel<16><<<dim3((unsigned)((cols + 127) / 128)), dim3(1024), 0, st>>>(part, (int)G, cols, ld_part,
                                                                                              fmt, flags, scale_out);
    return hipGetLastError();
}

// Per-column SCALES of a tall matrix in two levels through a scratch matrix (at
// least G * ld_part bfloat16, 16-byte aligned): scale_out[c] =
// scale(max_r |x[r, c]|).  Returns hipErrorNotSupported if the shape does not
// suit it (few rows, very wide rows): the caller then uses launch_amax and
// launch_scale.
hipError_t launch_col_scales_two_level(const void* x, int64_t rows, int64_t cols, int64_t ld, int fmt, int flags,
                                       float* scale_out, void* scratch, size_t scratch_bytes, hipStream_t st) {
    const int64_t nvec = cols / 8;
    const int64_t ld_part = (cols + 7) / 8 * 8;
    int64_t G = 1024;
    while (G > 64 && (size_t)(G * ld_part * 2) > scratch_bytes) G /= 2;
    if (rows < 8 * G || nvec > 256 * 16 || (size_t)(G * ld_part * 2) > scratch_bytes) return hipErrorNotSupported;
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    uint16_t* part = static_cast<uint16_t*>(scratch);
#define FP8K_CP(NV) colmax_partial_kernel<NV><<<dim3((unsigned)G), dim3(256), 0, st>>>(xp, rows, cols, ld, part, ld_part)
    if (nvec <= 256) FP8K_CP(1);
    else if (nvec <= 512) FP8K_CP(2);
    else if (nvec <= 1024) FP8K_CP(4);
    else if (nvec <= 2048) FP8K_CP(8);
    else FP8K_CP(16);
#undef FP8K_CP
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_colmax_final_scale(part, G, cols, ld_part, fmt, flags, scale_out, st);
}

hipError_t launch_amax(const void* x, int64_t rows, int64_t cols, int64_t ld, int gran, float* out,
                       hipStream_t st) {
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    if (rows == 0 || cols == 0) {
        // empty groups have amax 0
        const int64_t n = gran == GRAN_TENSOR ? 1 : (gran == GRAN_ROW ? rows : cols);
        return launch_fill_u32(reinterpret_cast<uint32_t*>(out), n, 0u, st);
    }
    if (gran == GRAN_TENSOR && (ld == cols || rows == 1)) {
        hipError_t e = launch_fill_u32(reinterpret_cast<uint32_t*>(out), 1, 0u, st);
        if (e != hipSuccess) return e;
        const int64_t n = rows * cols;
        int64_t blocks = (n / 8 + 256 * 8 - 1) / (256 * 8);
        if (blocks < 1) blocks = 1;
        // few long-lived blocks: one atomic per block on a single address serialises, and tens of
        // thousands of them cost more than the read itself (measured on 134 MB: 512 blocks 23 us,
        // 32768 blocks 52 us)
        if (blocks > 512) blocks = 512;
        amax_flat_kernel<false><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(xp, n, out);
        return hipGetLastError();
    }
    if (gran == GRAN_TENSOR || gran == GRAN_ROW) {
        const int single = gran == GRAN_TENSOR;
        if (single) {
            hipError_t e = launch_fill_u32(reinterpret_cast<uint32_t*>(out), 1, 0u, st);
            if (e != hipSuccess) return e;
        }
        const int64_t nvec = cols / 8;
        if (nvec <= 16) {
            amax_rows_kernel<16><<<dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, st>>>(xp, rows, cols, ld, out, single);
        } else if (nvec <= 64) {
            amax_rows_kernel<64><<<dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st>>>(xp, rows, cols, ld, out, single);
        } else {
            amax_rows_kernel<256><<<dim3((unsigned)rows), dim3(256), 0, st>>>(xp, rows, cols, ld, out, single);
        }
        return hipGetLastError();
    }
    // GRAN_COL
    hipError_t e = launch_fill_u32(reinterpret_cast<uint32_t*>(out), cols, 0u, st);
    if (e != hipSuccess) return e;
    int64_t rpb = 256;
    while ((rows + rpb - 1) / rpb > 65535) rpb *= 2;
    dim3 grid((unsigned)((cols + 511) / 512), (unsigned)((rows + rpb - 1) / rpb));
    amax_cols_kernel<<<grid, dim3(AMAX_COLS_WAVES * 64), 0, st>>>(xp, rows, cols, ld, out, rpb);
    return hipGetLastError();
}

// ---------------------------------------------------------------- scale
__global__ void scale_kernel(const float* __restrict__ amax, int64_t n, int fmt, int flags,
                             float* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = scale_from_amax(amax[i], fmt, flags);
}

hipError_t launch_scale(const float* amax, int64_t n, int fmt, int flags, float* out, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    scale_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st>>>(amax, n, fmt, flags, out);
    return hipGetLastError();
}

// ---------------------------------------------------------------- cast
// Row-major cast: a thread converts 16 consecutive elements of one row
// (two 128-bit loads, one 128-bit store).  blockDim = (TX, TY).
template <int FMT, int GRAN>
__global__ __launch_bounds__(256) void cast_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                    int64_t ld, const float* __restrict__ scale,
                                                    uint8_t* __restrict__ q, int64_t ld_out, int n_part = 0,
                                                    int sflags = 0, float* __restrict__ scale_out = nullptr,
                                                    const uint16_t* __restrict__ x2 = nullptr, int64_t rows2 = 0,
                                                    const float* __restrict__ scale2 = nullptr,
                                                    uint8_t* __restrict__ q2 = nullptr,
                                                    float* __restrict__ scale_out2 = nullptr) {
    // gridDim.z == 2: a second tensor of the same width and leading dimensions in the blocks with blockIdx.z == 1
    if (blockIdx.z) { x = x2; rows = rows2; scale = scale2; q = q2; scale_out = scale_out2; }
    const int64_t c = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 16;
    float s_t = 0.0f;
    if constexpr (GRAN == GRAN_TENSOR) {
        // n_part > 0: scale points at the per-block maxima of the amax pass instead of at the scale
        if (n_part > 0)
            s_t = tensor_scale_from_partials<FMT>(scale, n_part, sflags, threadIdx.y * blockDim.x + threadIdx.x,
                                                  blockIdx.x == 0 && blockIdx.y == 0, scale_out);
        else
            s_t = scale[0];
    }
    if (c >= cols) return;
    for (int64_t r = (int64_t)blockIdx.y * blockDim.y + threadIdx.y; r < rows; r += (int64_t)gridDim.y * blockDim.y) {
        const uint16_t* src = x + r * ld + c;
        uint8_t* dst = q + r * ld_out + c;
        if constexpr (GRAN == GRAN_ROW) s_t = scale[r];
        if (c + 16 <= cols) {
            const uint4 v0 = load_stream(src);
            const uint4 v1 = load_stream(src + 8);
            uint2 lo, hi;
            if constexpr (GRAN == GRAN_COL) {
                float s[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) s[e] = scale[c + e];
                lo = cast8<FMT>(v0, s);
#pragma unroll
                for (int e = 0; e < 8; ++e) s[e] = scale[c + 8 + e];
                hi = cast8<FMT>(v1, s);
            } else {
                lo = cast8<FMT>(v0, s_t);
                hi = cast8<FMT>(v1, s_t);
            }
            store_stream(dst, make_uint4(lo.x, lo.y, hi.x, hi.y));
        } else {
            for (int e = 0; c + e < cols; ++e) {
                const float s = GRAN == GRAN_COL ? scale[c + e] : s_t;
                const float p = __uint_as_float((uint32_t)src[e] << 16) * s;
                dst[e] = (uint8_t)(cvt2<FMT>(p, p) & 0xFFu);
            }
        }
    }
}

// 4x4 byte transpose: rows a,b,c,d (byte j = column j) -> o[j] = column j
__device__ __forceinline__ void transpose4x4_bytes(uint32_t a, uint32_t b, uint32_t c, uint32_t d, uint32_t (&o)[4]) {
    const uint32_t t0 = __builtin_amdgcn_perm(b, a, 0x05010400u);
    const uint32_t t1 = __builtin_amdgcn_perm(b, a, 0x07030602u);
    const uint32_t u0 = __builtin_amdgcn_perm(d, c, 0x05010400u);
    const uint32_t u1 = __builtin_amdgcn_perm(d, c, 0x07030602u);
    o[0] = __builtin_amdgcn_perm(u0, t0, 0x05040100u);
    o[1] = __builtin_amdgcn_perm(u0, t0, 0x07060302u);
    o[2] = __builtin_amdgcn_perm(u1, t1, 0x05040100u);
    o[3] = __builtin_amdgcn_perm(u1, t1, 0x07060302u);
}

// Transposing cast.  A block converts a TR x 128 tile (TR = 128 or 256 input
// rows): each thread loads 8 x 8 sub-blocks (eight 128-bit loads each),
// converts them, transposes the bytes in registers and parks eight 64-bit
// column pieces in LDS; the block then streams the tile out as rows of the
// transposed matrix with 128-bit stores (TR contiguous bytes per output row).
// q_plain != nullptr additionally writes the untransposed codes (the
// tensorwise recipe needs both layouts of the same tensor in the backward).
// LDS tile: 128 output rows x TR bytes; the 8-byte slot index is XORed with
// 2 * ((row / 8) & 7) so that a wavefront's column pieces spread over banks.
// ACT: the tensor to cast is x * y * (1 - y) (gradient through a stored sigmoid output y of the same shape and
// leading dimension, cols a multiple of 8), formed on the fly.
// FOLD (per-column scales only): the scales may come from first-level column maxima, see below.
template <int FMT, int GRAN, int TR, bool ACT = false, bool FOLD = false>
__global__ __launch_bounds__(256) void cast_transpose_kernel(const uint16_t* __restrict__ x, int64_t rows,
                                                              int64_t cols, int64_t ld,
                                                              const float* __restrict__ scale,
                                                              uint8_t* __restrict__ qt, int64_t ld_t,
                                                              uint8_t* __restrict__ q_plain, int64_t ld_plain,
                                                              int nx, int ny, const uint16_t* __restrict__ yact = nullptr,
                                                              int n_part = 0, int sflags = 0,
                                                              float* __restrict__ scale_out = nullptr,
                                                              int split = NO_TWIN, const uint16_t* __restrict__ x2 = nullptr,
                                                              int64_t rows2 = 0, int64_t ld2 = 0,
                                                              const float* __restrict__ scale2 = nullptr,
                                                              uint8_t* __restrict__ qt2 = nullptr, int64_t ld_t2 = 0, int nx2 = 0,
                                                              int64_t ld_part = 0, int n_part2 = 0,
                                                              float* __restrict__ scale_out2 = nullptr,
                                                              uint8_t* __restrict__ q_plain2 = nullptr, int64_t ld_plain2 = 0) {
    int bid = blockIdx.x;
    if (bid >= split) {
        bid -= split; x = x2; rows = rows2; ld = ld2; scale = scale2; qt = qt2; ld_t = ld_t2; nx = nx2;
        n_part = n_part2; scale_out = scale_out2; q_plain = q_plain2; ld_plain = ld_plain2;
    }
    constexpr int SLOTS = TR / 8;   // 8-byte slots per output row
    constexpr int PARTS = TR / 16;  // 16-byte parts per output row
    __shared__ __attribute__((aligned(16))) uint2 tile[128 * SLOTS];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    // 1-D grid walked in patches of 16 x 16 tiles (input-row tiles fastest): the
    // workgroups in flight together read 4 KB runs of the input rows and write
    // 2 KB runs of the output rows, instead of isolated 256-byte / 128-byte pieces
    constexpr int PX = 16, PY = 16;
    const int pxc = (nx + PX - 1) / PX;
    const int patch = bid / (PX * PY), within = bid % (PX * PY);
    const int bx = (patch % pxc) * PX + within % PX, by = (patch / pxc) * PY + within / PX;
    if (bx >= nx || by >= ny) return;
    const int64_t r0 = (int64_t)bx * TR, c0 = (int64_t)by * 128;
    const int64_t c = c0 + tx * 8;

    float s_col[8];
    float s_t = 0.0f;
    if constexpr (GRAN == GRAN_TENSOR) {
        if (n_part == 0) s_t = scale[0];
    }
    if constexpr (GRAN == GRAN_COL) {
        if (!FOLD || n_part == 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) s_col[e] = (c + e < cols) ? scale[c + e] : 0.0f;
        }
    }

#pragma unroll
    for (int rh = 0; rh < TR / 128; ++rh) {
        uint32_t w[8][2];
        uint4 vv[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int64_t r = r0 + rh * 128 + ty * 8 + j;
            uint4 v = make_uint4(0, 0, 0, 0);
            if constexpr (FOLD) {
                // (cols is a multiple of 8 here.)  Unconditional loads from clamped addresses: all eight, and the
                // maxima after them, are in flight together whatever the compiler makes of the tile's edges
                const bool in = r < rows && c < cols;
                v = load_stream(x + (r < rows ? r : rows - 1) * ld + (c < cols ? c : 0));
                if (!in) v = make_uint4(0, 0, 0, 0);
            } else if (r < rows) {
                const uint16_t* src = x + r * ld + c;
                if (c + 8 <= cols) {
                    v = load_stream(src);
                    if constexpr (ACT) v = sigmoid_bwd8(v, load_stream(yact + r * ld + c));
                } else if (c < cols) {
                    uint32_t t[4] = {0, 0, 0, 0};
                    for (int e = 0; c + e < cols; ++e) t[e >> 1] |= (uint32_t)src[e] << ((e & 1) * 16);
                    v = make_uint4(t[0], t[1], t[2], t[3]);
                }
            }
            vv[j] = v;
        }
        if constexpr (GRAN == GRAN_TENSOR) {
            // n_part > 0: scale points at the per-block maxima of the amax pass instead of at the scale; the
            // scale is derived here, behind the tile's loads, so that its latency hides under them
            if (rh == 0 && n_part > 0)
                s_t = tensor_scale_from_partials<FMT>(scale, n_part, sflags, threadIdx.x, bid == 0, scale_out);
        }
        if constexpr (GRAN == GRAN_COL) {
            // n_part > 0: scale points at n_part rows (leading dimension ld_part) of first-level column maxima,
            // bfloat16 magnitudes; the block folds those of its 128 columns behind the tile's loads and the
            // blocks of the first row of tiles publish the scales.  Same maxima and scales as
            // colmax_final_scale_kernel, without its launch.
            if (FOLD && rh == 0 && n_part > 0) {
                __shared__ uint4 colred[16][16];
                const uint16_t* part = reinterpret_cast<const uint16_t*>(scale);
                uint4 acc = make_uint4(0, 0, 0, 0);
                for (int g0 = 0; g0 < n_part; g0 += 256) {   // (one trip: the launchers keep n_part <= 256)
                    uint4 pv[16];                            // sixteen rows of maxima per thread, all requested at once
#pragma unroll
                    for (int i = 0; i < 16; ++i) {   // (a row read twice does not change a maximum)
                        const int g = g0 + ty + 16 * i;
                        pv[i] = *reinterpret_cast<const uint4*>(part + (int64_t)(g < n_part ? g : n_part - 1) * ld_part + (c < cols ? c : 0));
                    }
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        acc.x = pk_absmax(acc.x, pv[i].x);
                        acc.y = pk_absmax(acc.y, pv[i].y);
                        acc.z = pk_absmax(acc.z, pv[i].z);
                        acc.w = pk_absmax(acc.w, pv[i].w);
                    }
                }
                colred[ty][tx] = acc;
                __syncthreads();
#pragma unroll
                for (int w = 0; w < 16; ++w) {
                    const uint4 o = colred[w][tx];
                    acc.x = pk_absmax(acc.x, o.x);
                    acc.y = pk_absmax(acc.y, o.y);
                    acc.z = pk_absmax(acc.z, o.z);
                    acc.w = pk_absmax(acc.w, o.w);
                }
                const uint32_t wds[4] = {acc.x, acc.y, acc.z, acc.w};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t mag = (wds[e >> 1] >> ((e & 1) * 16)) & 0x7FFFu;
                    s_col[e] = (c + e < cols) ? scale_from_amax(mag_to_float(mag), FMT, sflags) : 0.0f;
                    if (bx == 0 && ty == 0 && c + e < cols) scale_out[c + e] = s_col[e];
                }
            }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int64_t r = r0 + rh * 128 + ty * 8 + j;
            const uint4 v = vv[j];
            uint2 b;
            if constexpr (GRAN == GRAN_COL) {
                b = cast8<FMT>(v, s_col);
            } else {
                if constexpr (GRAN == GRAN_ROW) s_t = (r < rows) ? scale[r] : 0.0f;
                b = cast8<FMT>(v, s_t);
            }
            w[j][0] = b.x;
            w[j][1] = b.y;
            if (q_plain != nullptr && r < rows) {
                uint8_t* dst = q_plain + r * ld_plain + c;
                if (c + 8 <= cols) {
                    store_stream(dst, b);
                } else {
                    for (int e = 0; c + e < cols; ++e) dst[e] = (uint8_t)((e < 4 ? b.x >> (8 * e) : b.y >> (8 * (e - 4))) & 0xFFu);
                }
            }
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            uint32_t lo[4], hi[4];
            transpose4x4_bytes(w[0][h], w[1][h], w[2][h], w[3][h], lo);
            transpose4x4_bytes(w[4][h], w[5][h], w[6][h], w[7][h], hi);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int cc = tx * 8 + h * 4 + i;  // output row inside the tile
                tile[cc * SLOTS + ((rh * 16 + ty) ^ (2 * (tx & 7)))] = make_uint2(lo[i], hi[i]);
            }
        }
    }
    __syncthreads();

    const uint4* tile16 = reinterpret_cast<const uint4*>(tile);
    constexpr int ROWS_PER_IT = 256 / PARTS;
#pragma unroll
    for (int it = 0; it < 128 / ROWS_PER_IT; ++it) {
        const int cc = it * ROWS_PER_IT + (threadIdx.x / PARTS), p = threadIdx.x % PARTS;
        const int64_t oc = c0 + cc, orow = r0 + p * 16;
        if (oc >= cols || orow >= rows) continue;
        const uint4 v = tile16[cc * PARTS + (p ^ ((cc >> 3) & 7))];
        uint8_t* dst = qt + oc * ld_t + orow;
        if (orow + 16 <= rows) {
            store_stream(dst, v);
        } else {
            const uint32_t t[4] = {v.x, v.y, v.z, v.w};
            for (int e = 0; orow + e < rows; ++e) dst[e] = (uint8_t)((t[e >> 2] >> (8 * (e & 3))) & 0xFFu);
        }
    }
}

template <int FMT, int GRAN>
static hipError_t launch_cast_t(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, const float* scale,
                                int transpose, uint8_t* q, int64_t ld_out, uint8_t* q_plain, int64_t ld_plain,
                                hipStream_t st, int n_part = 0, int sflags = 0, float* scale_out = nullptr) {
    if (transpose) {
        // 128-row tiles measured best (256-row tiles: same on the 470 MB gradient
        // tensor, slower on the smaller operands)
        const int64_t gx = (cols + 127) / 128, gy = (rows + 127) / 128;
        const int64_t total = ((gy + 15) / 16) * ((gx + 15) / 16) * 256;
        if (total > 0x7FFFFFFF) return hipErrorInvalidValue;
        cast_transpose_kernel<FMT, GRAN, 128><<<dim3((unsigned)total), dim3(256), 0, st>>>(
            x, rows, cols, ld, scale, q, ld_out, q_plain, ld_plain, (int)gy, (int)gx, nullptr, n_part, sflags, scale_out);
        return hipGetLastError();
    }
    const int64_t items = (cols + 15) / 16;
    int tx = 1;
    while (tx < items && tx < 256) tx *= 2;
    const int ty = 256 / tx;
    int64_t gy = (rows + ty - 1) / ty;
    if (gy > 65535) gy = 65535;
    dim3 grid((unsigned)((items + tx - 1) / tx), (unsigned)gy);
    cast_kernel<FMT, GRAN><<<grid, dim3(tx, ty), 0, st>>>(x, rows, cols, ld, scale, q, ld_out, n_part, sflags, scale_out);
    return hipGetLastError();
}

// Tensorwise quantization of a dense tensor in two launches: per-block maxima into part (room for
// TENSOR_PARTIALS floats), then the cast, every block of which derives the scale from them; scale_out[0]
// receives the scale.  Same codes and scale as launch_amax + launch_scale + launch_cast.
hipError_t launch_quant_tensor(const void* x, int64_t rows, int64_t cols, int fmt, int flags, int transpose, uint8_t* q,
                               int64_t ld_out, uint8_t* q_plain, int64_t ld_plain, float* scale_out, float* part,
                               hipStream_t st) {
    if (rows == 0 || cols == 0) return hipSuccess;
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    const int64_t n = rows * cols;
    int64_t blocks = (n / 8 + 256 * 8 - 1) / (256 * 8);
    if (blocks < 1) blocks = 1;
    if (blocks > TENSOR_PARTIALS) blocks = TENSOR_PARTIALS;
    amax_flat_kernel<true><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(xp, n, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int sfl = flags & 1;
    if (fmt == FMT_E4M3FN)
        return launch_cast_t<FMT_E4M3FN, GRAN_TENSOR>(xp, rows, cols, cols, part, transpose, q, ld_out, q_plain, ld_plain, st,
                                                      (int)blocks, sfl, scale_out);
    return launch_cast_t<FMT_E5M2, GRAN_TENSOR>(xp, rows, cols, cols, part, transpose, q, ld_out, q_plain, ld_plain, st,
                                                (int)blocks, sfl, scale_out);
}

// The same for two dense tensors of the same width and format in two launches (one for both sets of maxima, one for
// both casts): X and W of a tensorwise forward, W and X of a stateless backward.
template <int FMT>
static hipError_t quant_tensor_pair(const TensorOperand& a, const TensorOperand& b, int64_t cols, int flags, int transpose,
                                    hipStream_t st) {
    const uint16_t *xa = static_cast<const uint16_t*>(a.x), *xb = static_cast<const uint16_t*>(b.x);
    auto blocks_of = [&](int64_t rows) {
        int64_t nb = (rows * cols / 8 + 256 * 8 - 1) / (256 * 8);
        return nb < 1 ? (int64_t)1 : nb > TENSOR_PARTIALS ? (int64_t)TENSOR_PARTIALS : nb;
    };
    const int64_t ba = blocks_of(a.rows), bb = blocks_of(b.rows), blocks = ba > bb ? ba : bb;   // (spare blocks of the smaller tensor store a zero)
    amax_flat_kernel<true><<<dim3((unsigned)blocks, 1, 2), dim3(256), 0, st>>>(xa, a.rows * cols, a.part, xb, b.rows * cols, b.part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int sfl = flags & 1;
    if (transpose) {
        const int64_t gx = (cols + 127) / 128, gya = (a.rows + 127) / 128, gyb = (b.rows + 127) / 128;
        const int64_t ta = ((gya + 15) / 16) * ((gx + 15) / 16) * 256, tb = ((gyb + 15) / 16) * ((gx + 15) / 16) * 256;
        if (ta + tb > 0x7FFFFFFF) return hipErrorInvalidValue;
        cast_transpose_kernel<FMT, GRAN_TENSOR, 128><<<dim3((unsigned)(ta + tb)), dim3(256), 0, st>>>(
            xa, a.rows, cols, cols, a.part, a.q, a.ld_out, a.q_plain, a.ld_plain, (int)gya, (int)gx, nullptr, (int)blocks, sfl,
            a.scale_out, (int)ta, xb, b.rows, cols, b.part, b.q, b.ld_out, (int)gyb, 0, (int)blocks, b.scale_out, b.q_plain,
            b.ld_plain);
        return hipGetLastError();
    }
    if (a.ld_out != b.ld_out) return hipErrorInvalidValue;
    const int64_t items = (cols + 15) / 16;
    int tx = 1;
    while (tx < items && tx < 256) tx *= 2;
    const int ty = 256 / tx;
    const int64_t rmax = a.rows > b.rows ? a.rows : b.rows;
    int64_t gy = (rmax + ty - 1) / ty;
    if (gy > 65535) gy = 65535;
    cast_kernel<FMT, GRAN_TENSOR><<<dim3((unsigned)((items + tx - 1) / tx), (unsigned)gy, 2), dim3(tx, ty), 0, st>>>(
        xa, a.rows, cols, cols, a.part, a.q, a.ld_out, (int)blocks, sfl, a.scale_out, xb, b.rows, b.part, b.q, b.scale_out);
    return hipGetLastError();
}

hipError_t launch_quant_tensor_pair(const TensorOperand& a, const TensorOperand& b, int64_t cols, int fmt, int flags,
                                    int transpose, hipStream_t st) {
    if (knob(KNOB_PAIRS) == 0) return hipErrorNotSupported;
    if (a.rows == 0 || b.rows == 0 || cols == 0) return hipErrorNotSupported;
    return fmt == FMT_E4M3FN ? quant_tensor_pair<FMT_E4M3FN>(a, b, cols, flags, transpose, st)
                             : quant_tensor_pair<FMT_E5M2>(a, b, cols, flags, transpose, st);
}

hipError_t launch_cast(const void* x, int64_t rows, int64_t cols, int64_t ld, const float* scale, int gran,
                       int fmt, int transpose, uint8_t* q, int64_t ld_out, uint8_t* q_plain, int64_t ld_plain,
                       hipStream_t st) {
    if (rows == 0 || cols == 0) return hipSuccess;
    const uint16_t* xp = static_cast<const uint16_t*>(x);
#define FP8K_CAST(F, G) \
    if (fmt == F && gran == G) return launch_cast_t<F, G>(xp, rows, cols, ld, scale, transpose, q, ld_out, q_plain, ld_plain, st)
    FP8K_CAST(FMT_E4M3FN, GRAN_TENSOR);
    FP8K_CAST(FMT_E4M3FN, GRAN_ROW);
    FP8K_CAST(FMT_E4M3FN, GRAN_COL);
    FP8K_CAST(FMT_E5M2, GRAN_TENSOR);
    FP8K_CAST(FMT_E5M2, GRAN_ROW);
    FP8K_CAST(FMT_E5M2, GRAN_COL);
#undef FP8K_CAST
    return hipErrorInvalidValue;
}

// ------------------------------------------------- fused rowwise quantize
// amax -> scale -> cast of whole rows in ONE pass over HBM: a group of TX
// threads owns a row and keeps it in registers (NV 128-bit vectors per
// thread) between the reduction and the conversion.
template <int FMT, int TX, int NV>
__global__ __launch_bounds__(256) void quant_row_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                         int64_t ld, int flags, uint8_t* __restrict__ q,
                                                         int64_t ld_out, float* __restrict__ scale_out,
                                                         int split = NO_TWIN, const uint16_t* __restrict__ x2 = nullptr,
                                                         int64_t rows2 = 0, int64_t ld2 = 0, uint8_t* __restrict__ q2 = nullptr,
                                                         int64_t ld_out2 = 0, float* __restrict__ scale_out2 = nullptr) {
    constexpr int TY = 256 / TX;
    const int tx = threadIdx.x % TX, ty = threadIdx.x / TX;
    int bid = blockIdx.x;
    if (bid >= split) { bid -= split; x = x2; rows = rows2; ld = ld2; q = q2; ld_out = ld_out2; scale_out = scale_out2; }
    const int64_t r = (int64_t)bid * TY + ty;
    const bool live = r < rows;
    const int64_t nvec = cols >> 3;
    const int ntail = (int)(cols & 7);
    const uint16_t* row = x + (live ? r : 0) * ld;
    const uint4* rv = reinterpret_cast<const uint4*>(row);

    uint4 v[NV];
    uint32_t acc = 0;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int64_t vi = tx + (int64_t)j * TX;
        v[j] = (live && vi < nvec) ? load_stream(rv + vi) : make_uint4(0, 0, 0, 0);
    }
    uint32_t tail = 0;
    if (live && tx < ntail) tail = row[(nvec << 3) + tx];
#pragma unroll
    for (int j = 0; j < NV; ++j) acc = pk_absmax4(acc, v[j]);
    acc = pk_absmax(acc, tail);

    uint32_t m = wave_max_u32<(TX < 64 ? TX : 64)>(pk_fold(acc));
    if constexpr (TX > 64) {
        __shared__ uint32_t part[256 / 64];
        if ((threadIdx.x & 63) == 0) part[threadIdx.x / 64] = m;
        __syncthreads();
        constexpr int WPR = TX / 64;
        const int w0 = ty * WPR;
        m = part[w0];
#pragma unroll
        for (int i = 1; i < WPR; ++i) m = part[w0 + i] > m ? part[w0 + i] : m;
    }
    if (!live) return;
    const float s = scale_from_amax(mag_to_float(m), FMT, flags);
    if (tx == 0) scale_out[r] = s;

    uint8_t* dst = q + r * ld_out;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int64_t vi = tx + (int64_t)j * TX;
        if (vi < nvec) store_stream(reinterpret_cast<uint2*>(dst) + vi, cast8<FMT>(v[j], s));
    }
    if (tx < ntail) {
        const float p = __uint_as_float(tail << 16) * s;
        dst[(nvec << 3) + tx] = (uint8_t)(cvt2<FMT>(p, p) & 0xFFu);
    }
}

template <int FMT>
static bool launch_quant_row_t(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, int flags, uint8_t* q,
                               int64_t ld_out, float* scale_out, hipStream_t st) {
    const int64_t nvec = cols / 8;
#define FP8K_QR(TX, NV)                                                                              \
    quant_row_kernel<FMT, TX, NV><<<dim3((unsigned)((rows + (256 / TX) - 1) / (256 / TX))), dim3(256), 0, st>>>( \
        x, rows, cols, ld, flags, q, ld_out, scale_out)
    if (nvec <= 16) FP8K_QR(16, 1);
    else if (nvec <= 64) FP8K_QR(64, 1);
    else if (nvec <= 256) FP8K_QR(256, 1);
    else if (nvec <= 512) FP8K_QR(256, 2);
    else if (nvec <= 1024) FP8K_QR(256, 4);
    else if (nvec <= 2048) FP8K_QR(256, 8);
    else if (nvec <= 4096) FP8K_QR(256, 16);
    else return false;
#undef FP8K_QR
    return true;
}

// returns hipErrorNotSupported when a row does not fit in registers (the
// caller then runs amax, scale and cast as separate passes)
hipError_t launch_quant_row(const void* x, int64_t rows, int64_t cols, int64_t ld, int fmt, int flags, uint8_t* q,
                            int64_t ld_out, float* scale_out, hipStream_t st) {
    if (rows == 0) return hipSuccess;
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    const bool ok = fmt == FMT_E4M3FN
                        ? launch_quant_row_t<FMT_E4M3FN>(xp, rows, cols, ld, flags, q, ld_out, scale_out, st)
                        : launch_quant_row_t<FMT_E5M2>(xp, rows, cols, ld, flags, q, ld_out, scale_out, st);
    if (!ok) return hipErrorNotSupported;
    return hipGetLastError();
}

// ------------------------------ fused rowwise quantize + column maxima (first level)
// The gradient of a rowwise-scaled linear layer is quantized twice: per row for
// dX = dY W and per column for dW = dY^T X (Appendix A).  This kernel serves
// both from ONE read: block b walks rows b, b + G, b + 2G, ...; a row sits in
// registers while its maximum is reduced and its codes are written (as in
// quant_row_kernel), and every thread also folds the row into the running
// maxima of its own 8 * NV columns.  The block's column maxima go to row b of
// a [G, cols] matrix of bfloat16 magnitudes, which amax_cols_kernel reduces;
// the per-column cast then reads the tensor a second (and last) time.
// With up to four vectors per thread the next rows are requested before the
// current ones are reduced; wider rows rely on the other resident blocks to keep
// loads in flight (a second row in registers would halve the occupancy).  Rows
// of up to 2048 (4096) elements travel four (two) at a time: a block of a small
// tensor has only a handful of rows, and each trip to memory that it has to
// wait for costs about a microsecond.  The wave maxima alternate between two
// LDS slots, so one barrier per trip is enough.
// ACT: the tensor to quantize is dz = x * y * (1 - y), formed on the fly from the gradient x and the stored
// sigmoid output y (same shape and leading dimension): the backward through Sigmoid + Linear never
// materialises dz.
template <int FMT, int NV, bool ACT = false>
__global__ __launch_bounds__(256) void quant_row_colmax_kernel(const uint16_t* __restrict__ x, int64_t rows,
                                                                int64_t cols, int64_t ld, int flags,
                                                                uint8_t* __restrict__ q, int64_t ld_out,
                                                                float* __restrict__ scale_out,
                                                                uint16_t* __restrict__ part, int64_t ld_part,
                                                                const uint16_t* __restrict__ yact = nullptr,
                                                                int split = NO_TWIN, const uint16_t* __restrict__ x2 = nullptr,
                                                                int64_t rows2 = 0, int64_t ld2 = 0, uint8_t* __restrict__ q2 = nullptr,
                                                                int64_t ld_out2 = 0, float* __restrict__ scale_out2 = nullptr,
                                                                uint16_t* __restrict__ part2 = nullptr) {
    constexpr bool PREFETCH = NV <= 4;
    constexpr int R = NV == 1 ? 4 : NV == 2 ? 2 : 1;   // rows in flight together (narrow rows: one round trip to memory serves R rows)
    int bid = blockIdx.x, nb = split == NO_TWIN ? (int)gridDim.x : split;
    if (bid >= split) {
        bid -= split; nb = (int)gridDim.x - split;
        x = x2; rows = rows2; ld = ld2; q = q2; ld_out = ld_out2; scale_out = scale_out2; part = part2;
    }
    const int64_t nvec = cols >> 3;     // cols is a multiple of 8 (checked by the launcher)
    const int tid = threadIdx.x;
    __shared__ uint32_t red[2][R][4];
    uint4 cmax[NV], v[R][NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) cmax[j] = make_uint4(0, 0, 0, 0);
    // rows r0, r0 + nb, ..., r0 + (R - 1) nb; zeros for rows beyond the end
    auto load_rows = [&](int64_t r0, uint4 (&dst)[R][NV]) {
#pragma unroll
        for (int k = 0; k < R; ++k) {
            const int64_t r = r0 + (int64_t)k * nb;
            const bool in = r < rows;
            const uint4* rv = reinterpret_cast<const uint4*>(x + (in ? r : 0) * ld);
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                const int64_t vi = tid + (int64_t)j * 256;
                dst[k][j] = (in && vi < nvec) ? rv[vi] : make_uint4(0, 0, 0, 0);
            }
            if constexpr (ACT) {
                const uint4* yv = reinterpret_cast<const uint4*>(yact + (in ? r : 0) * ld);
#pragma unroll
                for (int j = 0; j < NV; ++j) {
                    const int64_t vi = tid + (int64_t)j * 256;
                    if (in && vi < nvec) dst[k][j] = sigmoid_bwd8(dst[k][j], yv[vi]);
                }
            }
        }
    };
    const int64_t stride = (int64_t)R * nb;
    int64_t r = bid;
    if (PREFETCH && r < rows) load_rows(r, v);
    int slot = 0;
    for (; r < rows; r += stride) {
        const int64_t rn = r + stride;
        uint4 nv[PREFETCH ? R : 1][PREFETCH ? NV : 1];
        if constexpr (PREFETCH) {
            if (rn < rows) load_rows(rn, nv);
        } else {
            load_rows(r, v);
        }
#pragma unroll
        for (int k = 0; k < R; ++k) {
            uint32_t acc = 0;
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                cmax[j].x = pk_absmax(cmax[j].x, v[k][j].x);
                cmax[j].y = pk_absmax(cmax[j].y, v[k][j].y);
                cmax[j].z = pk_absmax(cmax[j].z, v[k][j].z);
                cmax[j].w = pk_absmax(cmax[j].w, v[k][j].w);
                acc = pk_absmax4(acc, v[k][j]);
            }
            const uint32_t m = wave_max_u32<64>(pk_fold(acc));
            if ((tid & 63) == 0) red[slot][k][tid >> 6] = m;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < R; ++k) {
            const int64_t rk = r + (int64_t)k * nb;
            if (rk >= rows) break;
            uint32_t m = red[slot][k][0];
#pragma unroll
            for (int i = 1; i < 4; ++i) m = red[slot][k][i] > m ? red[slot][k][i] : m;
            const float s = scale_from_amax(mag_to_float(m), FMT, flags);
            if (tid == 0) scale_out[rk] = s;
            uint8_t* dst = q + rk * ld_out;
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                const int64_t vi = tid + (int64_t)j * 256;
                if (vi < nvec) store_stream(reinterpret_cast<uint2*>(dst) + vi, cast8<FMT>(v[k][j], s));
            }
        }
        slot ^= 1;
        if constexpr (PREFETCH) {
            if (rn < rows) {
#pragma unroll
                for (int k = 0; k < R; ++k)
#pragma unroll
                    for (int j = 0; j < NV; ++j) v[k][j] = nv[k][j];
            }
        }
    }
    uint16_t* prow = part + (int64_t)bid * ld_part;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int64_t vi = tid + (int64_t)j * 256;
        if (vi < nvec) reinterpret_cast<uint4*>(prow)[vi] = cmax[j];
    }
}

// number of blocks of the kernel that the device keeps resident at once
template <typename K>
static int resident_blocks(K kernel) {
    int per_cu = 0, dev = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, 256, 0) != hipSuccess) return 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    return per_cu * cus;
}

// Rowwise codes + scales of x, and the per-column scales scale_cols[c] =
// scale(max_r |x[r, c]|), from one read of x.  scratch: at least 128 * cols * 2 bytes, 16-byte aligned (more lets
// more blocks run).  hipErrorNotSupported if the shape does not suit
// (cols not a multiple of 8, rows too few or too wide for registers).
hipError_t launch_quant_row_colmax(const void* x, int64_t rows, int64_t cols, int64_t ld, int fmt, int flags,
                                   uint8_t* q, int64_t ld_out, float* scale_out, float* scale_cols, void* scratch,
                                   size_t scratch_bytes, hipStream_t st) {
    const int64_t nvec = cols / 8;
    if (cols % 8 != 0 || nvec > 256 * 16 || nvec < 64) return hipErrorNotSupported;
    const int64_t ld_part = cols;
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    uint16_t* part = static_cast<uint16_t*>(scratch);
    // G blocks, all resident at once (a second, partly filled round of blocks would
    // idle most of the chip), each with at least 8 rows (fewer where that would leave CUs without a block:
    // a 1024 x 16384 tensor took 24 us with 128 blocks), G rows of scratch
    int64_t G = 0;
#define FP8K_QRC(FMT, NV)                                                                                     \
    do {                                                                                                      \
        static CachedInt resident_c;   /* per kernel */                                                       \
        const int resident = resident_c.get([] { return resident_blocks(quant_row_colmax_kernel<FMT, NV>); }); \
        G = resident < 1024 ? resident : 1024;                                                                \
        { /* at least 8 rows per block, but not fewer than 256 blocks while each still has 2 rows */          \
            int64_t cap = rows / 8;                                                                           \
            if (cap < 256) cap = rows / 2 < 256 ? rows / 2 : 256;                                             \
            if (G > cap) G = cap;                                                                             \
        }                                                                                                     \
        if ((size_t)(G * ld_part * 2) > scratch_bytes) G = (int64_t)(scratch_bytes / (size_t)(ld_part * 2));  \
        if (G < 128) return hipErrorNotSupported;                                                             \
        quant_row_colmax_kernel<FMT, NV><<<dim3((unsigned)G), dim3(256), 0, st>>>(xp, rows, cols, ld, flags, q, ld_out, \
                                                                                  scale_out, part, ld_part);  \
    } while (0)
#define FP8K_QRC_NV(FMT)                 \
    if (nvec <= 256) FP8K_QRC(FMT, 1);   \
    else if (nvec <= 512) FP8K_QRC(FMT, 2);  \
    else if (nvec <= 1024) FP8K_QRC(FMT, 4); \
    else if (nvec <= 2048) FP8K_QRC(FMT, 8); \
    else FP8K_QRC(FMT, 16)
    if (fmt == FMT_E4M3FN) { FP8K_QRC_NV(FMT_E4M3FN); }
    else { FP8K_QRC_NV(FMT_E5M2); }
#undef FP8K_QRC_NV
#undef FP8K_QRC
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_colmax_final_scale(part, G, cols, ld_part, fmt, flags, scale_cols, st);
}


// ------------------------------------------------------------------ paired launches
// The quantizations of a linear layer come in twos and threes of the same kind.  The functions below issue them as
// twin launches (see NO_TWIN above) and share one second-level launch for all column scales.  They return
// hipErrorNotSupported when a tensor does not suit the kernels involved: the caller then quantizes one by one.

// Side storage for first-level column maxima: with it they stay out of the transposed output, so the transposing cast
// can fold them itself and the second-level launch falls away.  Worth it for small tensors only: every block of the
// cast reads all the maxima of its 128 columns, and the first level must make do with FOLD_ROWS blocks (measured:
// 3-8 us less per forward + backward step with tensors of 1024 rows, 3-5 us more with 4096).  0 for the others.
int64_t quant_fold_bytes(int64_t rows, int64_t cols) {
    if (rows < 256 || rows > 2048 || cols < 8 || cols % 8 != 0 || rows * cols > ((int64_t)4 << 20)) return 0;
    return FOLD_ROWS * ((cols + 7) / 8 * 8) * 2;
}

namespace {

int64_t output_scratch(int64_t out_rows, int64_t out_cols, int64_t ld_out) {   // bytes of a transposed output that may hold partial maxima
    return ld_out == out_cols ? out_rows * out_cols : out_cols;
}

// where the first-level maxima of a tensor go: the caller's side storage, if any (the cast then folds them), else the
// transposed output itself, which the cast overwrites afterwards
struct Partials { uint16_t* at; int64_t room; bool folded; };
Partials partials_of(void* fold, int64_t rows, int64_t cols, uint8_t* q_col_t, int64_t ld_col_t) {
    const int64_t fb = fold ? quant_fold_bytes(rows, cols) : 0;
    if (fb) return Partials{static_cast<uint16_t*>(fold), fb, true};
    return Partials{reinterpret_cast<uint16_t*>(q_col_t), output_scratch(cols, rows, ld_col_t), false};
}

// blocks of quant_row_colmax_kernel for a tensor, given how many the device keeps resident for it (0: not suited)
int64_t row_colmax_blocks(int64_t rows, int64_t cols, int64_t scratch_bytes, int64_t resident) {
    int64_t G = resident < 1024 ? resident : 1024;
    int64_t cap = rows / 8;                       // at least 8 rows per block, but not fewer than 256 blocks while each still has 2 rows
    if (cap < 256) cap = rows / 2 < 256 ? rows / 2 : 256;
    if (G > cap) G = cap;
    if (G * cols * 2 > scratch_bytes) G = scratch_bytes / (cols * 2);
    return G < 128 ? 0 : G;
}

// blocks of colmax_partial_kernel for a tensor (0: not suited)
int64_t colmax_partial_blocks(int64_t rows, int64_t cols, int64_t scratch_bytes) {
    const int64_t ld_part = (cols + 7) / 8 * 8;
    int64_t G = 1024;
    while (G > 64 && (G * ld_part * 2 > scratch_bytes || rows < 4 * G)) G /= 2;
    if (rows < 4 * G || cols / 8 > 256 * 16 || G * ld_part * 2 > scratch_bytes) return 0;
    return G;
}

struct FinalSeg { const uint16_t* part; int64_t G, cols, ld_part; int fmt; float* scale_out; };
// second level of up to three column-scale problems in one launch (none: no launch)
hipError_t launch_colmax_final_scale_multi(const FinalSeg* seg, int n, int flags, hipStream_t st) {
    if (n == 0) return hipSuccess;
    int64_t nb[3] = {0, 0, 0};
    for (int i = 0; i < n; ++i) nb[i] = (seg[i].cols + 63) / 64;
    const FinalSeg z{nullptr, 0, 0, 0, 0, nullptr};
    const FinalSeg &a = seg[0], &b = n > 1 ? seg[1] : z, &c = n > 2 ? seg[2] : z;
    const int64_t total = nb[0] + nb[1] + nb[2];
    if (total > 0x7FFFFFFF) return hipErrorInvalidValue;
    colmax_final_scale_kernel<8><<<dim3((unsigned)total), dim3(1024), 0, st>>>(
        a.part, (int)a.G, a.cols, a.ld_part, a.fmt, flags, a.scale_out,
        n > 1 ? (int)nb[0] : NO_TWIN, b.part, (int)b.G, b.cols, b.ld_part, b.fmt, b.scale_out,
        n > 2 ? (int)(nb[0] + nb[1]) : NO_TWIN, c.part, (int)c.G, c.cols, c.ld_part, c.fmt, c.scale_out);
    return hipGetLastError();
}

// Transposing per-column cast of one tensor (b == nullptr) or two of the same width in one launch.  An operand with
// folded partials (pa / pb .folded, Ga / Gb rows of leading dimension ld_part) derives and publishes its scales itself;
// the others read scale_col.
template <int FMT>
hipError_t cast_t_col(const ColOperand& a, const Partials& pa, int64_t Ga, const ColOperand* b, const Partials& pb, int64_t Gb,
                      int64_t cols, int64_t ld_part, int flags, hipStream_t st) {
    const int64_t gx = (cols + 127) / 128;
    const int64_t gya = (a.rows + 127) / 128, gyb = b ? (b->rows + 127) / 128 : 0;
    const int64_t ta = ((gya + 15) / 16) * ((gx + 15) / 16) * 256, tb = ((gyb + 15) / 16) * ((gx + 15) / 16) * 256;
    if (ta + tb > 0x7FFFFFFF) return hipErrorInvalidValue;
    const float* sa = pa.folded ? reinterpret_cast<const float*>(pa.at) : a.scale_col;
    const float* sb = !b ? nullptr : pb.folded ? reinterpret_cast<const float*>(pb.at) : b->scale_col;
    auto kern = pa.folded || (b && pb.folded) ? cast_transpose_kernel<FMT, GRAN_COL, 128, false, true>
                                              : cast_transpose_kernel<FMT, GRAN_COL, 128, false, false>;
    kern<<<dim3((unsigned)(ta + tb)), dim3(256), 0, st>>>(
        static_cast<const uint16_t*>(a.x), a.rows, cols, a.ld, sa, a.q_col_t, a.ld_col_t, nullptr, 0, (int)gya, (int)gx,
        nullptr, pa.folded ? (int)Ga : 0, flags & 1, a.scale_col,
        b ? (int)ta : NO_TWIN, b ? static_cast<const uint16_t*>(b->x) : nullptr, b ? b->rows : 0, b ? b->ld : 0, sb,
        b ? b->q_col_t : nullptr, b ? b->ld_col_t : 0, (int)gyb, ld_part, b && pb.folded ? (int)Gb : 0, b ? b->scale_col : nullptr,
        nullptr, 0);
    return hipGetLastError();
}
hipError_t cast_t_col(int fmt, const ColOperand& a, const Partials& pa, int64_t Ga, const ColOperand* b, const Partials& pb,
                      int64_t Gb, int64_t cols, int64_t ld_part, int flags, hipStream_t st) {
    return fmt == FMT_E4M3FN ? cast_t_col<FMT_E4M3FN>(a, pa, Ga, b, pb, Gb, cols, ld_part, flags, st)
                             : cast_t_col<FMT_E5M2>(a, pa, Ga, b, pb, Gb, cols, ld_part, flags, st);
}

// first level of the column maxima of two tensors of the same width in one launch; Ga, Gb: blocks (rows of partials) of each
hipError_t colmax_partial_pair(const ColOperand& a, uint16_t* pa, int64_t Ga, const ColOperand& b, uint16_t* pb, int64_t Gb,
                               int64_t cols, hipStream_t st) {
    const int64_t nvec = cols / 8, ld_part = (cols + 7) / 8 * 8;
    const uint16_t *xa = static_cast<const uint16_t*>(a.x), *xb = static_cast<const uint16_t*>(b.x);
#define FP8K_CPP(NV) colmax_partial_kernel<NV><<<dim3((unsigned)(Ga + Gb)), dim3(256), 0, st>>>(xa, a.rows, cols, a.ld, pa, ld_part, (int)Ga, xb, b.rows, b.ld, pb)
    if (nvec <= 256) FP8K_CPP(1);
    else if (nvec <= 512) FP8K_CPP(2);
    else if (nvec <= 1024) FP8K_CPP(4);
    else if (nvec <= 2048) FP8K_CPP(8);
    else FP8K_CPP(16);
#undef FP8K_CPP
    return hipGetLastError();
}

// rowwise codes + first-level column maxima of one tensor (b == nullptr) or two of the same width and format in one
// launch, the maxima going to pa / pb.  Ga / Gb receive the numbers of blocks = rows of partials; 0 blocks: not suited
// (nothing launched).
template <int FMT, int NV>
hipError_t row_colmax_first_level(const RowColOperand& a, const Partials& pa, const RowColOperand* b, const Partials& pb,
                                  int64_t cols, int flags, int64_t* Ga, int64_t* Gb, hipStream_t st) {
    static CachedInt resident_c;
    const int64_t resident = resident_c.get([] { return resident_blocks(quant_row_colmax_kernel<FMT, NV>); });
    // two tensors share the resident blocks in proportion to their rows
    const int64_t ra = b ? resident * a.rows / (a.rows + b->rows) : resident;
    *Ga = row_colmax_blocks(a.rows, cols, pa.room, ra);
    *Gb = b ? row_colmax_blocks(b->rows, cols, pb.room, resident - ra) : 0;
    if (*Ga == 0 || (b && *Gb == 0)) return hipErrorNotSupported;
    if (b)
        quant_row_colmax_kernel<FMT, NV><<<dim3((unsigned)(*Ga + *Gb)), dim3(256), 0, st>>>(
            static_cast<const uint16_t*>(a.x), a.rows, cols, a.ld, flags, a.q_row, a.ld_row, a.scale_row, pa.at, cols, nullptr,
            (int)*Ga, static_cast<const uint16_t*>(b->x), b->rows, b->ld, b->q_row, b->ld_row, b->scale_row, pb.at);
    else
        quant_row_colmax_kernel<FMT, NV><<<dim3((unsigned)*Ga), dim3(256), 0, st>>>(
            static_cast<const uint16_t*>(a.x), a.rows, cols, a.ld, flags, a.q_row, a.ld_row, a.scale_row, pa.at, cols);
    return hipGetLastError();
}

hipError_t row_colmax_first_level(const RowColOperand& a, const Partials& pa, const RowColOperand* b, const Partials& pb,
                                  int64_t cols, int fmt, int flags, int64_t* Ga, int64_t* Gb, hipStream_t st) {
    const int64_t nvec = cols / 8;
    if (cols % 8 != 0 || nvec > 256 * 16 || nvec < 64) return hipErrorNotSupported;
#define FP8K_RCF(FMT)                                                                                     \
    if (nvec <= 256) return row_colmax_first_level<FMT, 1>(a, pa, b, pb, cols, flags, Ga, Gb, st);        \
    if (nvec <= 512) return row_colmax_first_level<FMT, 2>(a, pa, b, pb, cols, flags, Ga, Gb, st);        \
    if (nvec <= 1024) return row_colmax_first_level<FMT, 4>(a, pa, b, pb, cols, flags, Ga, Gb, st);       \
    if (nvec <= 2048) return row_colmax_first_level<FMT, 8>(a, pa, b, pb, cols, flags, Ga, Gb, st);       \
    return row_colmax_first_level<FMT, 16>(a, pa, b, pb, cols, flags, Ga, Gb, st)
    if (fmt == FMT_E4M3FN) { FP8K_RCF(FMT_E4M3FN); }
    FP8K_RCF(FMT_E5M2);
#undef FP8K_RCF
}

ColOperand col_part(const RowColOperand& o) { return ColOperand{o.x, o.rows, o.ld, o.q_col_t, o.ld_col_t, o.scale_col, o.fold}; }
Partials partials_of(const RowColOperand& o, int64_t cols) { return partials_of(o.fold, o.rows, cols, o.q_col_t, o.ld_col_t); }
Partials partials_of(const ColOperand& o, int64_t cols) { return partials_of(o.fold, o.rows, cols, o.q_col_t, o.ld_col_t); }

}  // namespace

hipError_t launch_quant_row_pair(const void* x1, int64_t rows1, int64_t ld1, uint8_t* q1, int64_t ld_q1, float* s1, const void* x2,
                                 int64_t rows2, int64_t ld2, uint8_t* q2, int64_t ld_q2, float* s2, int64_t cols, int fmt,
                                 int flags, hipStream_t st) {
    if (knob(KNOB_PAIRS) == 0) return hipErrorNotSupported;
    if (rows1 == 0 || rows2 == 0) return hipErrorNotSupported;
    const int64_t nvec = cols / 8;
    const uint16_t *a = static_cast<const uint16_t*>(x1), *b = static_cast<const uint16_t*>(x2);
#define FP8K_QRP(FMT, TX, NV)                                                                                     \
    do {                                                                                                          \
        const int64_t ba = (rows1 + (256 / TX) - 1) / (256 / TX), bb = (rows2 + (256 / TX) - 1) / (256 / TX);     \
        if (ba + bb > 0x7FFFFFFF) return hipErrorInvalidValue;                                                    \
        quant_row_kernel<FMT, TX, NV><<<dim3((unsigned)(ba + bb)), dim3(256), 0, st>>>(a, rows1, cols, ld1, flags, q1, ld_q1, s1, \
                                                                                       (int)ba, b, rows2, ld2, q2, ld_q2, s2); \
    } while (0)
#define FP8K_QRP_F(FMT)                          \
    if (nvec <= 16) FP8K_QRP(FMT, 16, 1);        \
    else if (nvec <= 64) FP8K_QRP(FMT, 64, 1);   \
    else if (nvec <= 256) FP8K_QRP(FMT, 256, 1); \
    else if (nvec <= 512) FP8K_QRP(FMT, 256, 2); \
    else if (nvec <= 1024) FP8K_QRP(FMT, 256, 4);\
    else if (nvec <= 2048) FP8K_QRP(FMT, 256, 8);\
    else if (nvec <= 4096) FP8K_QRP(FMT, 256, 16);\
    else return hipErrorNotSupported
    if (fmt == FMT_E4M3FN) { FP8K_QRP_F(FMT_E4M3FN); }
    else { FP8K_QRP_F(FMT_E5M2); }
#undef FP8K_QRP_F
#undef FP8K_QRP
    return hipGetLastError();
}

hipError_t launch_quant_row_col_pair(const RowColOperand& a, const RowColOperand* b, int64_t cols, int fmt, int flags,
                                     hipStream_t st) {
    if (b && knob(KNOB_PAIRS) == 0) return hipErrorNotSupported;
    if (a.rows == 0 || (b && b->rows == 0) || cols == 0) return hipErrorNotSupported;
    const Partials pa = partials_of(a, cols), pb = b ? partials_of(*b, cols) : Partials{nullptr, 0, false};
    int64_t Ga = 0, Gb = 0;
    hipError_t e = row_colmax_first_level(a, pa, b, pb, cols, fmt, flags, &Ga, &Gb, st);
    if (e != hipSuccess) return e;
    FinalSeg seg[2];
    int n = 0;
    if (!pa.folded) seg[n++] = FinalSeg{pa.at, Ga, cols, cols, fmt, a.scale_col};
    if (b && !pb.folded) seg[n++] = FinalSeg{pb.at, Gb, cols, cols, fmt, b->scale_col};
    e = launch_colmax_final_scale_multi(seg, n, flags, st);
    if (e != hipSuccess) return e;
    const ColOperand ca = col_part(a), cb = b ? col_part(*b) : ColOperand{};
    return cast_t_col(fmt, ca, pa, Ga, b ? &cb : nullptr, pb, Gb, cols, cols, flags, st);
}

hipError_t launch_quant_col_t_pair(const ColOperand& a, const ColOperand& b, int64_t cols, int fmt, int flags, hipStream_t st) {
    if (knob(KNOB_PAIRS) == 0) return hipErrorNotSupported;
    if (a.rows == 0 || b.rows == 0 || cols == 0) return hipErrorNotSupported;
    const Partials pa = partials_of(a, cols), pb = partials_of(b, cols);
    const int64_t Ga = colmax_partial_blocks(a.rows, cols, pa.room), Gb = colmax_partial_blocks(b.rows, cols, pb.room);
    if (Ga == 0 || Gb == 0) return hipErrorNotSupported;
    hipError_t e = colmax_partial_pair(a, pa.at, Ga, b, pb.at, Gb, cols, st);
    if (e != hipSuccess) return e;
    const int64_t ld_part = (cols + 7) / 8 * 8;
    FinalSeg seg[2];
    int n = 0;
    if (!pa.folded) seg[n++] = FinalSeg{pa.at, Ga, cols, ld_part, fmt, a.scale_col};
    if (!pb.folded) seg[n++] = FinalSeg{pb.at, Gb, cols, ld_part, fmt, b.scale_col};
    e = launch_colmax_final_scale_multi(seg, n, flags, st);
    if (e != hipSuccess) return e;
    return cast_t_col(fmt, a, pa, Ga, &b, pb, Gb, cols, ld_part, flags, st);
}

hipError_t launch_quant_bwd_rowwise(const RowColOperand& g, int64_t cols_g, int fmt_g, const ColOperand& w, const ColOperand& x,
                                    int64_t cols_wx, int fmt_wx, int flags, hipStream_t st) {
    if (knob(KNOB_PAIRS) == 0) return hipErrorNotSupported;
    if (g.rows == 0 || w.rows == 0 || x.rows == 0 || cols_g == 0 || cols_wx == 0) return hipErrorNotSupported;
    // everything is checked before the first launch, so that "not suited" leaves nothing half done
    const Partials pg = partials_of(g, cols_g), pw = partials_of(w, cols_wx), px = partials_of(x, cols_wx);
    const int64_t Gw = colmax_partial_blocks(w.rows, cols_wx, pw.room), Gx = colmax_partial_blocks(x.rows, cols_wx, px.room);
    if (Gw == 0 || Gx == 0) return hipErrorNotSupported;
    int64_t Gg = 0, unused = 0;
    hipError_t e = row_colmax_first_level(g, pg, nullptr, Partials{nullptr, 0, false}, cols_g, fmt_g, flags, &Gg, &unused, st);   // (launches only if suited)
    if (e != hipSuccess) return e;
    e = colmax_partial_pair(w, pw.at, Gw, x, px.at, Gx, cols_wx, st);
    if (e != hipSuccess) return e;
    const int64_t ld_part = (cols_wx + 7) / 8 * 8;
    FinalSeg seg[3];
    int n = 0;
    if (!pg.folded) seg[n++] = FinalSeg{pg.at, Gg, cols_g, cols_g, fmt_g, g.scale_col};
    if (!pw.folded) seg[n++] = FinalSeg{pw.at, Gw, cols_wx, ld_part, fmt_wx, w.scale_col};
    if (!px.folded) seg[n++] = FinalSeg{px.at, Gx, cols_wx, ld_part, fmt_wx, x.scale_col};
    e = launch_colmax_final_scale_multi(seg, n, flags, st);
    if (e != hipSuccess) return e;
    e = cast_t_col(fmt_g, col_part(g), pg, Gg, nullptr, Partials{nullptr, 0, false}, 0, cols_g, cols_g, flags, st);
    if (e != hipSuccess) return e;
    return cast_t_col(fmt_wx, w, pw, Gw, &x, px, Gx, cols_wx, ld_part, flags, st);
}

// The gradient through Sigmoid + Linear, quantized along both axes without materialising
// dz = dy * y * (1 - y): rowwise codes + scales and per-column scales from one read of (dy, y), then
// the per-column transposed codes from a second.  Same conditions as launch_quant_row_colmax
// (hipErrorNotSupported otherwise: the caller then materialises dz).
hipError_t launch_quant_row_col_sigmoid_bwd(const void* dy, const void* y, int64_t rows, int64_t cols, int64_t ld,
                                            int fmt, int flags, uint8_t* q_row, int64_t ld_row, float* scale_row,
                                            uint8_t* q_col_t, int64_t ld_col_t, float* scale_col, hipStream_t st) {
    const int64_t nvec = cols / 8;
    if (cols % 8 != 0 || nvec > 256 * 16 || nvec < 64) return hipErrorNotSupported;
    const uint16_t* xp = static_cast<const uint16_t*>(dy);
    const uint16_t* yp = static_cast<const uint16_t*>(y);
    const int64_t ld_part = cols;
    uint16_t* part = reinterpret_cast<uint16_t*>(q_col_t);          // overwritten by the transposed codes afterwards
    // only bytes that the transposed cast rewrites: all of a dense output, else its first row
    const size_t scratch_bytes = ld_col_t == rows ? (size_t)cols * (size_t)rows : (size_t)rows;
    int64_t G = 0;
#define FP8K_QRCA(FMT, NV)                                                                                    \
    do {                                                                                                      \
        static CachedInt resident_c;                                                                          \
        const int resident = resident_c.get([] { return resident_blocks(quant_row_colmax_kernel<FMT, NV, true>); }); \
        G = resident < 1024 ? resident : 1024;                                                                \
        { /* at least 8 rows per block, but not fewer than 256 blocks while each still has 2 rows */          \
            int64_t cap = rows / 8;                                                                           \
            if (cap < 256) cap = rows / 2 < 256 ? rows / 2 : 256;                                             \
            if (G > cap) G = cap;                                                                             \
        }                                                                                                     \
        if ((size_t)(G * ld_part * 2) > scratch_bytes) G = (int64_t)(scratch_bytes / (size_t)(ld_part * 2));  \
        if (G < 128) return hipErrorNotSupported;                                                             \
        quant_row_colmax_kernel<FMT, NV, true><<<dim3((unsigned)G), dim3(256), 0, st>>>(                       \
            xp, rows, cols, ld, flags, q_row, ld_row, scale_row, part, ld_part, yp);                          \
    } while (0)
#define FP8K_QRCA_NV(FMT)                 \
    if (nvec <= 256) FP8K_QRCA(FMT, 1);   \
    else if (nvec <= 512) FP8K_QRCA(FMT, 2);  \
    else if (nvec <= 1024) FP8K_QRCA(FMT, 4); \
    else if (nvec <= 2048) FP8K_QRCA(FMT, 8); \
    else FP8K_QRCA(FMT, 16)
    if (fmt == FMT_E4M3FN) { FP8K_QRCA_NV(FMT_E4M3FN); }
    else { FP8K_QRCA_NV(FMT_E5M2); }
#undef FP8K_QRCA_NV
#undef FP8K_QRCA
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = launch_colmax_final_scale(part, G, cols, ld_part, fmt, flags, scale_col, st);
    if (e != hipSuccess) return e;
    const int64_t gx = (cols + 127) / 128, gy = (rows + 127) / 128;
    const int64_t total = ((gy + 15) / 16) * ((gx + 15) / 16) * 256;
    if (total > 0x7FFFFFFF) return hipErrorInvalidValue;
    if (fmt == FMT_E4M3FN)
        cast_transpose_kernel<FMT_E4M3FN, GRAN_COL, 128, true><<<dim3((unsigned)total), dim3(256), 0, st>>>(
            xp, rows, cols, ld, scale_col, q_col_t, ld_col_t, nullptr, 0, (int)gy, (int)gx, yp);
    else
        cast_transpose_kernel<FMT_E5M2, GRAN_COL, 128, true><<<dim3((unsigned)total), dim3(256), 0, st>>>(
            xp, rows, cols, ld, scale_col, q_col_t, ld_col_t, nullptr, 0, (int)gy, (int)gx, yp);
    return hipGetLastError();
}

// dz = dy * y * (1 - y) materialised (bfloat16, dense): the fallback for shapes the fused kernels do not take
__global__ __launch_bounds__(256) void sigmoid_bwd_kernel(const uint16_t* __restrict__ dy, const uint16_t* __restrict__ y,
                                                           int64_t n, uint16_t* __restrict__ dz) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v * 8 + 8 <= n) {
        const uint4 g = load_stream(dy + v * 8), s = load_stream(y + v * 8);
        store_stream(dz + v * 8, sigmoid_bwd8(g, s));
    } else {
        for (int64_t i = v * 8; i < n; ++i)
            dz[i] = (uint16_t)sigmoid_bwd_bf16_bits(__uint_as_float((uint32_t)dy[i] << 16), __uint_as_float((uint32_t)y[i] << 16));
    }
}
hipError_t launch_sigmoid_bwd(const void* dy, const void* y, int64_t n, void* dz, hipStream_t st) {
    if (n == 0) return hipSuccess;
    const int64_t blocks = ((n + 7) / 8 + 255) / 256;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    sigmoid_bwd_kernel<<<dim3((unsigned)blocks), dim3(256), 0, st>>>(static_cast<const uint16_t*>(dy), static_cast<const uint16_t*>(y), n,
                                                                      static_cast<uint16_t*>(dz));
    return hipGetLastError();
}

// ------------------------------------------------------------ MX block quantization
// Blocks of 32 consecutive elements of a row share one power-of-two scale
// (OCP MX specification v1.0, Section 6.3): shared exponent = floor(log2(block
// maximum)) - emax of the element format (8 for E4M3, 15 for E5M2), stored as
// the E8M0 byte exponent + 127 (clamped to [0, 254]; an all-zero block gets 0);
// elements = x * 2^-exponent (exact), saturating round-to-nearest-even cast.
// Offset of the scale byte of block kb of row r.  ld_e >= 0: rows of ld_e bytes (the layout of the public
// entry points).  ld_e < 0: slabs of sixteen blocks, [kb / 16][row][16 bytes] with -ld_e rows per slab: the
// scales that one 256-row tile of the block-scaled GEMM needs for four K steps are then 4 KB in a row (the
// linear entry points use it between their quantizers and the GEMM).  Four consecutive blocks from a multiple
// of four stay consecutive in both layouts.
__device__ __forceinline__ int64_t e8_off(int64_t r, int64_t kb, int64_t ld_e) {
    return ld_e >= 0 ? r * ld_e + kb : ((kb >> 4) * -ld_e + r) * 16 + (kb & 15);
}

// Four lanes own a block (one 128-bit load each); the maximum is taken on the
// bfloat16 magnitude bits, whose exponent field gives floor(log2) directly.
template <int FMT, bool DENSE>
__global__ __launch_bounds__(256) void mx_quant_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                        int64_t ld, uint8_t* __restrict__ q, int64_t ld_q,
                                                        uint8_t* __restrict__ e8m0, int64_t ld_e) {
    constexpr int U = DENSE ? 4 : 1;                    // vectors per thread, all loads issued before the first use
    constexpr int EMAX = FMT == FMT_E4M3FN ? 8 : 15;
    const int64_t vpr = cols >> 3;                      // 128-bit vectors per row (cols % 32 == 0)
    const int64_t nvec = rows * vpr;
    const int64_t v0 = (int64_t)blockIdx.x * (256 * U) + threadIdx.x;
    uint4 d[U];
    int64_t xo[U], qo[U], eo[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t v = v0 + u * 256;
        const bool live = v < nvec;
        // DENSE: all three matrices have no row padding, so the flat vector index addresses them directly
        // (no 64-bit division per thread)
        if constexpr (DENSE) {
            xo[u] = v * 8; qo[u] = v * 8;
            eo[u] = ld_e >= 0 ? v >> 2 : (live ? e8_off(v / vpr, (v % vpr) >> 2, ld_e) : 0);
        } else {
            const int64_t r = live ? v / vpr : 0, cv = live ? v % vpr : 0;
            xo[u] = r * ld + cv * 8; qo[u] = r * ld_q + cv * 8; eo[u] = e8_off(r, cv >> 2, ld_e);
        }
        d[u] = live ? load_stream(x + xo[u]) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        uint32_t m = pk_fold(pk_absmax4(0u, d[u]));
        m = pk_absmax_xor<2>(pk_absmax_xor<1>(m));           // block maximum (four lanes), 15 magnitude bits of bfloat16
        int byte = 0;
        if (m != 0) {
            const int ef = (int)(m >> 7);
            // normal: 2^(ef - 127) * 1.f; subnormal: mantissa * 2^-133
            const int fl = ef > 0 ? ef - 127 : (31 - __builtin_clz(m)) - 133;
            byte = fl - EMAX + 127;
            byte = byte < 0 ? 0 : (byte > 254 ? 254 : byte);
        }
        // 2^(127 - byte): byte <= 246 for bfloat16 input, so the factor is a normal binary32
        const float factor = __uint_as_float((uint32_t)(254 - byte) << 23);
        if (v0 + u * 256 < nvec) {
            store_stream(q + qo[u], cast8<FMT>(d[u], factor));
            if ((threadIdx.x & 3) == 0) e8m0[eo[u]] = (uint8_t)byte;
        }
    }
}

hipError_t launch_mx_quant(const void* x, int64_t rows, int64_t cols, int64_t ld, int fmt, uint8_t* q, int64_t ld_q,
                           uint8_t* e8m0, int64_t ld_e, hipStream_t st) {
    if (rows == 0 || cols == 0) return hipSuccess;
    const int64_t nvec = rows * (cols / 8);
    const bool dense = ld == cols && ld_q == cols && (ld_e == cols / 32 || ld_e < 0);
    const int64_t per_block = dense ? 1024 : 256;       // the dense kernel takes 4 vectors per thread
    const int64_t blocks = (nvec + per_block - 1) / per_block;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    const uint16_t* xp = static_cast<const uint16_t*>(x);
#define FP8K_MXQ(FMT, D) mx_quant_kernel<FMT, D><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(xp, rows, cols, ld, q, ld_q, e8m0, ld_e)
    if (fmt == FMT_E4M3FN) { if (dense) FP8K_MXQ(FMT_E4M3FN, true); else FP8K_MXQ(FMT_E4M3FN, false); }
    else { if (dense) FP8K_MXQ(FMT_E5M2, true); else FP8K_MXQ(FMT_E5M2, false); }
#undef FP8K_MXQ
    return hipGetLastError();
}

// ------------------------------------------------------------ blockwise FP8
// The blockwise recipe on the paper's list of prototype features ("FP8 blockwise
// quantization introduced by DeepSeek"): activations in tiles of 1 x 128 along
// the contraction axis, weights in blocks of 128 x 128.  The scale of a block
// is that of the rowwise / tensorwise recipes applied to the block and rounded
// down to a power of two, s = 2^k, so that its reciprocal is an E8M0 byte
// (127 - k) that the block-scaled matrix instruction applies by itself; the
// byte is written in the layout of the MX scales ([rows, cols / 32]: four
// copies per 128 columns, one row of copies per row of a 128 x 128 block), which
// makes the MX GEMM the product of two blockwise operands too.
//
// The power-of-two scale of a block from the 15 magnitude bits of its bfloat16 maximum, without the
// binary64 division of scale_from_amax(., ., pow2): FMAX = 1.75 * 2^E (E = 8 / 15) and amax = m * 2^e with
// 1 <= m < 2 in steps of 2^-7, so FMAX / amax = (1.75 / m) * 2^(E - e) lies in [2^(E-e), 2^(E-e+1)) for
// m <= 1.75 and in (0.995 * 2^(E-e), ... ) rounded down to 2^(E-e-1) for m > 1.75 (1.75 / m <= 0.9956 there:
// the binary32 rounding of the quotient cannot reach the next power of two).  Maxima not above 1e-12 (bits
// below 0x2B8D: 2^-40 * (1 + 13/128) is the first bfloat16 above 1e-12) take the clamp's scale,
// floor_pow2(fp32(FMAX * 1e12)) = 2^(40 + E).  Identical to the division for every bfloat16 maximum (tested
// on all of them).  Returns the scale; byte receives 127 - log2(scale).
template <int FMT>
__device__ __forceinline__ float pow2_block_scale(uint32_t mag, uint32_t& byte) {
    constexpr int E = FMT == FMT_E4M3FN ? 8 : 15;
    int k = 40 + E;
    if (mag >= 0x2B8Du) k = E - ((int)(mag >> 7) - 127) - ((mag & 0x7Fu) > 96u ? 1 : 0);
    byte = (uint32_t)(127 - k);
    return __uint_as_float((uint32_t)(k + 127) << 23);
}

// 1 x 128 tiles: a thread holds 8 elements of each of four tiles (all four loads in flight together), the 16
// threads of a tile combine their maxima with four cross-lane steps.  cols % 128 == 0.
template <int FMT>
__global__ __launch_bounds__(256) void block_quant_1x128_kernel(const uint16_t* __restrict__ x, int64_t rows,
                                                                 int64_t cols, int64_t ld, uint8_t* __restrict__ q,
                                                                 int64_t ld_q, uint8_t* __restrict__ e8m0,
                                                                 int64_t ld_e) {
    constexpr int U = 4;
    const int64_t vpr = cols >> 3, nvec = rows * vpr;          // a multiple of 16: tiles never straddle the end
    const int64_t v0 = (int64_t)blockIdx.x * (256 * U) + threadIdx.x;
    uint4 d[U];
    int64_t r[U], cv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t v = v0 + u * 256;
        const bool live = v < nvec;
        r[u] = live ? v / vpr : 0;
        cv[u] = live ? v % vpr : 0;
        d[u] = live ? load_stream(x + r[u] * ld + cv[u] * 8) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        uint32_t m = wave_max_u32<16>(pk_fold(pk_absmax4(0u, d[u])));     // the tile's sixteen lanes
        uint32_t byte;
        const float s = pow2_block_scale<FMT>(m, byte);
        if (v0 + u * 256 < nvec) {
            store_stream(q + r[u] * ld_q + cv[u] * 8, cast8<FMT>(d[u], s));
            if ((threadIdx.x & 15) == 0)     // ld_e % 4 == 0 and (cv / 4) % 4 == 0: an aligned dword
                *reinterpret_cast<uint32_t*>(e8m0 + e8_off(r[u], cv[u] >> 2, ld_e)) = byte * 0x01010101u;
        }
    }
}

// 128 x 128 blocks: one workgroup per block, the block held in registers (8 x 8 elements per thread)
// between the reduction and the conversion: one pass over HBM.  The bottom row of blocks may be partial.
template <int FMT>
__global__ __launch_bounds__(256) void block_quant_128x128_kernel(const uint16_t* __restrict__ x, int64_t rows,
                                                                   int64_t cols, int64_t ld, uint8_t* __restrict__ q,
                                                                   int64_t ld_q, uint8_t* __restrict__ e8m0,
                                                                   int64_t ld_e) {
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int64_t r0 = (int64_t)blockIdx.y * 128, c0 = (int64_t)blockIdx.x * 128, c = c0 + tx * 8;
    uint4 v[8];
    uint32_t acc = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int64_t r = r0 + ty * 8 + j;
        v[j] = r < rows ? load_stream(x + r * ld + c) : make_uint4(0, 0, 0, 0);
        acc = pk_absmax4(acc, v[j]);
    }
    uint32_t m = wave_max_u32<64>(pk_fold(acc));
    __shared__ uint32_t red[4];
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    m = red[0];
#pragma unroll
    for (int i = 1; i < 4; ++i) m = red[i] > m ? red[i] : m;
    uint32_t byte;
    const float s = pow2_block_scale<FMT>(m, byte);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int64_t r = r0 + ty * 8 + j;
        if (r < rows) store_stream(q + r * ld_q + c, cast8<FMT>(v[j], s));
    }
    if (threadIdx.x < 128 && r0 + threadIdx.x < rows) {
        *reinterpret_cast<uint32_t*>(e8m0 + e8_off(r0 + threadIdx.x, c0 >> 5, ld_e)) = byte * 0x01010101u;
    }
}

// block_rows: 1 (tiles of 1 x 128) or 128 (blocks of 128 x 128); cols % 128 == 0
hipError_t launch_block_quant(const void* x, int64_t rows, int64_t cols, int64_t ld, int block_rows, int fmt, uint8_t* q,
                              int64_t ld_q, uint8_t* e8m0, int64_t ld_e, hipStream_t st) {
    if (rows == 0 || cols == 0) return hipSuccess;
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    if (block_rows == 1) {
        const int64_t blocks = (rows * (cols / 8) + 1023) / 1024;
        if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
        if (fmt == FMT_E4M3FN) block_quant_1x128_kernel<FMT_E4M3FN><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(xp, rows, cols, ld, q, ld_q, e8m0, ld_e);
        else block_quant_1x128_kernel<FMT_E5M2><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(xp, rows, cols, ld, q, ld_q, e8m0, ld_e);
    } else {
        const int64_t gy = (rows + 127) / 128;
        if (gy > 65535) return hipErrorInvalidValue;
        const dim3 grid((unsigned)(cols / 128), (unsigned)gy);
        if (fmt == FMT_E4M3FN) block_quant_128x128_kernel<FMT_E4M3FN><<<grid, dim3(256), 0, st>>>(xp, rows, cols, ld, q, ld_q, e8m0, ld_e);
        else block_quant_128x128_kernel<FMT_E5M2><<<grid, dim3(256), 0, st>>>(xp, rows, cols, ld, q, ld_q, e8m0, ld_e);
    }
    return hipGetLastError();
}

// MX block quantization with the blocks running DOWN the columns of x and the
// output written transposed: qt [cols, rows] codes and et [cols, rows / 32] E8M0
// bytes, i.e. the K-contiguous operand of a product that contracts over the
// rows of x (the backward products of the MX linear layer).  rows % 32 == 0.
// Same tile scheme as the transposing cast above (128 x 128 tile, 8 x 8 register
// blocks, byte transpose, swizzled LDS tile, 128-bit streaming stores); a
// wavefront holds exactly one block of 32 rows (4 thread rows x 8), so the
// block maxima of its 128 columns are two cross-lane steps away.
// ROWS_TOO: the same read also yields the quantization with the blocks running ALONG the rows
// (q_row [rows, cols], e_row [rows, cols / 32]; cols % 32 == 0): the four threads that hold 32
// consecutive elements of a row combine their maxima with two cross-lane steps.  A tensor that is
// needed in both orientations (the gradient in the backward) then costs 4 bytes per element
// instead of 6.
template <int FMT, bool ROWS_TOO>
__global__ __launch_bounds__(256) void mx_quant_t_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                          int64_t ld, uint8_t* __restrict__ qt, int64_t ld_t,
                                                          uint8_t* __restrict__ et, int64_t ld_e,
                                                          uint8_t* __restrict__ q_row, int64_t ld_row,
                                                          uint8_t* __restrict__ e_row, int64_t ld_er, int nx, int ny) {
    constexpr int TR = 128, SLOTS = TR / 8, PARTS = TR / 16;
    constexpr int EMAX = FMT == FMT_E4M3FN ? 8 : 15;
    __shared__ __attribute__((aligned(16))) uint2 tile[128 * SLOTS];
    __shared__ __attribute__((aligned(16))) uint8_t ebytes[128 * 4];   // [column of the tile][block of the tile]
    __shared__ __attribute__((aligned(16))) uint8_t rbytes[ROWS_TOO ? 128 * 4 : 4];   // [row of the tile][column block of the tile]
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    constexpr int PX = 16, PY = 16;
    const int pxc = (nx + PX - 1) / PX;
    const int patch = blockIdx.x / (PX * PY), within = blockIdx.x % (PX * PY);
    const int bx = (patch % pxc) * PX + within % PX, by = (patch / pxc) * PY + within / PX;
    if (bx >= nx || by >= ny) return;
    const int64_t r0 = (int64_t)bx * TR, c0 = (int64_t)by * 128;
    const int64_t c = c0 + tx * 8;

    uint4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int64_t r = r0 + ty * 8 + j;
        v[j] = make_uint4(0, 0, 0, 0);
        if (r < rows) {
            const uint16_t* src = x + r * ld + c;
            if (c + 8 <= cols) {
                v[j] = load_stream(src);
            } else if (c < cols) {
                uint32_t t[4] = {0, 0, 0, 0};
                for (int e = 0; c + e < cols; ++e) t[e >> 1] |= (uint32_t)src[e] << ((e & 1) * 16);
                v[j] = make_uint4(t[0], t[1], t[2], t[3]);
            }
        }
    }
    if constexpr (ROWS_TOO) {
        // blocks along the rows: row r0 + 8 ty + j, columns c0 + 32 (tx / 4) .. + 31 (the tile is inside the
        // matrix in this direction or the block is not stored: cols % 32 == 0)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            uint32_t mr = pk_fold(pk_absmax4(0u, v[j]));
            mr = pk_absmax_xor<2>(pk_absmax_xor<1>(mr));
            int byte = 0;
            if (mr != 0) {
                const int ef = (int)(mr >> 7);
                const int fl = ef > 0 ? ef - 127 : (31 - __builtin_clz(mr)) - 133;
                byte = fl - EMAX + 127;
                byte = byte < 0 ? 0 : (byte > 254 ? 254 : byte);
            }
            const float f = __uint_as_float((uint32_t)(254 - byte) << 23);
            const int64_t r = r0 + ty * 8 + j;
            if (r < rows && c < cols) store_stream(q_row + r * ld_row + c, cast8<FMT>(v[j], f));
            if ((tx & 3) == 0) rbytes[(ty * 8 + j) * 4 + (tx >> 2)] = (uint8_t)byte;
        }
    }
    // maxima of the 8 columns over this thread's 8 rows (two 15-bit magnitudes per register), then over the
    // 4 thread rows of the wavefront (lanes l, l ^ 16, l ^ 32, l ^ 48)
    uint32_t m[4] = {0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        m[0] = pk_absmax(m[0], v[j].x);
        m[1] = pk_absmax(m[1], v[j].y);
        m[2] = pk_absmax(m[2], v[j].z);
        m[3] = pk_absmax(m[3], v[j].w);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) m[i] = pk_absmax_xor<32>(pk_absmax_xor<16>(m[i]));
    float factor[8];
    uint32_t bytes_lo = 0, bytes_hi = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t mag = (m[e >> 1] >> ((e & 1) * 16)) & 0x7FFFu;
        int byte = 0;
        if (mag != 0) {
            const int ef = (int)(mag >> 7);
            const int fl = ef > 0 ? ef - 127 : (31 - __builtin_clz(mag)) - 133;
            byte = fl - EMAX + 127;
            byte = byte < 0 ? 0 : (byte > 254 ? 254 : byte);
        }
        factor[e] = __uint_as_float((uint32_t)(254 - byte) << 23);
        if (e < 4) bytes_lo |= (uint32_t)byte << (8 * e); else bytes_hi |= (uint32_t)byte << (8 * (e - 4));
    }
    if ((ty & 3) == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            ebytes[(tx * 8 + e) * 4 + (ty >> 2)] = (uint8_t)(((e < 4 ? bytes_lo : bytes_hi) >> (8 * (e & 3))) & 0xFFu);
    }

    uint32_t w[8][2];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint2 b = cast8<FMT>(v[j], factor);
        w[j][0] = b.x;
        w[j][1] = b.y;
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        uint32_t lo[4], hi[4];
        transpose4x4_bytes(w[0][h], w[1][h], w[2][h], w[3][h], lo);
        transpose4x4_bytes(w[4][h], w[5][h], w[6][h], w[7][h], hi);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int cc = tx * 8 + h * 4 + i;  // output row inside the tile
            tile[cc * SLOTS + (ty ^ (2 * (tx & 7)))] = make_uint2(lo[i], hi[i]);
        }
    }
    __syncthreads();

    const uint4* tile16 = reinterpret_cast<const uint4*>(tile);
    constexpr int ROWS_PER_IT = 256 / PARTS;
#pragma unroll
    for (int it = 0; it < 128 / ROWS_PER_IT; ++it) {
        const int cc = it * ROWS_PER_IT + (threadIdx.x / PARTS), p = threadIdx.x % PARTS;
        const int64_t oc = c0 + cc, orow = r0 + p * 16;
        if (oc >= cols || orow >= rows) continue;      // rows % 32 == 0: a 16-byte piece is inside or outside
        store_stream(qt + oc * ld_t + orow, tile16[cc * PARTS + (p ^ ((cc >> 3) & 7))]);
    }
    if (threadIdx.x < 128 && c0 + threadIdx.x < cols) {
        uint8_t* dst = et + e8_off(c0 + threadIdx.x, r0 / 32, ld_e);
        const uint32_t four = reinterpret_cast<const uint32_t*>(ebytes)[threadIdx.x];
        if (r0 + TR <= rows) {
            *reinterpret_cast<uint32_t*>(dst) = four;   // ld_e % 4 == 0 and r0 / 32 % 4 == 0
        } else {
            for (int b = 0; r0 + 32 * b < rows; ++b) dst[b] = (uint8_t)((four >> (8 * b)) & 0xFFu);
        }
    }
    if constexpr (ROWS_TOO) {
        // the tile's 128 x 4 row-direction scale bytes, one dword per row (threads 128..255)
        const int rr = (int)threadIdx.x - 128;
        if (rr >= 0 && r0 + rr < rows) {
            uint8_t* dst = e_row + e8_off(r0 + rr, c0 / 32, ld_er);
            const uint32_t four = reinterpret_cast<const uint32_t*>(rbytes)[rr];
            if (c0 + 128 <= cols) {
                *reinterpret_cast<uint32_t*>(dst) = four;   // ld_er % 4 == 0 and c0 / 32 % 4 == 0
            } else {
                for (int b = 0; c0 + 32 * b < cols; ++b) dst[b] = (uint8_t)((four >> (8 * b)) & 0xFFu);
            }
        }
    }
}

// Blockwise FP8 of the TRANSPOSED matrix, written transposed: qt [cols, rows] and et [cols, rows / 32] are what
// block_quant_* gives on x^T, i.e. the contraction-contiguous operands of the backward products.  rows % 128 == 0.
//   SQUARE = false: tiles of 1 x 128 of x^T = 128 rows x 1 column of x (the activation-like operands of
//     dW = dY^T X, whose contraction runs down the rows of dY and X): the column maxima over the tile's 128 rows
//     come from the 8 rows of a thread, two cross-lane steps (4 thread rows of a wavefront) and LDS (4 wavefronts).
//   SQUARE = true: blocks of 128 x 128 (the weight in dX = dY W; the same numbers as the forward's blocks of W).
// Tile scheme, byte transpose, swizzled LDS tile and 128-bit streaming stores as in the transposing cast.
// ROWS_TOO (with SQUARE = false, cols % 128 == 0): the same read also yields the tiles of 1 x 128 ALONG the rows
// of x (q_row [rows, cols], e_row [rows, cols / 32]): the 16 threads that hold a row of the tile combine their
// maxima with four cross-lane steps.  The gradient, needed in both orientations by the backward, then costs
// 4 bytes of HBM traffic per element instead of 6.
template <int FMT, bool SQUARE, bool ROWS_TOO = false>
__global__ __launch_bounds__(256) void block_quant_t_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                             int64_t ld, uint8_t* __restrict__ qt, int64_t ld_t,
                                                             uint8_t* __restrict__ et, int64_t ld_e, int nx, int ny,
                                                             uint8_t* __restrict__ q_row = nullptr, int64_t ld_row = 0,
                                                             uint8_t* __restrict__ e_row = nullptr, int64_t ld_er = 0) {
    constexpr int TR = 128, SLOTS = TR / 8, PARTS = TR / 16;
    __shared__ __attribute__((aligned(16))) uint2 tile[128 * SLOTS];
    __shared__ uint32_t red[4][16][4];
    __shared__ uint8_t ebytes[128];                                   // scale byte of each column of the tile
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4, wave = threadIdx.x >> 6;
    constexpr int PX = 16, PY = 16;
    const int pxc = (nx + PX - 1) / PX;
    const int patch = blockIdx.x / (PX * PY), within = blockIdx.x % (PX * PY);
    const int bx = (patch % pxc) * PX + within % PX, by = (patch / pxc) * PY + within / PX;
    if (bx >= nx || by >= ny) return;
    const int64_t r0 = (int64_t)bx * TR, c0 = (int64_t)by * 128;
    const int64_t c = c0 + tx * 8;

    uint4 v[8];
    uint32_t m[4] = {0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int64_t r = r0 + ty * 8 + j;                            // rows % 128 == 0: inside the matrix
        v[j] = c + 8 <= cols ? load_stream(x + r * ld + c) : make_uint4(0, 0, 0, 0);   // cols % 8 == 0
        m[0] = pk_absmax(m[0], v[j].x);
        m[1] = pk_absmax(m[1], v[j].y);
        m[2] = pk_absmax(m[2], v[j].z);
        m[3] = pk_absmax(m[3], v[j].w);
    }
    if constexpr (ROWS_TOO) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            uint32_t mr = wave_max_u32<16>(pk_fold(pk_absmax4(0u, v[j])));
            uint32_t byte;
            const float sr = pow2_block_scale<FMT>(mr, byte);
            const int64_t r = r0 + ty * 8 + j;
            store_stream(q_row + r * ld_row + c, cast8<FMT>(v[j], sr));                   // cols % 128 == 0: inside
            if (tx == 0) *reinterpret_cast<uint32_t*>(e_row + e8_off(r, c0 >> 5, ld_er)) = byte * 0x01010101u;
        }
    }
    float factor[8];
    if constexpr (SQUARE) {
        uint32_t a = pk_absmax(pk_absmax(m[0], m[1]), pk_absmax(m[2], m[3]));
        a = wave_max_u32<64>(pk_fold(a));
        if ((threadIdx.x & 63) == 0) red[wave][0][0] = a;
        __syncthreads();
        a = red[0][0][0];
#pragma unroll
        for (int w_ = 1; w_ < 4; ++w_) a = red[w_][0][0] > a ? red[w_][0][0] : a;
        uint32_t byte;
        const float s = pow2_block_scale<FMT>(a, byte);
#pragma unroll
        for (int e = 0; e < 8; ++e) factor[e] = s;
        if (threadIdx.x < 128) ebytes[threadIdx.x] = (uint8_t)byte;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) m[i] = pk_absmax_xor<32>(pk_absmax_xor<16>(m[i]));
        if ((threadIdx.x & 63) < 16) {
#pragma unroll
            for (int i = 0; i < 4; ++i) red[wave][tx][i] = m[i];
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t a = red[0][tx][i];
#pragma unroll
            for (int w_ = 1; w_ < 4; ++w_) a = pk_absmax(a, red[w_][tx][i]);
            m[i] = a;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            uint32_t byte;
            factor[e] = pow2_block_scale<FMT>((m[e >> 1] >> ((e & 1) * 16)) & 0x7FFFu, byte);
            if (ty == 0) ebytes[tx * 8 + e] = (uint8_t)byte;
        }
    }

    uint32_t w[8][2];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint2 b = cast8<FMT>(v[j], factor);
        w[j][0] = b.x;
        w[j][1] = b.y;
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        uint32_t lo[4], hi[4];
        transpose4x4_bytes(w[0][h], w[1][h], w[2][h], w[3][h], lo);
        transpose4x4_bytes(w[4][h], w[5][h], w[6][h], w[7][h], hi);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int cc = tx * 8 + h * 4 + i;  // output row inside the tile
            tile[cc * SLOTS + (ty ^ (2 * (tx & 7)))] = make_uint2(lo[i], hi[i]);
        }
    }
    __syncthreads();

    const uint4* tile16 = reinterpret_cast<const uint4*>(tile);
    constexpr int ROWS_PER_IT = 256 / PARTS;
#pragma unroll
    for (int it = 0; it < 128 / ROWS_PER_IT; ++it) {
        const int cc = it * ROWS_PER_IT + (threadIdx.x / PARTS), p = threadIdx.x % PARTS;
        const int64_t oc = c0 + cc;
        if (oc >= cols) continue;
        store_stream(qt + oc * ld_t + r0 + p * 16, tile16[cc * PARTS + (p ^ ((cc >> 3) & 7))]);
    }
    if (threadIdx.x < 128 && c0 + threadIdx.x < cols)                 // ld_e % 4 == 0 and (r0 / 32) % 4 == 0
        *reinterpret_cast<uint32_t*>(et + e8_off(c0 + threadIdx.x, r0 / 32, ld_e)) = (uint32_t)ebytes[threadIdx.x] * 0x01010101u;
}

// block_rows: blocks of x^T, 1 (tiles of 1 x 128 of x^T) or 128 (128 x 128); rows % 128 == 0, cols % 8 == 0.
// q_row != nullptr (block_rows == 1, cols % 128 == 0): also the tiles of 1 x 128 along the rows of x.
hipError_t launch_block_quant_t(const void* x, int64_t rows, int64_t cols, int64_t ld, int block_rows, int fmt, uint8_t* qt,
                                int64_t ld_t, uint8_t* et, int64_t ld_e, hipStream_t st, uint8_t* q_row, int64_t ld_row,
                                uint8_t* e_row, int64_t ld_er) {
    if (rows == 0 || cols == 0) return hipSuccess;
    const int64_t gx = (cols + 127) / 128, gy = rows / 128;
    const int64_t total = ((gy + 15) / 16) * ((gx + 15) / 16) * 256;
    if (total > 0x7FFFFFFF) return hipErrorInvalidValue;
    const uint16_t* xp = static_cast<const uint16_t*>(x);
#define FP8K_BQT(FMT, SQ, RT) block_quant_t_kernel<FMT, SQ, RT><<<dim3((unsigned)total), dim3(256), 0, st>>>(xp, rows, cols, ld, qt, ld_t, et, ld_e, (int)gy, (int)gx, q_row, ld_row, e_row, ld_er)
    if (q_row != nullptr) {
        if (block_rows != 1 || cols % 128 != 0) return hipErrorInvalidValue;
        if (fmt == FMT_E4M3FN) FP8K_BQT(FMT_E4M3FN, false, true); else FP8K_BQT(FMT_E5M2, false, true);
    } else if (fmt == FMT_E4M3FN) { if (block_rows == 128) FP8K_BQT(FMT_E4M3FN, true, false); else FP8K_BQT(FMT_E4M3FN, false, false); }
    else { if (block_rows == 128) FP8K_BQT(FMT_E5M2, true, false); else FP8K_BQT(FMT_E5M2, false, false); }
#undef FP8K_BQT
    return hipGetLastError();
}

hipError_t launch_mx_quant_t(const void* x, int64_t rows, int64_t cols, int64_t ld, int fmt, uint8_t* qt, int64_t ld_t,
                             uint8_t* et, int64_t ld_e, uint8_t* q_row, int64_t ld_row, uint8_t* e_row, int64_t ld_er,
                             hipStream_t st) {
    if (rows == 0 || cols == 0) return hipSuccess;
    const int64_t gx = (cols + 127) / 128, gy = (rows + 127) / 128;
    const int64_t total = ((gy + 15) / 16) * ((gx + 15) / 16) * 256;
    if (total > 0x7FFFFFFF) return hipErrorInvalidValue;
    const uint16_t* xp = static_cast<const uint16_t*>(x);
#define FP8K_MXT(FMT, R) mx_quant_t_kernel<FMT, R><<<dim3((unsigned)total), dim3(256), 0, st>>>(xp, rows, cols, ld, qt, ld_t, et, ld_e, q_row, ld_row, e_row, ld_er, (int)gy, (int)gx)
    if (fmt == FMT_E4M3FN) { if (q_row) FP8K_MXT(FMT_E4M3FN, true); else FP8K_MXT(FMT_E4M3FN, false); }
    else { if (q_row) FP8K_MXT(FMT_E5M2, true); else FP8K_MXT(FMT_E5M2, false); }
#undef FP8K_MXT
    return hipGetLastError();
}

}  // namespace fp8k
