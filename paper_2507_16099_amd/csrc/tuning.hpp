// Tuning and test switches of the launchers, and the small pieces of cached host state they share.
//
// Every switch has a measured default.  A switch can be preset through the environment variable
// FP8MI355_<NAME>; the environment is read ONCE per process, on the first use of any switch, never on a launch
// path afterwards.  After that only set_knob changes a value (exported as fp8_internal_set_knob: the tests use
// it to force every kernel form).  -1 means "not set: take the default".  All state here is atomic.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>

namespace fp8k {

enum Knob {
    KNOB_GEMM_VARIANT = 0,  // 0 = 128x128 tiles, 4 = LDS-DMA 256x256 kernel, 5 = few-row kernel, 6 / 7 = 64x64 / 128x128 with loads ahead
    KNOB_SNAKE_HALF,        // 0 = no half tiles for a partly filled last round
    KNOB_SKINNY_NW,         // few-row kernel: 1, 2 or 4 column groups of 16 per wavefront
    KNOB_SKINNY_DMA,        // few-row kernel: 0 = operands straight into registers, 1 = through LDS
    KNOB_MX_VARIANT,        // MX GEMM: 0 = register-staged kernel, 1 = LDS-DMA kernel
    KNOB_MX_SLAB,           // 0 = plain scale rows inside the MX / blockwise linear calls
    KNOB_BF16_VARIANT,      // bfloat16 dW: 0 = register-staged kernel, 1 = LDS-DMA kernel
    KNOB_GEMM_STREAM,       // persistent LDS-DMA kernel: 0 = never, 2 = wherever it fits, >= 8 = wherever it fits, with that many workgroups
    KNOB_GEMM_TILE_M,       // persistent kernel: 256, 224 or 192 forces the tile height
    KNOB_GEMM_BIG_FROM,     // number of 128 x 128 tiles from which a product goes to the 256 x 256 kernels
    KNOB_PAIRS,             // 0 = no shared launches: every tensor of a linear step quantized, every product launched, by itself
    KNOB_DECODE_FUSED,      // few tokens against a quantized weight: 0 = activation quantization always a launch of its own, 2 = inside the product wherever that kernel applies
    KNOB_COUNT
};

int knob(Knob k);
// name without the FP8MI355_ prefix; returns false for an unknown name
bool set_knob(const char* name, int value);

// number of compute units of the current device (0 if the query fails); cached
int compute_units();

// hipFuncSetAttribute(MaxDynamicSharedMemorySize) once per kernel: one object per kernel instantiation
// (a function-local static of the launcher).  The call is idempotent, so two threads racing through it both succeed.
struct DynamicLdsOnce {
    std::atomic<int> done{0};
    hipError_t ensure(const void* kernel, int bytes) {
        if (done.load(std::memory_order_acquire)) return hipSuccess;
        const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e == hipSuccess) done.store(1, std::memory_order_release);
        return e;
    }
};

// a value computed once per call site (e.g. the number of resident blocks of a kernel); racing threads compute the same value
struct CachedInt {
    std::atomic<int> v{-1};
    template <class F> int get(F compute) {
        int x = v.load(std::memory_order_acquire);
        if (x < 0) { x = compute(); v.store(x, std::memory_order_release); }
        return x;
    }
};

}  // namespace fp8k
