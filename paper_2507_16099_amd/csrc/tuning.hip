// Host-only: the tuning / test switches (see tuning.hpp).
#include "tuning.hpp"

#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>

namespace fp8k {
namespace {
const char* const kNames[KNOB_COUNT] = {"GEMM_VARIANT", "SNAKE_HALF", "SKINNY_NW", "SKINNY_DMA",
                                        "MX_VARIANT",   "MX_SLAB",    "BF16_VARIANT", "GEMM_STREAM", "GEMM_TILE_M",
                                        "GEMM_BIG_FROM", "PAIRS", "DECODE_FUSED"};
std::atomic<int> g_value[KNOB_COUNT];
std::once_flag g_once;

void read_environment() {
    for (int i = 0; i < KNOB_COUNT; ++i) {
        const std::string var = std::string("FP8MI355_") + kNames[i];
        const char* e = std::getenv(var.c_str());
        g_value[i].store((e && *e) ? std::atoi(e) : -1, std::memory_order_relaxed);
    }
}
}  // namespace

int knob(Knob k) {
    std::call_once(g_once, read_environment);
    return g_value[k].load(std::memory_order_relaxed);
}

bool set_knob(const char* name, int value) {
    std::call_once(g_once, read_environment);
    if (!name) return false;
    for (int i = 0; i < KNOB_COUNT; ++i)
        if (std::strcmp(name, kNames[i]) == 0) {
            g_value[i].store(value, std::memory_order_relaxed);
            return true;
        }
    return false;
}

int compute_units() {
    static CachedInt cus;
    return cus.get([] {
        int dev = 0, n = 0;
        return (hipGetDevice(&dev) == hipSuccess &&
                hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess) ? n : 0;
    });
}

}  // namespace fp8k

// Test and tuning aid, not part of the public header: forces a switch for the rest of the process
// (value -1 restores the default).  Returns 0, or -3 (FP8_ERR_ENUM) for an unknown name.
extern "C" int fp8_internal_set_knob(const char* name, int value) { return fp8k::set_knob(name, value) ? 0 : -3; }
