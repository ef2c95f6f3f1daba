// Optional phase timestamps for timing builds (-DMORPH_TIMING; build.py --timing writes
// libmorph_timing.so, profile_phases.py reads it): thread 0 of every workgroup stores the shader
// clock and the 100 MHz wall clock at a few points of a kernel.  Compiled out of the product library.
#pragma once
#include <hip/hip_runtime.h>

#ifdef MORPH_TIMING
namespace morph {
constexpr int kTickBlocks = 8192, kTickSlots = 8;
static __device__ unsigned long long g_ticks[kTickBlocks * kTickSlots * 2];   // one copy per translation unit
}
#define MORPH_TICK(i)                                                                          \
    do {                                                                                       \
        const unsigned morph_tick_wg = blockIdx.y * gridDim.x + blockIdx.x;                    \
        if (threadIdx.x == 0 && morph_tick_wg < (unsigned)morph::kTickBlocks) {                \
            morph::g_ticks[morph_tick_wg * 16 + 2 * (i)]     = __builtin_readcyclecounter();   \
            morph::g_ticks[morph_tick_wg * 16 + 2 * (i) + 1] = wall_clock64();                 \
        }                                                                                      \
    } while (0)
#define MORPH_NOTE(i, value)                                                                   \
    do {                                                                                       \
        const unsigned morph_tick_wg = blockIdx.y * gridDim.x + blockIdx.x;                    \
        if (threadIdx.x == 0 && morph_tick_wg < (unsigned)morph::kTickBlocks) {                \
            morph::g_ticks[morph_tick_wg * 16 + 2 * (i)]     = (unsigned long long)(value);    \
            morph::g_ticks[morph_tick_wg * 16 + 2 * (i) + 1] = wall_clock64();                 \
        }                                                                                      \
    } while (0)
#define MORPH_TICK_EXPORTS(name)                                                               \
    extern "C" int morph_debug_read_##name(unsigned long long* host_out, int n)                \
    {                                                                                          \
        return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(morph::g_ticks), sizeof(unsigned long long) * n); \
    }                                                                                          \
    extern "C" int morph_debug_clear_##name()                                                  \
    {                                                                                          \
        static unsigned long long z[morph::kTickBlocks * morph::kTickSlots * 2];               \
        return (int)hipMemcpyToSymbol(HIP_SYMBOL(morph::g_ticks), z, sizeof(z));               \
    }
#else
#define MORPH_TICK(i) do { } while (0)
#define MORPH_NOTE(i, value) do { } while (0)
#define MORPH_TICK_EXPORTS(name)
#endif
