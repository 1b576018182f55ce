// Phase timers of debug builds (-DTOPLOC_TIMING); they compile to nothing otherwise.
#pragma once
#include <hip/hip_runtime.h>

#ifdef TOPLOC_TIMING
// debug builds only: wall-clock ticks (100 MHz) per phase, summed over workgroups by lane 0
__device__ unsigned long long g_toploc_ticks[16];
#define TOPLOC_TICK_BEGIN(name) const long long tick_##name = wall_clock64()
#define TOPLOC_TICK_END(name, slot) \
    do { if (threadIdx.x == 0) atomicAdd(&g_toploc_ticks[slot], (unsigned long long)(wall_clock64() - tick_##name)); } while (0)
#else
#define TOPLOC_TICK_BEGIN(name)
#define TOPLOC_TICK_END(name, slot)
#endif
