// Optional device-side stage clock for studying where a kernel's time goes (builds with
// -DSVIP_STAGE_CLOCK only; the product library is built without it and STAGE() is empty).
// STAGE(i) lets thread 0 of a workgroup note the 100 MHz wall clock at stage i < 8 (STAGE_WHERE the
// hardware ids of the compute unit it runs on); the host reads the
// notes back with svip_bench_stage_clock.
#pragma once
#include <hip/hip_runtime.h>

#ifdef SVIP_STAGE_CLOCK
namespace svip {
constexpr int STAGE_SLOTS = 16, STAGE_GROUPS = 16384;     // slots 8, 9: where the workgroup ran (HW_ID, XCC_ID)
__device__ unsigned long long g_stage_clock[STAGE_GROUPS * STAGE_SLOTS];
}
#define STAGE(i)                                                                                     \
    do {                                                                                             \
        if (threadIdx.x == 0 && blockIdx.x < svip::STAGE_GROUPS)                                      \
            svip::g_stage_clock[blockIdx.x * svip::STAGE_SLOTS + (i)] = wall_clock64();               \
    } while (0)
#define STAGE_WHERE()                                                                                \
    do {                                                                                             \
        if (threadIdx.x == 0 && blockIdx.x < svip::STAGE_GROUPS) {                                    \
            svip::g_stage_clock[blockIdx.x * svip::STAGE_SLOTS + 8] = __builtin_amdgcn_s_getreg(63492); \
            svip::g_stage_clock[blockIdx.x * svip::STAGE_SLOTS + 9] = __builtin_amdgcn_s_getreg(63508); \
        }                                                                                            \
    } while (0)
// STAGE_LOADED(i): the same note, taken once every outstanding load of the thread has arrived
#define STAGE_LOADED(i)                                                                              \
    do {                                                                                             \
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                                             \
        STAGE(i);                                                                                    \
    } while (0)
#else
#define STAGE_LOADED(i) do { } while (0)
#define STAGE(i) do { } while (0)
#define STAGE_WHERE() do { } while (0)
#endif
