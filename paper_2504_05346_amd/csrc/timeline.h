// Optional instrumentation of the block update (k_update) and of the tile product inside it:
// wall-clock timestamps (100 MHz) per workgroup, compiled in only with -DTHANOS_TIMELINE
// (libthanos_timeline.so, a diagnostic build used by timeline_probe.py; the product library is
// built without it and TL_MARK is empty there).
//
// Slots of a workgroup (kTlSlots per workgroup, workgroups 0 .. kTlWgs-1 of the selected launch):
//   0 start | 1 product done | 2 tile staged in LDS | 3 old tile values have arrived |
//   4 row pass done (new values stored) | 5 end of the kernel
//   8 + 4 it + {0, 1}: producer wavefront 4, slab it: fill starts / next loads are out
//   8 + 4 it + {2, 3}: multiplying wavefront 0, slab it: multiply starts / ends
// A launch is recorded when its grid has exactly the selected number of workgroups
// (thanos_timeline_select) -- the caller picks a grid size that only the launch of interest has.
#pragma once
#ifdef THANOS_TIMELINE
#include <hip/hip_runtime.h>
namespace thanos {
constexpr int kTlSlots = 80;
constexpr int kTlWgs = 4096;
static __device__ unsigned long long g_timeline[kTlWgs * kTlSlots];
static __constant__ int g_timeline_grid;  // constant space: read once per kernel, not per mark
}  // namespace thanos
#define TL_MARK(slot)                                                                         \
  do {                                                                                        \
    if ((int)gridDim.x == thanos::g_timeline_grid && (threadIdx.x & 63) == 0 &&               \
        blockIdx.x < thanos::kTlWgs && (slot) < thanos::kTlSlots)                             \
      thanos::g_timeline[blockIdx.x * thanos::kTlSlots + (slot)] = wall_clock64();            \
  } while (0)
#define TL_WAIT_LOADS() __builtin_amdgcn_s_waitcnt(0x0F70) /* vmcnt(0): old values are here */
#else
#define TL_MARK(slot) \
  do {                \
  } while (0)
#define TL_WAIT_LOADS() \
  do {                  \
  } while (0)
#endif
