// Bounds checks of the debug build (-DKVR_BOUNDS, linked into libkvr_bounds.so).
//
// The long-head kernels index LDS tables, gathered rows and output lists with values they
// compute from the data (pool slots from ballots, list positions, token indices read back from
// tables, triangle addresses of the race).  In the debug build every such index goes through
// kvr_ix(index, limit, id): an index outside [0, limit) is recorded (the largest id seen, one
// counter per source file) and clamped, so that the debug build neither traps nor faults; the
// product build compiles kvr_ix to its first argument.  kvr_debug_bounds_violation() of the
// C-ABI reads the counters.  The ids are <file number> * 100 + <site>, listed where they are used.
#pragma once
#include <hip/hip_runtime.h>

namespace kvr {

#ifdef KVR_BOUNDS
static __device__ unsigned int g_bounds_bad = 0;

__device__ __forceinline__ int kvr_ix(int i, int limit, unsigned int id) {
  if (i < 0 || i >= limit) {
    atomicMax(&g_bounds_bad, id);
    return i < 0 ? 0 : limit - 1;
  }
  return i;
}

// The same for an index that only the lanes with `used` go on to use.
__device__ __forceinline__ int kvr_ix_if(bool used, int i, int limit, unsigned int id) {
  return used ? kvr_ix(i, limit, id) : i;
}

// (synchronises the device: debug only)
static inline unsigned int bounds_fetch_and_clear() {
  unsigned int v = 0, z = 0;
  if (hipMemcpyFromSymbol(&v, HIP_SYMBOL(g_bounds_bad), sizeof(v)) != hipSuccess) return 0xffffffffu;
  if (hipMemcpyToSymbol(HIP_SYMBOL(g_bounds_bad), &z, sizeof(z)) != hipSuccess) return 0xffffffffu;
  return v;
}
#define KVR_BOUNDS_TU(name) \
  unsigned int bounds_bad_##name() { return bounds_fetch_and_clear(); }
#else
__device__ __forceinline__ int kvr_ix(int i, int, unsigned int) { return i; }
__device__ __forceinline__ int kvr_ix_if(bool, int i, int, unsigned int) { return i; }
#define KVR_BOUNDS_TU(name) \
  unsigned int bounds_bad_##name() { return 0u; }
#endif

}  // namespace kvr
