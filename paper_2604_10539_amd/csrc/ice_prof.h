// In-kernel time stamps for performance work.  NOT part of the product build: ice_internal.h
// includes this file only when the library is compiled with -DICE_PROF (no committed build step
// does); without it every ICE_*STAMP macro is empty and no ice_debug_prof_* symbol exists.
// Each kernel file gets stamp arrays of its own (static device arrays) and names its export with
// ICE_PROF_EXPORT(symbol): int symbol(long long *host, int n) copies the first n stamps (n <= 64)
// and, behind them when n > 64, per-unit stamps (4 per unit, 1024 units).
#pragma once
#include <hip/hip_runtime.h>

namespace ice {
namespace prof {
static __device__ long long stamps[64];
static __device__ long long wave_stamps[128];
static __device__ long long unit_stamps[4 * 1024];
}  // namespace prof
}  // namespace ice

// decode kernels: thread 0 of unit 0 (`u` in scope); per unit: start, end of scoring, of selection, end
#define ICE_STAMP(i) do { if (threadIdx.x == 0 && u == 0) ice::prof::stamps[i] = wall_clock64(); } while (0)
#define ICE_USTAMP(i) do { if (threadIdx.x == 0 && u < 1024) ice::prof::unit_stamps[4 * u + (i)] = wall_clock64(); } while (0)
#define ICE_PROF_ATTEND 1
// build kernels: thread 0 of workgroup (0, *, 0); per wave of that workgroup for tile 1
#define ICE_BSTAMP(i) do { if (threadIdx.x == 0 && blockIdx.x == 0 && blockIdx.z == 0) ice::prof::stamps[i] = wall_clock64(); } while (0)
#define ICE_WSTAMP(t, i) do { if ((t) == 1 && (threadIdx.x & 63) == 0 && blockIdx.x == 0 && blockIdx.z == 0) { ice::prof::wave_stamps[(threadIdx.x >> 6) * 8 + (i)] = wall_clock64(); ice::prof::wave_stamps[64 + (threadIdx.x >> 6) * 8 + (i)] = clock64(); } } while (0)
// hierarchical kernel: thread 0 of workgroup 0
#define ICE_HSTAMP(i) do { if (threadIdx.x == 0 && blockIdx.x == 0) ice::prof::stamps[i] = wall_clock64(); } while (0)

#define ICE_PROF_EXPORT(symbol)                                                                              \
    extern "C" int symbol(long long *host, int n) {                                                          \
        int rc = (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(ice::prof::stamps), sizeof(long long) * (n < 64 ? n : 64)); \
        if (rc == 0 && n > 64 && n <= 64 + 128)                                                              \
            rc = (int)hipMemcpyFromSymbol(host + 64, HIP_SYMBOL(ice::prof::wave_stamps), sizeof(long long) * (n - 64)); \
        if (rc == 0 && n > 64 + 128)                                                                         \
            rc = (int)hipMemcpyFromSymbol(host + 64, HIP_SYMBOL(ice::prof::unit_stamps), sizeof(long long) * (n - 64)); \
        return rc;                                                                                           \
    }
