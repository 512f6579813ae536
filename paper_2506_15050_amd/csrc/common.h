// Internal helpers shared by the HIP translation units of libtppo (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tppo.h"

#define TPPO_VERSION 100

namespace tppo {

constexpr int kWave = 64;

static inline bool is_aligned(const void* p, size_t a) {
    return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0;
}

static constexpr size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static inline int launch_result() {
    return hipGetLastError() == hipSuccess ? TPPO_OK : TPPO_ERR_LAUNCH;
}

__device__ __forceinline__ void set_status(int32_t* status, int32_t bit) {
    if (status) atomicOr(status, bit);
}

// Loads of wave-uniform values through the scalar data cache (read-only data written before the launch).  Cheap
// when the line is there (kernel arguments, a header every wavefront reads); a MISS was measured at 4000-6000
// cycles with thousands of wavefronts in flight, several times a vector load's latency -- so per-tile data that
// a wavefront waits for goes through vector loads, and scalar loads are for what is fetched well ahead.
__device__ __forceinline__ int32_t load_uniform(const int32_t* p) {
    return *(const int32_t __attribute__((address_space(4)))*)(p);
}
__device__ __forceinline__ float load_uniform(const float* p) {
    return *(const float __attribute__((address_space(4)))*)(p);
}
__device__ __forceinline__ long long load_uniform(const long long* p) {
    return *(const long long __attribute__((address_space(4)))*)(p);
}

// Compute units of the current device (asked once per device; <= 0 when the runtime cannot say).
int device_compute_units();

// largest s in [lo, hi] with off[s] <= p  (off non-decreasing, off[lo] <= p)
__device__ __forceinline__ int find_segment(const int32_t* off, int lo, int hi, int p) {
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (off[mid] <= p) lo = mid; else hi = mid - 1;
    }
    return lo;
}

}  // namespace tppo
