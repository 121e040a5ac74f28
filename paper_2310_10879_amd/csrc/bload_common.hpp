// Shared host/device helpers of the BLoad library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bload.h"

namespace bload {

constexpr int kWave = 64;          // CDNA wavefront width
constexpr int kThreads = 256;      // workgroup size used by every kernel (4 waves)

// Last failing HIP call of this thread (reported by bload_last_hip_error()).
extern thread_local int g_last_hip_error;

inline bool hip_ok(hipError_t e)
{
    if (e == hipSuccess) return true;
    g_last_hip_error = (int)e;
    return false;
}

// Status of the launch that was just enqueued.
inline bload_status launch_status()
{
    return hip_ok(hipGetLastError()) ? BLOAD_OK : BLOAD_EHIP;
}

inline bool aligned_to(const void* p, size_t a)
{
    return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0;
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

inline size_t round_up(size_t a, size_t b) { return (a + b - 1) / b * b; }

// ---- device helpers -------------------------------------------------------

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }
__device__ __forceinline__ int wave_id() { return (int)(threadIdx.x >> 6); }

// Streaming 16-byte accesses: the packer touches every payload byte once, so
// it asks the caches not to keep them.
typedef unsigned int vec16 __attribute__((ext_vector_type(4)));   // 16 bytes

__device__ __forceinline__ vec16 load_stream(const vec16* p)
{
    return __builtin_nontemporal_load(p);
}
__device__ __forceinline__ void store_stream(vec16* p, vec16 v)
{
    __builtin_nontemporal_store(v, p);
}

// The hardware deals consecutive workgroups round-robin to the 8 XCDs (each with
// its own L2 and its own path to HBM).  This maps workgroup b of n to a work item
// so that every XCD walks one contiguous eighth of the items: b -> (XCD b % 8,
// step b / 8) -> first item of that XCD + step.  A bijection of [0, n) for any n.
constexpr uint32_t kXcds = 8;
__device__ __forceinline__ uint32_t xcd_contiguous(uint32_t b, uint32_t n)
{
    const uint32_t full = n / kXcds, rem = n % kXcds;
    const uint32_t x = b % kXcds, y = b / kXcds;
    return x * full + min(x, rem) + y;
}

}  // namespace bload
