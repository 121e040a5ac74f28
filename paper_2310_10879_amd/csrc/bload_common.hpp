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

// 64 bytes of pinned host memory per calling thread, made at the thread's first call and kept
// until the process ends; null if it cannot be had.  An entry point whose caller waits for a few
// numbers lets its last kernel write them there, so that only the wait for the stream follows
// the launches (a copy back from device memory costs about 9 us more per call).  Only for plain
// stores by one kernel: nothing that kernels read back or update atomically.
inline void* host_result_buffer()
{
    static thread_local void* mem = nullptr;
    static thread_local bool tried = false;
    if (!tried) {
        tried = true;
        if (hipHostMalloc(&mem, 64, hipHostMallocPortable) != hipSuccess) {
            mem = nullptr;
            (void)hipGetLastError();
        }
    }
    return mem;
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

// ---- moves between the lanes of a wavefront without LDS traffic (DPP) --------------
//
// dpp_move<CTRL, ROW_MASK>(v, idle): every lane reads v of the lane that CTRL names; a lane
// whose source does not exist, or whose row of 16 lanes is not in ROW_MASK, gets `idle`.
constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118;
constexpr int kDppRowBcast15 = 0x142;   // lane 15 of each row -> every lane of the next row
constexpr int kDppRowBcast31 = 0x143;   // lane 31 -> every lane of rows 2 and 3
constexpr int kDppWaveShr1 = 0x138;     // lane l reads lane l - 1
constexpr int kDppWaveShl1 = 0x130;     // lane l reads lane l + 1

template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ uint32_t dpp_move(uint32_t v, uint32_t idle)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)idle, (int)v, CTRL, ROW_MASK, 0xF, false);
}
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ int32_t dpp_move(int32_t v, int32_t idle)
{
    return __builtin_amdgcn_update_dpp(idle, v, CTRL, ROW_MASK, 0xF, false);
}
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_move(float v, float idle)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(idle), __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ long long dpp_move(long long v, long long idle)
{
    const uint32_t lo = dpp_move<CTRL, ROW_MASK>((uint32_t)v, (uint32_t)idle);
    const uint32_t hi = dpp_move<CTRL, ROW_MASK>((uint32_t)((unsigned long long)v >> 32),
                                                 (uint32_t)((unsigned long long)idle >> 32));
    return (long long)(((unsigned long long)hi << 32) | lo);
}

// Inclusive scan over the 64 lanes of a wavefront: x[l] = op(x[0], ..., x[l]).  `Move` gives
// the value of another lane (a dpp_move per component, with the operation's identity for
// lanes that have no source); op(left, right) must be associative.  Six steps: distances 1, 2,
// 4, 8 inside rows of 16 lanes, then each row's last lane into the next row, then lane 31
// into the upper half.
template <typename T, typename Op, typename Move>
__device__ __forceinline__ T wave_scan(T x, Op op, Move move)
{
    x = op(move.template at<kDppRowShr1, 0xF>(x), x);
    x = op(move.template at<kDppRowShr2, 0xF>(x), x);
    x = op(move.template at<kDppRowShr4, 0xF>(x), x);
    x = op(move.template at<kDppRowShr8, 0xF>(x), x);
    x = op(move.template at<kDppRowBcast15, 0xA>(x), x);
    x = op(move.template at<kDppRowBcast31, 0xC>(x), x);
    return x;
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
