// Streaming kernels without any of the packer's logic: what an access pattern alone reaches on
// this GPU.  See include/bload_yardsticks.h for what each one moves and why it has that shape.
#include "bload_yardsticks.h"

#include <hip/hip_runtime.h>

namespace {

typedef unsigned int vec16 __attribute__((ext_vector_type(4)));
constexpr int kThreads = 256;
constexpr unsigned kUnlikely = 0x12345678u;

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int launched()
{
    return hipGetLastError() == hipSuccess ? 0 : 6;
}

__global__ __launch_bounds__(kThreads) void ys_copy_kernel(const vec16* __restrict__ src, vec16* __restrict__ dst,
                                                           size_t n_vec)
{
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n_vec) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

__global__ __launch_bounds__(kThreads) void ys_read_kernel(const vec16* __restrict__ src, size_t n_vec,
                                                           unsigned* __restrict__ sink)
{
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n_vec) return;
    const vec16 x = __builtin_nontemporal_load(src + i);
    if ((x[0] ^ x[1] ^ x[2] ^ x[3]) == kUnlikely && x[0] == kUnlikely + 1u) *sink = x[1];
}

// workgroup b of n -> a tile, so that every XCD (the hardware deals workgroups round-robin to 8 of
// them) walks one contiguous eighth of the tiles
__device__ __forceinline__ unsigned xcd_contiguous(unsigned b, unsigned n)
{
    const unsigned full = n / 8u, rem = n % 8u, x = b % 8u, y = b / 8u;
    return x * full + (x < rem ? x : rem) + y;
}

__global__ __launch_bounds__(kThreads) void ys_token_pack_kernel(
    const vec16* __restrict__ src, vec16* __restrict__ payload, vec16* __restrict__ plane_a,
    vec16* __restrict__ plane_b, unsigned* __restrict__ flags_a, unsigned* __restrict__ flags_b,
    unsigned n_blocks, int padding_percent, int scattered)
{
    const unsigned tile = xcd_contiguous(blockIdx.x, gridDim.x);       // 256 quads of 4 slots
    const unsigned block = tile / 4u;
    const size_t q = (size_t)tile * kThreads + threadIdx.x;
    vec16 x = {~0u, ~0u, ~0u, ~0u};
    if ((int)(block % 100u) >= padding_percent) {
        unsigned from_block = block;
        if (scattered) from_block = (unsigned)(((unsigned long long)block * 0x9E3779B97F4A7C15ull >> 20) % n_blocks);
        x = __builtin_nontemporal_load(src + ((size_t)from_block * 4u + tile % 4u) * kThreads + threadIdx.x);
    }
    __builtin_nontemporal_store(x, payload + q);
    __builtin_nontemporal_store(x, plane_a + q);
    __builtin_nontemporal_store(x, plane_b + q);
    __builtin_nontemporal_store(x[0], flags_a + q);
    __builtin_nontemporal_store(x[1], flags_b + q);
}

template <int ROWS_PER_WAVE, bool WRITE>
__global__ __launch_bounds__(kThreads) void ys_rows_kernel(const vec16* __restrict__ src, vec16* __restrict__ dst,
                                                           long long n_rows, long long row_vecs, int active,
                                                           unsigned* __restrict__ sink)
{
    constexpr int kLanes = 64 / ROWS_PER_WAVE, kBatch = 8;
    const int lane = (int)(threadIdx.x & 63u);
    const long long wave = ((long long)blockIdx.x * kThreads + threadIdx.x) >> 6;
    const long long row = wave * ROWS_PER_WAVE + lane / kLanes;
    const int col = lane % kLanes;
    if (row >= n_rows || col >= active) return;
    const vec16* s = src + row * row_vecs + col;
    vec16* d = WRITE ? dst + row * row_vecs + col : nullptr;
    unsigned acc = 0;
    for (long long at = 0; at + (long long)kBatch * active <= row_vecs; at += (long long)kBatch * active) {
        vec16 x[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) x[u] = __builtin_nontemporal_load(s + at + (long long)u * active);
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            if (WRITE) __builtin_nontemporal_store(x[u], d + at + (long long)u * active);
            else acc += x[u][0] ^ x[u][1] ^ x[u][2] ^ x[u][3];
        }
    }
    if (!WRITE && acc == kUnlikely) *sink = acc;
}

}  // namespace

extern "C" int bload_ys_copy(const void* d_src, void* d_dst, size_t bytes, void* hip_stream)
{
    if (!d_src || !d_dst || bytes % 16 != 0 || !aligned16(d_src) || !aligned16(d_dst)) return 1;
    const size_t n_vec = bytes / 16;
    if (n_vec == 0) return 0;
    if ((n_vec + kThreads - 1) / kThreads > 0x7fffffffull) return 1;
    hipLaunchKernelGGL(ys_copy_kernel, dim3((unsigned)((n_vec + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<const vec16*>(d_src),
                       static_cast<vec16*>(d_dst), n_vec);
    return launched();
}

extern "C" int bload_ys_read(const void* d_src, size_t bytes, void* d_sink, void* hip_stream)
{
    if (!d_src || !d_sink || bytes % 16 != 0 || !aligned16(d_src)) return 1;
    const size_t n_vec = bytes / 16;
    if (n_vec == 0) return 0;
    if ((n_vec + kThreads - 1) / kThreads > 0x7fffffffull) return 1;
    hipLaunchKernelGGL(ys_read_kernel, dim3((unsigned)((n_vec + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<const vec16*>(d_src), n_vec,
                       static_cast<unsigned*>(d_sink));
    return launched();
}

extern "C" int bload_ys_token_pack(const void* d_src, void* d_payload, void* d_plane_a, void* d_plane_b,
                                   void* d_flags_a, void* d_flags_b, int64_t n_slots, int padding_percent,
                                   int scattered, void* hip_stream)
{
    if (!d_src || !d_payload || !d_plane_a || !d_plane_b || !d_flags_a || !d_flags_b) return 1;
    if (n_slots < 0 || n_slots % 4096 != 0 || padding_percent < 0 || padding_percent > 100) return 1;
    if (!aligned16(d_src) || !aligned16(d_payload) || !aligned16(d_plane_a) || !aligned16(d_plane_b) ||
        !aligned16(d_flags_a) || !aligned16(d_flags_b))
        return 1;
    if (n_slots == 0) return 0;
    const int64_t tiles = n_slots / 1024;
    if (tiles > 0x7fffffffLL) return 1;
    hipLaunchKernelGGL(ys_token_pack_kernel, dim3((unsigned)tiles), dim3(kThreads), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<const vec16*>(d_src),
                       static_cast<vec16*>(d_payload), static_cast<vec16*>(d_plane_a), static_cast<vec16*>(d_plane_b),
                       static_cast<unsigned*>(d_flags_a), static_cast<unsigned*>(d_flags_b), (unsigned)(tiles / 4),
                       padding_percent, scattered);
    return launched();
}

extern "C" int bload_ys_rows(const void* d_src, void* d_dst, int64_t n_rows, int64_t row_bytes, int rows_per_wave,
                             int active_lanes, void* d_sink, void* hip_stream)
{
    if (!d_src || !d_sink || n_rows < 0 || row_bytes < 0) return 1;
    if (rows_per_wave != 1 && rows_per_wave != 2 && rows_per_wave != 4) return 1;
    if (active_lanes < 1 || active_lanes > 64 / rows_per_wave) return 1;
    if (row_bytes % (8 * 16 * (int64_t)active_lanes) != 0) return 1;
    if (!aligned16(d_src) || (d_dst && !aligned16(d_dst))) return 1;
    if (n_rows == 0 || row_bytes == 0) return 0;
    const int64_t waves = (n_rows + rows_per_wave - 1) / rows_per_wave;
    const int64_t groups = (waves + 3) / 4;
    if (groups > 0x7fffffffLL) return 1;
    const dim3 grid((unsigned)groups), block(kThreads);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const vec16* src = static_cast<const vec16*>(d_src);
    vec16* dst = static_cast<vec16*>(d_dst);
    unsigned* sink = static_cast<unsigned*>(d_sink);
    const long long row_vecs = row_bytes / 16;
#define BLOAD_YS_ROWS(R)                                                                                          \
    do {                                                                                                          \
        if (dst) hipLaunchKernelGGL((ys_rows_kernel<R, true>), grid, block, 0, stream, src, dst, (long long)n_rows, \
                                    row_vecs, active_lanes, sink);                                                \
        else hipLaunchKernelGGL((ys_rows_kernel<R, false>), grid, block, 0, stream, src, dst, (long long)n_rows,    \
                                row_vecs, active_lanes, sink);                                                    \
    } while (0)
    if (rows_per_wave == 1) BLOAD_YS_ROWS(1);
    else if (rows_per_wave == 2) BLOAD_YS_ROWS(2);
    else BLOAD_YS_ROWS(4);
#undef BLOAD_YS_ROWS
    return launched();
}
