// bload_strategy_counts: frames of padding and frames deleted under the strategies the
// paper compares (Problem Statement; Table 1, rows "padding amount" and "# frames
// deleted"), for a given set of lengths.  One pass over the lengths.
#include "bload_common.hpp"

namespace bload {

struct CountAcc {
    unsigned long long total, samples, deleted;
    int32_t longest;
    int32_t pad_;
};

__global__ void counts_clear_kernel(CountAcc* acc)
{
    acc->total = 0;
    acc->samples = 0;
    acc->deleted = 0;
    acc->longest = 0;
    acc->pad_ = 0;
}

__device__ __forceinline__ unsigned long long wave_sum(unsigned long long v)
{
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) v += __shfl_down(v, d, kWave);
    return v;
}

__global__ __launch_bounds__(kThreads) void counts_kernel(const int32_t* __restrict__ lengths,
                                                          int64_t n_seq, int32_t t_chunk,
                                                          CountAcc* __restrict__ acc)
{
    unsigned long long total = 0, samples = 0, deleted = 0;
    int32_t longest = 0;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n_seq; i += stride) {
        const int32_t len = max(lengths[i], 0);
        const int32_t whole = len / t_chunk;
        total += (unsigned long long)len;
        samples += (unsigned long long)whole;
        deleted += (unsigned long long)(len - whole * t_chunk);
        longest = max(longest, len);
    }
    total = wave_sum(total);
    samples = wave_sum(samples);
    deleted = wave_sum(deleted);
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) longest = max(longest, __shfl_down(longest, d, kWave));
    // one set of atomics per workgroup
    __shared__ unsigned long long s_part[kThreads / kWave][3];
    __shared__ int32_t s_longest[kThreads / kWave];
    if (lane_id() == 0) {
        s_part[wave_id()][0] = total;
        s_part[wave_id()][1] = samples;
        s_part[wave_id()][2] = deleted;
        s_longest[wave_id()] = longest;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kThreads / kWave; ++w) {
            total += s_part[w][0];
            samples += s_part[w][1];
            deleted += s_part[w][2];
            longest = max(longest, s_longest[w]);
        }
        if (total) atomicAdd(&acc->total, total);
        if (samples) atomicAdd(&acc->samples, samples);
        if (deleted) atomicAdd(&acc->deleted, deleted);
        if (longest) atomicMax(&acc->longest, longest);
    }
}

}  // namespace bload

using namespace bload;

extern "C" bload_status bload_strategy_counts(const int32_t* d_lengths, int64_t n_seq, int32_t t_max,
                                              int32_t t_chunk, int64_t num_blocks, int32_t t_blk,
                                              bload_strategy_counts_t* h_counts, void* d_workspace,
                                              size_t workspace_bytes, void* hip_stream)
{
    if (!h_counts || n_seq < 0 || t_chunk < 1 || num_blocks < 0 || t_blk < 0) return BLOAD_EINVAL;
    *h_counts = bload_strategy_counts_t{};
    if (n_seq > BLOAD_MAX_SEQ) return BLOAD_EOVERFLOW;
    if (n_seq == 0) return BLOAD_OK;
    if (!d_lengths || !d_workspace) return BLOAD_EINVAL;
    if (!aligned_to(d_lengths, 4) || !aligned_to(d_workspace, 16)) return BLOAD_EALIGN;
    if (workspace_bytes < 64) return BLOAD_EWORKSPACE;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    CountAcc* acc = static_cast<CountAcc*>(d_workspace);
    const uint32_t grid = (uint32_t)(ceil_div(n_seq, kThreads) < 512 ? ceil_div(n_seq, kThreads) : 512);
    hipLaunchKernelGGL(counts_clear_kernel, dim3(1), dim3(1), 0, stream, acc);
    hipLaunchKernelGGL(counts_kernel, dim3(grid), dim3(kThreads), 0, stream, d_lengths, n_seq, t_chunk,
                       acc);
    if (launch_status() != BLOAD_OK) return BLOAD_EHIP;
    CountAcc host{};
    if (!hip_ok(hipMemcpyAsync(&host, acc, sizeof(host), hipMemcpyDeviceToHost, stream)))
        return BLOAD_EHIP;
    if (!hip_ok(hipStreamSynchronize(stream))) return BLOAD_EHIP;

    const int64_t longest_to = t_max > 0 ? t_max : host.longest;
    h_counts->total_frames = (int64_t)host.total;
    h_counts->longest = host.longest;
    h_counts->pad_to_longest = n_seq * longest_to - (int64_t)host.total;
    h_counts->pad_blocks = num_blocks > 0 ? num_blocks * (int64_t)t_blk - (int64_t)host.total : 0;
    h_counts->chunk_samples = (int64_t)host.samples;
    h_counts->chunk_deleted = (int64_t)host.deleted;
    return BLOAD_OK;
}
