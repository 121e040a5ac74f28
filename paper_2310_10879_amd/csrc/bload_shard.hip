// bload_plan_shard: the share of one data-parallel worker in a plan (BLoad,
// Problem Statement: every worker has to receive the same number of samples,
// otherwise the gradient exchange stalls).  Worker `rank` of `world` takes the
// blocks b with b mod world == rank, renumbered j = b / world; workers that
// would fall one block short get one block of pure padding, so that all hold
// ceil(B / world) blocks.  The result is a plan in the worker's own numbering,
// which bload_pack and bload_segment_reduce take like any other plan.
#include "bload_common.hpp"

namespace bload {

// block_first_local[j] = number of sequences in the worker's blocks before j
// (one workgroup, chunked scan with a running carry), [blocks_local] = n_local.
__global__ __launch_bounds__(kThreads) void shard_block_first_kernel(
    const int32_t* __restrict__ block_first, int64_t num_blocks, int32_t rank, int32_t world,
    int64_t blocks_local, int32_t* __restrict__ block_first_local, int64_t* __restrict__ n_local_out)
{
    __shared__ int32_t s_wave[kThreads / kWave];
    __shared__ int32_t s_carry;
    const int lane = lane_id(), wave = wave_id();
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    for (int64_t base = 0; base < blocks_local; base += kThreads) {
        const int64_t j = base + threadIdx.x;
        const int64_t b = j * world + rank;
        int32_t cnt = 0;
        if (j < blocks_local && b < num_blocks) cnt = block_first[b + 1] - block_first[b];
        int32_t incl = cnt;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int32_t y = __shfl_up(incl, d, kWave);
            if (lane >= d) incl += y;
        }
        if (lane == kWave - 1) s_wave[wave] = incl;
        __syncthreads();
        int32_t before = s_carry;
        for (int w = 0; w < wave; ++w) before += s_wave[w];
        if (j < blocks_local) block_first_local[j] = before + incl - cnt;
        __syncthreads();
        if (threadIdx.x == kThreads - 1) s_carry = before + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        block_first_local[blocks_local] = s_carry;
        *n_local_out = s_carry;
    }
}

// One thread per shuffled position: move the worker's sequences to their local
// positions, mark the others, and put -1 behind the worker's last position.
__global__ __launch_bounds__(kThreads) void shard_fill_kernel(
    const int32_t* __restrict__ order, const int32_t* __restrict__ block_of_seq,
    const int32_t* __restrict__ block_first, const int32_t* __restrict__ block_first_local,
    int32_t n_seq, int64_t blocks_local, int32_t rank, int32_t world,
    int32_t* __restrict__ order_local, int32_t* __restrict__ block_of_seq_local)
{
    const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (p >= n_seq) return;
    if (p >= block_first_local[blocks_local]) order_local[p] = -1;
    const uint32_t i = (uint32_t)order[p];
    if (i >= (uint32_t)n_seq) return;
    const int32_t b = block_of_seq[i];
    if (b >= 0 && b % world == rank) {
        const int32_t j = b / world;
        order_local[block_first_local[j] + ((int32_t)p - block_first[b])] = (int32_t)i;
        block_of_seq_local[i] = j;
    } else {
        block_of_seq_local[i] = -1;
    }
}

}  // namespace bload

using namespace bload;

extern "C" bload_status bload_plan_shard(const int32_t* d_order, const int32_t* d_block_of_seq,
                                         const int32_t* d_block_first, int64_t n_seq,
                                         int64_t num_blocks, int32_t rank, int32_t world,
                                         int32_t* d_order_local, int32_t* d_block_of_seq_local,
                                         int32_t* d_block_first_local, int64_t* h_num_blocks_local,
                                         int64_t* h_n_seq_local, void* d_workspace,
                                         size_t workspace_bytes, void* hip_stream)
{
    if (!h_num_blocks_local || !h_n_seq_local || n_seq < 0 || num_blocks < 0 || world < 1 ||
        rank < 0 || rank >= world || num_blocks > n_seq)
        return BLOAD_EINVAL;
    *h_n_seq_local = 0;
    const int64_t blocks_local = ceil_div(num_blocks, world);
    *h_num_blocks_local = blocks_local;
    if (n_seq > BLOAD_MAX_SEQ) return BLOAD_EOVERFLOW;
    if (n_seq == 0) return BLOAD_OK;
    if (!d_order || !d_block_of_seq || !d_block_first || !d_order_local || !d_block_of_seq_local ||
        !d_block_first_local || !d_workspace)
        return BLOAD_EINVAL;
    if (!aligned_to(d_order, 4) || !aligned_to(d_block_of_seq, 4) || !aligned_to(d_block_first, 4) ||
        !aligned_to(d_order_local, 4) || !aligned_to(d_block_of_seq_local, 4) ||
        !aligned_to(d_block_first_local, 4) || !aligned_to(d_workspace, 16))
        return BLOAD_EALIGN;
    if (workspace_bytes < 16) return BLOAD_EWORKSPACE;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int64_t* pinned = static_cast<int64_t*>(host_result_buffer());
    int64_t* n_local = pinned ? pinned : static_cast<int64_t*>(d_workspace);
    hipLaunchKernelGGL(shard_block_first_kernel, dim3(1), dim3(kThreads), 0, stream, d_block_first,
                       num_blocks, rank, world, blocks_local, d_block_first_local, n_local);
    hipLaunchKernelGGL(shard_fill_kernel, dim3((uint32_t)ceil_div(n_seq, kThreads)), dim3(kThreads), 0,
                       stream, d_order, d_block_of_seq, d_block_first, d_block_first_local,
                       (int32_t)n_seq, blocks_local, rank, world, d_order_local, d_block_of_seq_local);
    if (launch_status() != BLOAD_OK) return BLOAD_EHIP;
    int64_t host = 0;
    if (!pinned && !hip_ok(hipMemcpyAsync(&host, n_local, sizeof(host), hipMemcpyDeviceToHost, stream)))
        return BLOAD_EHIP;
    if (!hip_ok(hipStreamSynchronize(stream))) return BLOAD_EHIP;
    *h_n_seq_local = pinned ? *pinned : host;
    return BLOAD_OK;
}
