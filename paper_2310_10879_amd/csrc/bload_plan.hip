// bload_plan: seeded order + next-fit block assignment on the device
// (BLoad, Methods section: blocks of T_max frames made of randomly ordered
// whole sequences, each closed as near T_max as the order allows).
//
// Next-fit is a sequential recurrence (whether a sequence opens a new block
// depends on everything before it).  Its exact parallel form, all in integers:
//   P        exclusive prefix sum of the lengths in shuffled order
//   next[p]  the position that would open the next block if p opened one:
//            the smallest q > p with P[q+1] - P[p] > T_blk (binary search in P)
//   heads    the orbit of position 0 under next[], marked by pointer jumping
//            (round k: every marked p marks jump[p], then jump = jump o jump)
//   block    inclusive count of heads up to p, minus one
//   offset   P[p] - P[head of p's block]
#include "bload_common.hpp"
#include "bload_order.hpp"

namespace bload {

constexpr int kItems = 8;                         // consecutive positions per thread
constexpr int kTile = kThreads * kItems;          // positions per workgroup in the scans

// ---- workgroup scans --------------------------------------------------------

// (number of heads, position of the last head): combined by sum and max.
struct HeadPair { int32_t cnt; int32_t head; };
struct HeadOp {
    __device__ HeadPair operator()(HeadPair a, HeadPair b) const
    {
        return HeadPair{a.cnt + b.cnt, max(a.head, b.head)};
    }
};
struct SumI64 { __device__ int64_t operator()(int64_t a, int64_t b) const { return a + b; } };

__device__ __forceinline__ int64_t shuffle_up(int64_t v, int d)
{
    return (int64_t)__shfl_up((long long)v, d, kWave);
}
__device__ __forceinline__ HeadPair shuffle_up(HeadPair v, int d)
{
    return HeadPair{__shfl_up(v.cnt, d, kWave), __shfl_up(v.head, d, kWave)};
}

template <typename T, typename Op>
__device__ __forceinline__ T wave_inclusive_scan(T x, Op op)
{
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const T y = shuffle_up(x, d);
        if (lane >= d) x = op(y, x);
    }
    return x;
}

// Exclusive scan of one value per thread across the workgroup; `total` gets
// the reduction of all values.  `ident` is the identity of `op`.
template <typename T, typename Op>
__device__ __forceinline__ T block_exclusive_scan(T x, T ident, Op op, T* total)
{
    __shared__ T wave_tot[kThreads / kWave];
    const int lane = lane_id(), wave = wave_id();
    const T incl = wave_inclusive_scan(x, op);
    T excl = shuffle_up(incl, 1);
    if (lane == 0) excl = ident;
    __syncthreads();                                  // wave_tot may still be read by a previous call
    if (lane == kWave - 1) wave_tot[wave] = incl;
    __syncthreads();
    T before = ident, all = ident;
#pragma unroll
    for (int w = 0; w < kThreads / kWave; ++w) {
        const T t = wave_tot[w];
        if (w < wave) before = op(before, t);
        all = op(all, t);
    }
    *total = all;
    return op(before, excl);
}


// ---- kernels ------------------------------------------------------------------

// order[p], the shuffled lengths, the length check, and each tile's length sum.
__global__ __launch_bounds__(kThreads) void plan_order_kernel(
    const int32_t* __restrict__ lengths, int32_t n_seq, int32_t t_blk, OrderKey key,
    int32_t* __restrict__ order, int32_t* __restrict__ shuffled_len,
    int64_t* __restrict__ tile_sum, PlanResult* __restrict__ result)
{
    const int64_t base = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems;
    int64_t sum = 0;
    bool bad = false;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        const int64_t p = base + j;
        if (p < n_seq) {
            const int32_t i = order_at((uint32_t)p, (uint32_t)n_seq, key);
            const int32_t len = lengths[i];
            order[p] = i;
            shuffled_len[p] = len;
            bad |= (len < 1) | (len > t_blk);
            sum += len;
        }
    }
    if (bad) atomicOr(&result->bad_length, 1);
    int64_t total;
    block_exclusive_scan<int64_t>(sum, 0, SumI64(), &total);
    if (threadIdx.x == 0) tile_sum[blockIdx.x] = total;
}

// In-place exclusive scans over the per-tile partials (one workgroup).
__global__ __launch_bounds__(kThreads) void plan_scan_tile_sums_kernel(int64_t* tile_sum, int32_t n_tiles)
{
    int64_t carry = 0;
    for (int32_t base = 0; base < n_tiles; base += kThreads) {
        const int32_t t = base + (int32_t)threadIdx.x;
        const int64_t x = t < n_tiles ? tile_sum[t] : 0;
        int64_t total;
        const int64_t excl = block_exclusive_scan<int64_t>(x, 0, SumI64(), &total);
        if (t < n_tiles) tile_sum[t] = carry + excl;
        carry += total;
    }
}

__global__ __launch_bounds__(kThreads) void plan_scan_tile_heads_kernel(int32_t* tile_cnt, int32_t* tile_head,
                                                                        int32_t n_tiles)
{
    HeadPair carry{0, -1};
    for (int32_t base = 0; base < n_tiles; base += kThreads) {
        const int32_t t = base + (int32_t)threadIdx.x;
        const HeadPair x = t < n_tiles ? HeadPair{tile_cnt[t], tile_head[t]} : HeadPair{0, -1};
        HeadPair total;
        const HeadPair excl = block_exclusive_scan<HeadPair>(x, HeadPair{0, -1}, HeadOp(), &total);
        if (t < n_tiles) {
            const HeadPair v = HeadOp()(carry, excl);
            tile_cnt[t] = v.cnt;
            tile_head[t] = v.head;
        }
        carry = HeadOp()(carry, total);
    }
}

// P[p] = frames before shuffled position p; P[n_seq] = total.
__global__ __launch_bounds__(kThreads) void plan_prefix_kernel(
    const int32_t* __restrict__ shuffled_len, int32_t n_seq, const int64_t* __restrict__ tile_sum,
    int64_t* __restrict__ prefix)
{
    const int64_t base = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems;
    int32_t len[kItems];
    int64_t sum = 0;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        len[j] = (base + j < n_seq) ? shuffled_len[base + j] : 0;
        sum += len[j];
    }
    int64_t total;
    int64_t run = tile_sum[blockIdx.x] + block_exclusive_scan<int64_t>(sum, 0, SumI64(), &total);
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        if (base + j < n_seq) {
            prefix[base + j] = run;
            run += len[j];
            if (base + j == (int64_t)n_seq - 1) prefix[n_seq] = run;
        }
    }
}

// next[p]: smallest q > p with P[q+1] - P[p] > t_blk, n_seq if there is none.
// Every length is >= 1, so q - p <= t_blk bounds the search window.
__global__ __launch_bounds__(kThreads) void plan_next_kernel(
    const int64_t* __restrict__ prefix, int32_t n_seq, int32_t t_blk, int32_t* __restrict__ next,
    uint8_t* __restrict__ mark)
{
    const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (p >= n_seq) return;
    const int64_t limit = prefix[p] + t_blk;
    // first index e in (p+1, min(n_seq, p+1+t_blk)] with P[e] > limit; q = e - 1
    int64_t lo = p + 2, hi = min((int64_t)n_seq, p + 1 + (int64_t)t_blk) + 1;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (prefix[mid] > limit) hi = mid; else lo = mid + 1;
    }
    next[p] = (lo <= n_seq) ? (int32_t)(lo - 1) : n_seq;
    mark[p] = (uint8_t)(p == 0);
}

// One pointer-jumping round.
__global__ __launch_bounds__(kThreads) void plan_jump_kernel(const int32_t* __restrict__ jump_in,
                                                             int32_t* __restrict__ jump_out,
                                                             uint8_t* mark, int32_t n_seq)
{
    const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (p >= n_seq) return;
    const int32_t j = jump_in[p];
    if (j < n_seq) {
        if (mark[p]) mark[j] = 1;
        jump_out[p] = jump_in[j];
    } else {
        jump_out[p] = n_seq;
    }
}

// Per tile: number of heads and position of the last one.
__global__ __launch_bounds__(kThreads) void plan_count_heads_kernel(const uint8_t* __restrict__ mark,
                                                                    int32_t n_seq,
                                                                    int32_t* __restrict__ tile_cnt,
                                                                    int32_t* __restrict__ tile_head)
{
    const int64_t base = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems;
    HeadPair v{0, -1};
#pragma unroll
    for (int j = 0; j < kItems; ++j)
        if (base + j < n_seq && mark[base + j]) { v.cnt += 1; v.head = (int32_t)(base + j); }
    HeadPair total;
    block_exclusive_scan<HeadPair>(v, HeadPair{0, -1}, HeadOp(), &total);
    if (threadIdx.x == 0) { tile_cnt[blockIdx.x] = total.cnt; tile_head[blockIdx.x] = total.head; }
}

// Block and offset of every sequence, first position of every block, totals.
__global__ __launch_bounds__(kThreads) void plan_assign_kernel(
    const uint8_t* __restrict__ mark, const int32_t* __restrict__ order,
    const int64_t* __restrict__ prefix, int32_t n_seq, const int32_t* __restrict__ tile_cnt,
    const int32_t* __restrict__ tile_head, int32_t* __restrict__ block_of_seq,
    int32_t* __restrict__ offset_of_seq, int32_t* __restrict__ block_first,
    PlanResult* __restrict__ result)
{
    const int64_t base = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems;
    uint8_t m[kItems];
    HeadPair v{0, -1};
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        m[j] = (base + j < n_seq) ? mark[base + j] : (uint8_t)0;
        if (m[j]) { v.cnt += 1; v.head = (int32_t)(base + j); }
    }
    HeadPair total;
    HeadPair run = block_exclusive_scan<HeadPair>(v, HeadPair{0, -1}, HeadOp(), &total);
    run = HeadOp()(HeadPair{tile_cnt[blockIdx.x], tile_head[blockIdx.x]}, run);
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        const int64_t p = base + j;
        if (p < n_seq) {
            if (m[j]) {
                run.cnt += 1;
                run.head = (int32_t)p;
                block_first[run.cnt - 1] = (int32_t)p;
            }
            const int32_t i = order[p];
            block_of_seq[i] = run.cnt - 1;
            offset_of_seq[i] = (int32_t)(prefix[p] - prefix[run.head]);
            if (p == (int64_t)n_seq - 1) {
                block_first[run.cnt] = n_seq;
                result->num_blocks = run.cnt;
                result->total_frames = prefix[n_seq];
            }
        }
    }
}

// The whole plan of at most kTile sequences in one workgroup: the same steps
// as the kernels above with the prefix sums, jump tables and head marks in LDS
// and a barrier where the large path has a kernel boundary.
__global__ __launch_bounds__(kThreads) void plan_small_kernel(
    const int32_t* __restrict__ lengths, int32_t n_seq, int32_t t_blk, OrderKey key, int rounds,
    int32_t* __restrict__ order, int32_t* __restrict__ block_of_seq,
    int32_t* __restrict__ offset_of_seq, int32_t* __restrict__ block_first,
    PlanResult* __restrict__ result)
{
    __shared__ int64_t s_prefix[kTile + 1];
    __shared__ int32_t s_jump[2][kTile];
    __shared__ uint8_t s_mark[kTile];
    const int base = (int)threadIdx.x * kItems;

    int32_t ord[kItems], len[kItems];
    int64_t sum = 0;
    int bad = 0;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        const int p = base + j;
        ord[j] = 0;
        len[j] = 0;
        if (p < n_seq) {
            ord[j] = order_at((uint32_t)p, (uint32_t)n_seq, key);
            len[j] = lengths[ord[j]];
            order[p] = ord[j];
            bad |= (len[j] < 1) | (len[j] > t_blk);
            sum += len[j];
        }
    }
    int64_t total;
    int64_t run = block_exclusive_scan<int64_t>(sum, 0, SumI64(), &total);
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        if (base + j < n_seq) s_prefix[base + j] = run;
        run += len[j];
    }
    if (threadIdx.x == 0) s_prefix[n_seq] = total;
    bad = __syncthreads_or(bad);

    // next[p]: the position that opens the next block if p opens one
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        const int p = base + j;
        if (p < n_seq) {
            const int64_t limit = s_prefix[p] + t_blk;
            int lo = p + 2, hi = (int)min((int64_t)n_seq, (int64_t)p + 1 + t_blk) + 1;
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (s_prefix[mid] > limit) hi = mid; else lo = mid + 1;
            }
            s_jump[0][p] = (lo <= n_seq) ? lo - 1 : n_seq;
            s_mark[p] = (uint8_t)(p == 0);
        }
    }
    // pointer jumping
    int cur = 0;
    for (int r = 0; r < rounds; ++r) {
        __syncthreads();
#pragma unroll
        for (int j = 0; j < kItems; ++j) {
            const int p = base + j;
            if (p < n_seq) {
                const int32_t to = s_jump[cur][p];
                if (to < n_seq) {
                    if (s_mark[p]) s_mark[to] = 1;
                    s_jump[cur ^ 1][p] = s_jump[cur][to];
                } else {
                    s_jump[cur ^ 1][p] = n_seq;
                }
            }
        }
        cur ^= 1;
    }
    __syncthreads();

    // blocks, offsets, first positions
    uint8_t m[kItems];
    HeadPair v{0, -1};
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        m[j] = (base + j < n_seq) ? s_mark[base + j] : (uint8_t)0;
        if (m[j]) { v.cnt += 1; v.head = base + j; }
    }
    HeadPair all;
    HeadPair at = block_exclusive_scan<HeadPair>(v, HeadPair{0, -1}, HeadOp(), &all);
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        const int p = base + j;
        if (p < n_seq) {
            if (m[j]) {
                at.cnt += 1;
                at.head = p;
                block_first[at.cnt - 1] = p;
            }
            block_of_seq[ord[j]] = at.cnt - 1;
            offset_of_seq[ord[j]] = (int32_t)(s_prefix[p] - s_prefix[at.head]);
            if (p == n_seq - 1) {
                block_first[at.cnt] = n_seq;
                result->num_blocks = at.cnt;
                result->total_frames = total;
                result->bad_length = bad;
                result->pad_ = 0;
            }
        }
    }
}

__global__ void plan_clear_result_kernel(PlanResult* result)
{
    result->num_blocks = 0;
    result->total_frames = 0;
    result->bad_length = 0;
    result->pad_ = 0;
}

// Workspace layout (every part 16-byte aligned).
struct PlanLayout {
    size_t result, shuffled_len, prefix, jump_a, jump_b, mark, tile_sum, tile_cnt, tile_head, bytes;
    int32_t n_tiles;
};

static PlanLayout plan_layout(int64_t n_seq)
{
    PlanLayout l{};
    const size_t n = (size_t)(n_seq > 0 ? n_seq : 0);
    l.n_tiles = (int32_t)ceil_div((int64_t)n, kTile);
    size_t off = 0;
    auto take = [&off](size_t bytes) { const size_t at = off; off += round_up(bytes, 16); return at; };
    l.result = take(sizeof(PlanResult));
    l.shuffled_len = take(n * 4);
    l.prefix = take((n + 1) * 8);
    l.jump_a = take(n * 4);
    l.jump_b = take(n * 4);
    l.mark = take(n);
    l.tile_sum = take((size_t)l.n_tiles * 8);
    l.tile_cnt = take((size_t)l.n_tiles * 4);
    l.tile_head = take((size_t)l.n_tiles * 4);
    l.bytes = off;
    return l;
}

}  // namespace bload

using namespace bload;

extern "C" size_t bload_plan_workspace_bytes(int64_t n_seq)
{
    if (n_seq < 0 || n_seq > BLOAD_MAX_SEQ) return 0;
    return plan_layout(n_seq).bytes;
}

extern "C" bload_status bload_plan(const int32_t* d_lengths, int64_t n_seq, int32_t t_blk,
                                   uint64_t seed, int32_t* d_order, int32_t* d_block_of_seq,
                                   int32_t* d_offset_of_seq, int32_t* d_block_first,
                                   int64_t* h_num_blocks, int64_t* h_total_frames,
                                   void* d_workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!h_num_blocks || !h_total_frames || n_seq < 0 || t_blk < 1) return BLOAD_EINVAL;
    *h_num_blocks = 0;
    *h_total_frames = 0;
    if (n_seq > BLOAD_MAX_SEQ) return BLOAD_EOVERFLOW;
    if (n_seq == 0) return BLOAD_OK;
    if (!d_lengths || !d_order || !d_block_of_seq || !d_offset_of_seq || !d_block_first ||
        !d_workspace)
        return BLOAD_EINVAL;
    if (!aligned_to(d_lengths, 4) || !aligned_to(d_order, 4) || !aligned_to(d_block_of_seq, 4) ||
        !aligned_to(d_offset_of_seq, 4) || !aligned_to(d_block_first, 4) ||
        !aligned_to(d_workspace, 16))
        return BLOAD_EALIGN;
    const PlanLayout l = plan_layout(n_seq);
    if (workspace_bytes < l.bytes) return BLOAD_EWORKSPACE;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    uint8_t* ws = static_cast<uint8_t*>(d_workspace);
    PlanResult* result = reinterpret_cast<PlanResult*>(ws + l.result);
    int32_t* shuffled_len = reinterpret_cast<int32_t*>(ws + l.shuffled_len);
    int64_t* prefix = reinterpret_cast<int64_t*>(ws + l.prefix);
    int32_t* jump_a = reinterpret_cast<int32_t*>(ws + l.jump_a);
    int32_t* jump_b = reinterpret_cast<int32_t*>(ws + l.jump_b);
    uint8_t* mark = ws + l.mark;
    int64_t* tile_sum = reinterpret_cast<int64_t*>(ws + l.tile_sum);
    int32_t* tile_cnt = reinterpret_cast<int32_t*>(ws + l.tile_cnt);
    int32_t* tile_head = reinterpret_cast<int32_t*>(ws + l.tile_head);

    const int32_t n = (int32_t)n_seq;
    const OrderKey key = make_order_key(n_seq, seed);
    const dim3 block(kThreads);
    const dim3 tiles((uint32_t)l.n_tiles);
    const dim3 per_item((uint32_t)ceil_div(n_seq, kThreads));

    // 2^rounds >= n_seq >= number of heads
    int rounds = 0;
    while (((int64_t)1 << rounds) < n_seq) ++rounds;
    if (n_seq <= kTile) {
        hipLaunchKernelGGL(plan_small_kernel, dim3(1), block, 0, stream, d_lengths, n, t_blk, key,
                           rounds, d_order, d_block_of_seq, d_offset_of_seq, d_block_first, result);
    } else {
        hipLaunchKernelGGL(plan_clear_result_kernel, dim3(1), dim3(1), 0, stream, result);
        hipLaunchKernelGGL(plan_order_kernel, tiles, block, 0, stream, d_lengths, n, t_blk, key,
                           d_order, shuffled_len, tile_sum, result);
        hipLaunchKernelGGL(plan_scan_tile_sums_kernel, dim3(1), block, 0, stream, tile_sum, l.n_tiles);
        hipLaunchKernelGGL(plan_prefix_kernel, tiles, block, 0, stream, shuffled_len, n, tile_sum,
                           prefix);
        hipLaunchKernelGGL(plan_next_kernel, per_item, block, 0, stream, prefix, n, t_blk, jump_a,
                           mark);
        for (int r = 0; r < rounds; ++r) {
            hipLaunchKernelGGL(plan_jump_kernel, per_item, block, 0, stream, jump_a, jump_b, mark, n);
            int32_t* t = jump_a; jump_a = jump_b; jump_b = t;
        }
        hipLaunchKernelGGL(plan_count_heads_kernel, tiles, block, 0, stream, mark, n, tile_cnt,
                           tile_head);
        hipLaunchKernelGGL(plan_scan_tile_heads_kernel, dim3(1), block, 0, stream, tile_cnt, tile_head,
                           l.n_tiles);
        hipLaunchKernelGGL(plan_assign_kernel, tiles, block, 0, stream, mark, d_order, prefix, n,
                           tile_cnt, tile_head, d_block_of_seq, d_offset_of_seq, d_block_first, result);
    }
    if (launch_status() != BLOAD_OK) return BLOAD_EHIP;

    PlanResult host{};
    if (!hip_ok(hipMemcpyAsync(&host, result, sizeof(host), hipMemcpyDeviceToHost, stream)))
        return BLOAD_EHIP;
    if (!hip_ok(hipStreamSynchronize(stream))) return BLOAD_EHIP;
    if (host.bad_length) return BLOAD_ELENGTH;
    *h_num_blocks = host.num_blocks;
    *h_total_frames = host.total_frames;
    return BLOAD_OK;
}
