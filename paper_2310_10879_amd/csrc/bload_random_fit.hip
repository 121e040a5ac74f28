// bload_plan_random_fit: the block builder with the paper's own sampler (BLoad,
// caption of the pseudocode figure: a random entry of the length dictionary L_dict
// among those no longer than the frames remaining in the open block).
//
// The draws are a chain: what fits, and how many of each length are left, depends on
// every earlier draw.  So the chain itself runs on ONE wavefront and is kept as short
// as the hardware allows, and everything around it is parallel:
//   rf_order_kernel    seeded position p -> sequence, its length, checks, frame total
//   rf_count_kernel, rf_offsets_kernel, rf_scatter_kernel
//                      L_dict: where each length's list starts, the lists themselves in
//                      seeded order, and the running counts the chain starts from; the
//                      seeded positions are cut into chunks, one workgroup each, that
//                      count their lengths, learn where their part of every list
//                      begins, and fill it in order
//   rf_draw_kernel     the chain: per placement only (length, rank in its list, block,
//                      offset) - no global load on the chain
//   rf_assign_kernel   placement p -> sequence, and the per-sequence tables
//
// Counts per length live as two levels of running sums: inside groups of 64 lengths
// (rows in LDS) and over the groups (two registers per lane).  "How many fit" is one
// LDS read plus one lane read; "which length holds the k-th" is two compare-and-vote
// steps; taking a sequence out lowers the sums behind it.
#include "bload_common.hpp"
#include "bload_order.hpp"

#include <algorithm>

namespace bload {

constexpr int kRfMaxT = BLOAD_RANDOM_FIT_MAX_T_BLK;   // lengths 1..kRfMaxT
constexpr int kRfGroups = kRfMaxT / kWave;            // groups of 64 lengths
constexpr int kRfStride = kWave + 1;                  // a group's row: 65 running sums
static_assert(kRfGroups == 2 * kWave, "two group sums per lane");

// One placement, as the chain leaves it.
struct RfPick {
    int32_t length;
    int32_t rank;         // position inside the list of that length (the last remaining one)
    int32_t block;
    int32_t offset;
};

__global__ void rf_clear_kernel(PlanResult* result)
{
    result->num_blocks = 0;
    result->total_frames = 0;
    result->bad_length = 0;
    result->pad_ = 0;
}

// seeded[p], the length found there (0 where it is outside [1, t_blk]), the frame total.
__global__ __launch_bounds__(kThreads) void rf_order_kernel(
    const int32_t* __restrict__ lengths, int32_t n_seq, int32_t t_blk, OrderKey key,
    int32_t* __restrict__ seeded, int32_t* __restrict__ seeded_len, PlanResult* __restrict__ result)
{
    __shared__ unsigned long long s_sum;
    if (threadIdx.x == 0) s_sum = 0;
    __syncthreads();
    const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (p < n_seq) {
        const int32_t i = order_at((uint32_t)p, (uint32_t)n_seq, key);
        const int32_t len = lengths[i];
        const bool bad = (len < 1) | (len > t_blk);
        seeded[p] = i;
        seeded_len[p] = bad ? 0 : len;
        if (bad) atomicOr(&result->bad_length, 1);
        else atomicAdd(&s_sum, (unsigned long long)len);
    }
    __syncthreads();
    if (threadIdx.x == 0 && s_sum)
        atomicAdd(reinterpret_cast<unsigned long long*>(&result->total_frames), s_sum);
}

// L_dict.  first[e] = start of the list of length e+1 in entry[]; entry[first[e] + r] =
// the r-th sequence of that length in seeded order.  For the chain: within[g * 65 + j] =
// sequences of the lengths g*64+1 .. g*64+j (j = 0..64, lengths taken in groups of 64) and
// group_before[g] = sequences shorter than group g's lengths (the total for g past the end).
//
// The lists must come out in seeded order.  The seeded positions are cut into chunks of
// `per_chunk` consecutive positions (a multiple of 256).  Step 1, one workgroup per chunk:
// how many sequences of each length the chunk holds.
constexpr int kRfMaxChunks = 128;

__global__ __launch_bounds__(kThreads) void rf_count_kernel(const int32_t* __restrict__ seeded_len,
                                                            int32_t n_seq, int32_t t_blk, int32_t per_chunk,
                                                            int32_t* __restrict__ chunk_count)
{
    __shared__ int32_t s_fill[kRfMaxT];
    const int tid = (int)threadIdx.x;
    const int lengths_kept = ((t_blk + kWave - 1) / kWave) * kWave;
    for (int e = tid; e < lengths_kept; e += kThreads) s_fill[e] = 0;
    __syncthreads();
    const int64_t lo = (int64_t)blockIdx.x * per_chunk;
    const int64_t hi = min((int64_t)n_seq, lo + per_chunk);
    for (int64_t p = lo + tid; p < hi; p += kThreads) {
        const int32_t len = seeded_len[p];
        if (len) atomicAdd(&s_fill[len - 1], 1);
    }
    __syncthreads();
    for (int e = tid; e < lengths_kept; e += kThreads) chunk_count[(int64_t)blockIdx.x * kRfMaxT + e] = s_fill[e];
}

// Step 2, one workgroup: the totals per length, from them first[], within[] and group_before[],
// and in place of every chunk's counts the place where its part of each list begins.
__global__ __launch_bounds__(kThreads) void rf_offsets_kernel(
    int32_t n_chunks, int32_t t_blk, int32_t* __restrict__ chunk_count, int32_t* __restrict__ first,
    int32_t* __restrict__ within, int32_t* __restrict__ group_before)
{
    __shared__ int32_t s_fill[kRfMaxT];
    __shared__ int32_t s_scan[kThreads];
    const int tid = (int)threadIdx.x;
    const int groups = (t_blk + kWave - 1) / kWave;
    for (int e = tid; e < groups * kWave; e += kThreads) {
        int32_t total = 0;
        for (int c = 0; c < n_chunks; ++c) total += chunk_count[(int64_t)c * kRfMaxT + e];
        s_fill[e] = total;
    }
    __syncthreads();

    // running sums inside each group of 64 lengths, one group per thread
    int32_t mine = 0;
    if (tid < groups) {
        for (int j = 0; j < kWave; ++j) {
            within[tid * kRfStride + j] = mine;
            mine += s_fill[tid * kWave + j];
        }
        within[tid * kRfStride + kWave] = mine;
    }
    s_scan[tid] = mine;
    __syncthreads();
    static_assert(kRfGroups <= kThreads, "one thread per group");
    int32_t run = 0;
    for (int t = 0; t < tid; ++t) run += s_scan[t];
    if (tid < kRfGroups) group_before[tid] = run;          // = all of them past the last group
    if (tid < groups) {
        for (int j = 0; j < kWave; ++j) {
            const int e = tid * kWave + j;
            const int32_t c = s_fill[e];
            if (e < t_blk) first[e] = run;
            s_fill[e] = run;                // start of the list of length e + 1
            run += c;
        }
    }
    __syncthreads();
    // a chunk's part of a list begins behind the parts of the chunks before it
    for (int e = tid; e < groups * kWave; e += kThreads) {
        int32_t at = s_fill[e];
        for (int c = 0; c < n_chunks; ++c) {
            const int64_t k = (int64_t)c * kRfMaxT + e;
            const int32_t count = chunk_count[k];
            chunk_count[k] = at;
            at += count;
        }
    }
}

// Step 3, one workgroup per chunk: its sequences into their lists, in seeded order: tile by
// tile of 256 positions, each thread ranking its sequence among the equal lengths before it
// in the tile.
__global__ __launch_bounds__(kThreads) void rf_scatter_kernel(
    const int32_t* __restrict__ seeded, const int32_t* __restrict__ seeded_len, int32_t n_seq,
    int32_t t_blk, int32_t per_chunk, const int32_t* __restrict__ chunk_start, int32_t* __restrict__ entry)
{
    __shared__ int32_t s_fill[kRfMaxT];         // next free place of every list, for this chunk
    __shared__ int32_t s_key[kThreads];
    const int tid = (int)threadIdx.x;
    const int lengths_kept = ((t_blk + kWave - 1) / kWave) * kWave;
    for (int e = tid; e < lengths_kept; e += kThreads) s_fill[e] = chunk_start[(int64_t)blockIdx.x * kRfMaxT + e];
    __syncthreads();
    const int64_t lo = (int64_t)blockIdx.x * per_chunk;
    const int64_t hi = min((int64_t)n_seq, lo + per_chunk);
    for (int64_t tile = lo; tile < hi; tile += kThreads) {
        const int64_t p = tile + tid;
        const int32_t len = p < hi ? seeded_len[p] : 0;
        s_key[tid] = len;
        __syncthreads();
        int32_t rank = 0;
        for (int t = 0; t < kThreads; ++t) rank += (s_key[t] == len) & (t < tid);
        const int32_t at = len ? s_fill[len - 1] + rank : 0;
        __syncthreads();
        if (len) {
            entry[at] = seeded[p];
            atomicAdd(&s_fill[len - 1], 1);
        }
        __syncthreads();
    }
}

// The chain of draws, on one wavefront, everything wave-uniform except three things
// spread over the lanes: the 64 sums of a group (one LDS row), the sums of the groups
// (lane j holds groups j and 64 + j) and the next 64 random numbers.
//   how many fit    = groups below the room's group (a lane read) + the row entry of the room
//   the group of k  = the last group with "shorter sequences" <= k (compare, vote, find last)
//   the length of k = the same inside the group's row
//   taking it out   = one less in the row behind that length and in the groups behind
// TWO: more than 64 groups (t_blk > 4096).
template <bool TWO>
__global__ __launch_bounds__(kWave) void rf_draw_kernel(
    const int32_t* __restrict__ within, const int32_t* __restrict__ group_before, int32_t n_seq,
    int32_t t_blk, uint64_t seed, RfPick* __restrict__ pick, int32_t* __restrict__ block_first,
    PlanResult* __restrict__ result)
{
    __shared__ int32_t s_within[(TWO ? kRfGroups : kWave) * kRfStride];
    const int lane = (int)threadIdx.x;
    const int groups = (t_blk + kWave - 1) / kWave;
    for (int k = lane; k < groups * kRfStride; k += kWave) s_within[k] = within[k];
    int32_t before_lo = group_before[lane];
    int32_t before_hi = TWO ? group_before[kWave + lane] : 0;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    if (result->bad_length) return;

    // Every block takes at least one sequence (all of them fit an empty block) and every
    // placement uses up room, so both loops end whatever the sums hold; should a draw ever
    // land on a length that does not fit, the chain stops and says so.
    int32_t placed = 0, block = 0;
    bool consistent = true;
    uint32_t u_lo = 0, u_hi = 0;
    while (consistent && placed < n_seq && block < n_seq) {
        int32_t room = t_blk;
        if (lane == 0) block_first[block] = placed;
        while (room > 0 && placed < n_seq) {
            const int e_room = room - 1, g_room = e_room >> 6;
            int32_t fit = s_within[g_room * kRfStride + (e_room & 63) + 1];
            if (TWO && g_room >= kWave) fit += __builtin_amdgcn_readlane(before_hi, g_room - kWave);
            else fit += __builtin_amdgcn_readlane(before_lo, g_room);
            fit = __builtin_amdgcn_readfirstlane(fit);
            if (fit <= 0) break;

            if ((placed & (kWave - 1)) == 0) {          // the next 64 random numbers, one per lane
                const uint64_t u = splitmix64_at(seed, (uint64_t)(6 + placed + lane));
                u_lo = (uint32_t)u;
                u_hi = (uint32_t)(u >> 32);
            }
            const int turn = placed & (kWave - 1);
            const uint64_t u = ((uint64_t)__builtin_amdgcn_readlane(u_hi, turn) << 32) |
                               (uint32_t)__builtin_amdgcn_readlane(u_lo, turn);
            const int32_t k = (int32_t)__umul64hi(u, (uint64_t)fit);          // uniform in [0, fit)

            int g_pick = 63 - __builtin_clzll(__ballot(before_lo <= k));      // lane 0 holds 0 <= k
            int32_t below = __builtin_amdgcn_readlane(before_lo, g_pick);
            if (TWO) {
                const uint64_t vote_hi = __ballot(before_hi <= k);
                if (vote_hi) {
                    const int j = 63 - __builtin_clzll(vote_hi);
                    g_pick = kWave + j;
                    below = __builtin_amdgcn_readlane(before_hi, j);
                }
            }
            const int row = g_pick * kRfStride + lane;
            const int32_t shorter = s_within[row], upto = s_within[row + 1];
            const int j = 63 - __builtin_clzll(__ballot(shorter <= k - below));   // lane 0 holds 0
            const int32_t length = g_pick * kWave + j + 1;
            const int32_t left = __builtin_amdgcn_readlane(upto, j) - __builtin_amdgcn_readlane(shorter, j);
            if (length > room) {
                consistent = false;
                break;
            }

            // the last remaining sequence of that length leaves
            if (lane >= j) s_within[row + 1] = upto - 1;
            before_lo -= (lane > g_pick);
            if (TWO) before_hi -= (kWave + lane > g_pick);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

            if (lane == 0) pick[placed] = RfPick{length, left - 1, block, t_blk - room};
            room -= length;
            placed += 1;
        }
        block += 1;
    }
    if (lane == 0) {
        if (consistent && placed == n_seq) {
            block_first[block] = n_seq;
            result->num_blocks = block;
        } else {
            result->bad_length = 2;
        }
    }
}

__global__ __launch_bounds__(kThreads) void rf_assign_kernel(
    const RfPick* __restrict__ pick, const int32_t* __restrict__ first,
    const int32_t* __restrict__ entry, int32_t n_seq, int32_t* __restrict__ order,
    int32_t* __restrict__ block_of_seq, int32_t* __restrict__ offset_of_seq,
    PlanResult* __restrict__ result)
{
    const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (p >= n_seq || result->bad_length) return;
    const RfPick k = pick[p];
    const int64_t at = (int64_t)first[k.length - 1] + k.rank;
    if (k.rank < 0 || at >= n_seq) {                    // cannot happen with consistent sums
        result->bad_length = 2;
        return;
    }
    const int32_t i = entry[at];
    order[p] = i;
    block_of_seq[i] = k.block;
    offset_of_seq[i] = k.offset;
}

struct RfLayout {
    size_t result, seeded, seeded_len, entry, pick, first, within, group_before, chunk_count, bytes;
    int32_t n_chunks, per_chunk;
};

static RfLayout rf_layout(int64_t n_seq)
{
    RfLayout l{};
    const size_t n = (size_t)(n_seq > 0 ? n_seq : 0);
    size_t off = 0;
    auto take = [&off](size_t bytes) { const size_t at = off; off += round_up(bytes, 16); return at; };
    l.result = take(sizeof(PlanResult));
    l.seeded = take(n * 4);
    l.seeded_len = take(n * 4);
    l.entry = take(n * 4);
    l.pick = take(n * sizeof(RfPick));
    l.first = take((size_t)kRfMaxT * 4);
    l.within = take((size_t)kRfGroups * kRfStride * 4);
    l.group_before = take((size_t)kRfGroups * 4);
    // chunks of whole 256-position tiles, at most kRfMaxChunks of them, at least 4 tiles each
    const int64_t tiles = ceil_div((int64_t)n, kThreads);
    const int64_t tiles_per_chunk = std::max<int64_t>(4, ceil_div(tiles, kRfMaxChunks));
    l.per_chunk = (int32_t)(tiles_per_chunk * kThreads);
    l.n_chunks = (int32_t)std::max<int64_t>(1, ceil_div((int64_t)n, l.per_chunk));
    l.chunk_count = take((size_t)l.n_chunks * kRfMaxT * 4);
    l.bytes = off;
    return l;
}

}  // namespace bload

using namespace bload;

extern "C" size_t bload_plan_random_fit_workspace_bytes(int64_t n_seq)
{
    if (n_seq < 0 || n_seq > BLOAD_MAX_SEQ) return 0;
    return rf_layout(n_seq).bytes;
}

extern "C" bload_status bload_plan_random_fit(const int32_t* d_lengths, int64_t n_seq, int32_t t_blk,
                                              uint64_t seed, int32_t* d_order,
                                              int32_t* d_block_of_seq, int32_t* d_offset_of_seq,
                                              int32_t* d_block_first, int64_t* h_num_blocks,
                                              int64_t* h_total_frames, void* d_workspace,
                                              size_t workspace_bytes, void* hip_stream)
{
    if (!h_num_blocks || !h_total_frames || n_seq < 0 || t_blk < 1) return BLOAD_EINVAL;
    *h_num_blocks = 0;
    *h_total_frames = 0;
    if (n_seq > BLOAD_MAX_SEQ || t_blk > kRfMaxT) return BLOAD_EOVERFLOW;
    if (n_seq == 0) return BLOAD_OK;
    if (!d_lengths || !d_order || !d_block_of_seq || !d_offset_of_seq || !d_block_first ||
        !d_workspace)
        return BLOAD_EINVAL;
    if (!aligned_to(d_lengths, 4) || !aligned_to(d_order, 4) || !aligned_to(d_block_of_seq, 4) ||
        !aligned_to(d_offset_of_seq, 4) || !aligned_to(d_block_first, 4) ||
        !aligned_to(d_workspace, 16))
        return BLOAD_EALIGN;
    const RfLayout l = rf_layout(n_seq);
    if (workspace_bytes < l.bytes) return BLOAD_EWORKSPACE;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    uint8_t* ws = static_cast<uint8_t*>(d_workspace);
    PlanResult* result = reinterpret_cast<PlanResult*>(ws + l.result);
    int32_t* seeded = reinterpret_cast<int32_t*>(ws + l.seeded);
    int32_t* seeded_len = reinterpret_cast<int32_t*>(ws + l.seeded_len);
    int32_t* entry = reinterpret_cast<int32_t*>(ws + l.entry);
    RfPick* pick = reinterpret_cast<RfPick*>(ws + l.pick);
    int32_t* first = reinterpret_cast<int32_t*>(ws + l.first);
    int32_t* within = reinterpret_cast<int32_t*>(ws + l.within);
    int32_t* group_before = reinterpret_cast<int32_t*>(ws + l.group_before);
    int32_t* chunk_count = reinterpret_cast<int32_t*>(ws + l.chunk_count);

    const int32_t n = (int32_t)n_seq;
    const OrderKey key = make_order_key(n_seq, seed);
    const dim3 block(kThreads);
    const dim3 per_item((uint32_t)ceil_div(n_seq, kThreads));

    hipLaunchKernelGGL(rf_clear_kernel, dim3(1), dim3(1), 0, stream, result);
    hipLaunchKernelGGL(rf_order_kernel, per_item, block, 0, stream, d_lengths, n, t_blk, key, seeded,
                       seeded_len, result);
    hipLaunchKernelGGL(rf_count_kernel, dim3((uint32_t)l.n_chunks), block, 0, stream, seeded_len, n, t_blk,
                       l.per_chunk, chunk_count);
    hipLaunchKernelGGL(rf_offsets_kernel, dim3(1), block, 0, stream, l.n_chunks, t_blk, chunk_count, first,
                       within, group_before);
    hipLaunchKernelGGL(rf_scatter_kernel, dim3((uint32_t)l.n_chunks), block, 0, stream, seeded, seeded_len,
                       n, t_blk, l.per_chunk, chunk_count, entry);
    // after a length outside [1, t_blk] the last two kernels return at once
    if (t_blk > kWave * kWave)
        hipLaunchKernelGGL(rf_draw_kernel<true>, dim3(1), dim3(kWave), 0, stream, within, group_before,
                           n, t_blk, seed, pick, d_block_first, result);
    else
        hipLaunchKernelGGL(rf_draw_kernel<false>, dim3(1), dim3(kWave), 0, stream, within,
                           group_before, n, t_blk, seed, pick, d_block_first, result);
    hipLaunchKernelGGL(rf_assign_kernel, per_item, block, 0, stream, pick, first, entry, n, d_order,
                       d_block_of_seq, d_offset_of_seq, result);
    if (launch_status() != BLOAD_OK) return BLOAD_EHIP;
    PlanResult host{};
    if (!hip_ok(hipMemcpyAsync(&host, result, sizeof(host), hipMemcpyDeviceToHost, stream)))
        return BLOAD_EHIP;
    if (!hip_ok(hipStreamSynchronize(stream))) return BLOAD_EHIP;
    if (host.bad_length == 1) return BLOAD_ELENGTH;
    if (host.bad_length) return BLOAD_EHIP;            // the chain found its sums inconsistent
    *h_num_blocks = host.num_blocks;
    *h_total_frames = host.total_frames;
    return BLOAD_OK;
}
