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
// Up to 2048 sequences one workgroup does all of it in LDS, in one launch.
// Beyond that the scans work on tiles of 2048 positions (many small workgroups)
// and the orbit is found on tiles of 8192 in three steps that need no launch per
// jumping round: every tile jumps inside its own LDS until each of its positions
// has left the tile (exit[p]); one thread follows exit[] from position 0 and
// notes where the orbit enters each tile (one hop per tile); every tile then
// marks its heads from its entry by jumping in LDS again.  Seven launches at any size; five
// up to 8192 sequences, where the one tile is entered at position 0 and the first two of the
// three steps fall away; six up to 256 tiles of 8192, where every tile follows exit[] to its own
// entry.
#include "bload_common.hpp"
#include "bload_order.hpp"

namespace bload {

constexpr int kItems = 8;                         // consecutive positions per thread in the scans
constexpr int kTile = kThreads * kItems;          // positions per workgroup in the scans: 2048
constexpr int kJumpThreads = 512;                 // workgroup size where a workgroup jumps in LDS (8 waves:
                                                  // LDS look-ups of one wave hide behind the others')
constexpr int kJumpItems = 16;                    // positions per thread there
constexpr int kJumpTile = kJumpThreads * kJumpItems;   // 8192
constexpr int kWalkTiles = 256;                   // up to this many jump tiles, each finds its own entry (see plan_mark_kernel)
constexpr int kJumpRounds = 13;                   // 2^13 = kJumpTile: rounds that cross a whole tile
constexpr int kScanPerJump = kJumpTile / kTile;   // scan tiles in a jump tile
constexpr int kWavesPerScanTile = kTile / (kWave * kJumpItems);     // waves of the marking kernel per scan tile
static_assert(kScanPerJump * kWavesPerScanTile == kJumpThreads / kWave, "waves of the marking kernel tile the scan tiles");

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

// How a value of each scanned type comes from another lane (DPP), with the operation's
// identity where there is no such lane.
struct LaneMove {
    template <int CTRL, int ROW_MASK>
    __device__ __forceinline__ int64_t at(int64_t v) const
    {
        return (int64_t)dpp_move<CTRL, ROW_MASK>((long long)v, 0ll);
    }
    template <int CTRL, int ROW_MASK>
    __device__ __forceinline__ HeadPair at(HeadPair v) const
    {
        return HeadPair{dpp_move<CTRL, ROW_MASK>(v.cnt, 0), dpp_move<CTRL, ROW_MASK>(v.head, -1)};
    }
};

// Exclusive scan of one value per thread across the workgroup; `total` gets
// the reduction of all values.  `ident` is the identity of `op`.
template <typename T, typename Op>
__device__ __forceinline__ T block_exclusive_scan(T x, T ident, Op op, T* total)
{
    __shared__ T wave_tot[kThreads / kWave];
    const int lane = lane_id(), wave = wave_id();
    const T incl = wave_scan(x, op, LaneMove());
    const T excl = LaneMove().template at<kDppWaveShr1, 0xF>(incl);     // lane 0: the identity
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

// ---- steps shared by the one-workgroup plan and the tiled one --------------------------

// next[p]: smallest q > p with P[q+1] - P[p] > t_blk, n_seq if there is none; P is read
// through `prefix_at`.  Every length is >= 1, so q - p <= t_blk bounds the search window.
template <typename PrefixAt>
__device__ __forceinline__ int32_t next_head(PrefixAt prefix_at, int32_t p, int32_t n_seq, int32_t t_blk)
{
    const int64_t limit = prefix_at(p) + t_blk;
    // first index e in (p+1, min(n_seq, p+1+t_blk)] with P[e] > limit; q = e - 1
    int64_t lo = (int64_t)p + 2, hi = min((int64_t)n_seq, (int64_t)p + 1 + (int64_t)t_blk) + 1;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (prefix_at((int32_t)mid) > limit) hi = mid; else lo = mid + 1;
    }
    return (lo <= n_seq) ? (int32_t)(lo - 1) : n_seq;
}

// One round of pointer jumping over the `count` positions [lo, lo + count) held in LDS: a
// pointer that points behind them stays; with MARK a marked position marks where it points.
// Thread t works on positions t, t + NT, ...: neighbours in LDS.  Eight positions at a time,
// all first look-ups, then all second ones, then the stores, so that the look-ups of a batch
// are in flight together (`from`, `to` and `mark` are different arrays).  Returns whether a
// pointer of the calling thread still pointed into the tile (when none of the workgroup does,
// further rounds change nothing).  The caller puts a barrier between rounds.
template <bool MARK, int NT>
__device__ __forceinline__ bool jump_round(const int32_t* __restrict__ from, int32_t* __restrict__ to,
                                           uint8_t* mark, int32_t lo, int32_t count)
{
    constexpr int kBatch = 8;
    bool inside_any = false;           // did a pointer of this thread still point into the tile
    for (int32_t k0 = (int32_t)threadIdx.x; k0 < count; k0 += kBatch * NT) {
        int32_t at[kBatch], then[kBatch];
        uint8_t marked[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int32_t k = k0 + u * NT;
            at[u] = k < count ? from[k] : lo + count;
            marked[u] = (MARK && k < count) ? mark[k] : (uint8_t)0;
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const bool inside = at[u] - lo < count;
            inside_any |= inside;
            then[u] = inside ? from[at[u] - lo] : at[u];
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int32_t k = k0 + u * NT;
            if (k < count) {
                to[k] = then[u];
                if (MARK && marked[u] && at[u] - lo < count) mark[at[u] - lo] = 1;
            }
        }
    }
    return inside_any;
}

// The same round (without marks) over a whole jump tile of kJumpTile positions, four neighbouring
// positions per thread and step: their pointers come and go as one 16-byte LDS access, only the
// look-ups behind them are single words (24 LDS instructions per thread and round instead of
// 48).  Positions from `count` on must hold pointers that point behind the tile.
__device__ __forceinline__ bool jump_round_tile(const int32_t* __restrict__ from, int32_t* __restrict__ to,
                                                int32_t lo, int32_t count)
{
    typedef int32_t int4v __attribute__((ext_vector_type(4)));
    constexpr int kQuads = kJumpTile / 4 / kJumpThreads;      // quads of positions per thread
    static_assert(kQuads * 4 * kJumpThreads == kJumpTile, "the threads' quads tile the jump tile");
    int4v at[kQuads], then[kQuads];
#pragma unroll
    for (int u = 0; u < kQuads; ++u)
        at[u] = *reinterpret_cast<const int4v*>(from + 4 * ((int)threadIdx.x + u * kJumpThreads));
    bool inside_any = false;
#pragma unroll
    for (int u = 0; u < kQuads; ++u) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool inside = at[u][j] - lo < count;
            inside_any |= inside;
            then[u][j] = inside ? from[at[u][j] - lo] : at[u][j];
        }
    }
#pragma unroll
    for (int u = 0; u < kQuads; ++u)
        *reinterpret_cast<int4v*>(to + 4 * ((int)threadIdx.x + u * kJumpThreads)) = then[u];
    return inside_any;
}

// Pointers behind the tile for the positions of a jump tile that lie behind the last sequence.
__device__ __forceinline__ void pad_tile(int32_t* tile, int32_t lo, int32_t count)
{
    for (int32_t k = count + (int32_t)threadIdx.x; k < kJumpTile; k += kJumpThreads) tile[k] = lo + count;
}

// ---- kernels ------------------------------------------------------------------

// order[p], the shuffled lengths, and per tile: the sum of its lengths, and whether one of them
// is outside [1, t_blk].
__global__ __launch_bounds__(kThreads) void plan_order_kernel(
    const int32_t* __restrict__ lengths, int32_t n_seq, int32_t t_blk, OrderKey key,
    int32_t* __restrict__ order, int32_t* __restrict__ shuffled_len,
    int64_t* __restrict__ tile_sum, int32_t* __restrict__ tile_bad)
{
    const int64_t base = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems;
    int64_t sum = 0;
    int bad = 0;
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
    int64_t total;
    block_exclusive_scan<int64_t>(sum, 0, SumI64(), &total);
    bad = __syncthreads_or(bad);
    if (threadIdx.x == 0) { tile_sum[blockIdx.x] = total; tile_bad[blockIdx.x] = bad; }
}

// P[p] = frames before shuffled position p; P[n_seq] = total.  Every tile adds up the sums
// of the tiles before it by itself.
__global__ __launch_bounds__(kThreads) void plan_prefix_kernel(
    const int32_t* __restrict__ shuffled_len, int32_t n_seq, const int64_t* __restrict__ tile_sum,
    int64_t* __restrict__ prefix)
{
    int64_t mine = 0;
    for (int32_t t = (int32_t)threadIdx.x; t < (int32_t)blockIdx.x; t += kThreads) mine += tile_sum[t];
    int64_t before;
    block_exclusive_scan<int64_t>(mine, 0, SumI64(), &before);

    const int64_t base = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems;
    int32_t len[kItems];
    int64_t sum = 0;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        len[j] = (base + j < n_seq) ? shuffled_len[base + j] : 0;
        sum += len[j];
    }
    int64_t total;
    int64_t run = before + block_exclusive_scan<int64_t>(sum, 0, SumI64(), &total);
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        if (base + j < n_seq) {
            prefix[base + j] = run;
            run += len[j];
            if (base + j == (int64_t)n_seq - 1) prefix[n_seq] = run;
        }
    }
}

// next[p] for every position: one thread each (a chain of dependent look-ups in P).
__global__ __launch_bounds__(kThreads) void plan_next_kernel(const int64_t* __restrict__ prefix,
                                                             int32_t n_seq, int32_t t_blk,
                                                             int32_t* __restrict__ next)
{
    const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (p < n_seq) next[p] = next_head([&](int32_t q) { return prefix[q]; }, (int32_t)p, n_seq, t_blk);
}

// Copy `count` ints between global memory and LDS, thread t taking elements t, t + NT, ...,
// eight loads in flight per thread.
template <int NT>
__device__ __forceinline__ void copy_tile(const int32_t* __restrict__ from, int32_t* __restrict__ to,
                                          int32_t count)
{
    constexpr int kBatch = 8;
    for (int32_t k0 = (int32_t)threadIdx.x; k0 < count; k0 += kBatch * NT) {
        int32_t v[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) v[u] = k0 + u * NT < count ? from[k0 + u * NT] : 0;
#pragma unroll
        for (int u = 0; u < kBatch; ++u)
            if (k0 + u * NT < count) to[k0 + u * NT] = v[u];
    }
}

// For each position of a jump tile, where the orbit that passes through it leaves the tile:
// exit[p] = the first position at or behind the tile's end reached from p under next[].
__global__ __launch_bounds__(kJumpThreads) void plan_exit_kernel(const int32_t* __restrict__ next,
                                                                 int32_t n_seq,
                                                                 int32_t* __restrict__ exit_of)
{
    __shared__ __attribute__((aligned(16))) int32_t s_jump[2][kJumpTile];
    const int32_t lo = (int32_t)blockIdx.x * kJumpTile;
    const int32_t count = min(kJumpTile, n_seq - lo);
    copy_tile<kJumpThreads>(next + lo, s_jump[0], count);
    pad_tile(s_jump[0], lo, count);
    int cur = 0;
    for (int r = 0; r < kJumpRounds; ++r) {
        __syncthreads();
        const bool more = jump_round_tile(s_jump[cur], s_jump[cur ^ 1], lo, count);
        cur ^= 1;
        if (!__syncthreads_or(more ? 1 : 0)) break;       // every pointer has left the tile
    }
    __syncthreads();
    copy_tile<kJumpThreads>(s_jump[cur], exit_of + lo, count);
}

// Where the orbit of position 0 enters each jump tile (-1: it passes over the tile): one hop
// per tile along exit[].  One workgroup; thread 0 walks.
__global__ __launch_bounds__(kThreads) void plan_chain_kernel(const int32_t* __restrict__ exit_of,
                                                              int32_t n_seq, int32_t n_jump_tiles,
                                                              int32_t* __restrict__ tile_entry)
{
    for (int32_t t = (int32_t)threadIdx.x; t < n_jump_tiles; t += kThreads) tile_entry[t] = -1;
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t e = 0;
        while (e < n_seq) {               // exit[e] lies in a later tile: at most n_jump_tiles hops
            tile_entry[e / kJumpTile] = e;
            e = exit_of[e];
        }
    }
}

// The heads inside a jump tile, from the position where the orbit enters it: tile_entry[tile],
// or, with `tile_entry` null, found here by following exit[] from position 0 (at most one hop per
// tile in front of this one: for few tiles that is quicker than a launch that does it for all;
// `exit_of` null as well: there is one tile only, entered at position 0).  The heads found so far are kept as a list in
// orbit order, h_0 = the entry: round r jumps every position of the tile from next^(2^r) to
// next^(2^(r+1)) as the exit kernel does, and before that the first 2^r heads look up theirs,
// which are h_(2^r) .. h_(2^(r+1) - 1) where those still lie inside the tile (an orbit only
// moves forward, so they leave the tile in order and the list has no holes).  A round that
// adds no head ends the search.  Also, for each of its scan tiles (one per wave), the number of heads
// and the last head.
__global__ __launch_bounds__(kJumpThreads) void plan_mark_kernel(
    const int32_t* __restrict__ next, const int32_t* __restrict__ tile_entry,
    const int32_t* __restrict__ exit_of, int32_t n_seq,
    uint8_t* __restrict__ mark, int32_t* __restrict__ tile_cnt, int32_t* __restrict__ tile_head)
{
    __shared__ __attribute__((aligned(16))) int32_t s_jump[2][kJumpTile];
    __shared__ __attribute__((aligned(16))) uint8_t s_mark[kJumpTile];
    __shared__ uint16_t s_heads[kJumpTile];           // positions inside the tile, relative to its first
    __shared__ int32_t s_n_heads;
    __shared__ HeadPair s_wave[kJumpThreads / kWave];
    static_assert(kJumpTile <= 65536, "a head's place inside the tile is kept in 16 bits");
    const int32_t lo = (int32_t)blockIdx.x * kJumpTile;
    const int32_t count = min(kJumpTile, n_seq - lo);
    __shared__ int32_t s_entry;
    copy_tile<kJumpThreads>(next + lo, s_jump[0], count);
    pad_tile(s_jump[0], lo, count);
    if (threadIdx.x == 0) {
        int32_t e = 0;
        if (tile_entry) {
            e = tile_entry[blockIdx.x];
        } else if (exit_of) {
            while (e < lo) e = exit_of[e];            // exit[e] lies in a later tile than e: the walk ends
            if (e >= lo + count) e = -1;              // the orbit passes over this tile
        }
        s_entry = e;
    }
    __syncthreads();
    const int32_t entry = s_entry;
    for (int32_t k = (int32_t)threadIdx.x; k < count; k += kJumpThreads) s_mark[k] = (uint8_t)(lo + k == entry);
    if (threadIdx.x == 0) {
        s_heads[0] = (uint16_t)max(entry - lo, 0);
        s_n_heads = entry >= 0 ? 1 : 0;
    }
    __syncthreads();
    int32_t n_heads = entry >= 0 ? 1 : 0;            // the same in every thread
    if (n_heads > 0) {
        int cur = 0;
        for (int r = 0; r < kJumpRounds; ++r) {
            const int32_t* jump = s_jump[cur];
            for (int32_t i0 = (int32_t)threadIdx.x - lane_id(); i0 < n_heads; i0 += kJumpThreads) {   // wave-uniform
                const int32_t i = i0 + lane_id();
                const int32_t to = i < n_heads ? jump[s_heads[i]] - lo : count;
                const bool inside = to < count;
                if (inside) {
                    s_heads[n_heads + i] = (uint16_t)to;
                    s_mark[to] = 1;
                }
                // the new heads of a round are the first so many of its candidates: the last lane
                // that found one speaks for its wave
                const unsigned long long found = __ballot(inside);
                if (found != 0ull && lane_id() == 63 - __builtin_clzll(found)) atomicMax(&s_n_heads, n_heads + i + 1);
            }
            const bool more = jump_round_tile(s_jump[cur], s_jump[cur ^ 1], lo, count);
            cur ^= 1;
            const bool any_inside = __syncthreads_or(more ? 1 : 0) != 0;
            const int32_t now = s_n_heads;
            const bool grew = now > n_heads;
            n_heads = now;
            if (!grew || !any_inside) break;
            __syncthreads();                          // everyone has read s_n_heads before the next round updates it
        }
    }
    __syncthreads();
    // thread t: positions 16 t .. 16 t + 15 (one 16-byte vector of marks)
    static_assert(kJumpItems == 16, "a thread's marks are one 16-byte vector");
    const int32_t base = (int32_t)threadIdx.x * kJumpItems;
    HeadPair v{0, -1};
    if (base + kJumpItems <= count) {
        union { vec16 q; uint8_t b[16]; } u;
        u.q = *reinterpret_cast<const vec16*>(s_mark + base);
        *reinterpret_cast<vec16*>(mark + lo + base) = u.q;
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if (u.b[j]) { v.cnt += 1; v.head = lo + base + j; }
    } else {
        for (int j = 0; base + j < count; ++j) {
            const uint8_t m = s_mark[base + j];
            mark[lo + base + j] = m;
            if (m) { v.cnt += 1; v.head = lo + base + j; }
        }
    }
    // heads per scan tile: kWavesPerScanTile consecutive waves each
    const HeadPair upto = wave_scan(v, HeadOp(), LaneMove());
    if (lane_id() == kWave - 1) s_wave[wave_id()] = upto;
    __syncthreads();
    if (threadIdx.x < kScanPerJump) {
        const int32_t scan_tile = (int32_t)blockIdx.x * kScanPerJump + (int32_t)threadIdx.x;
        if ((int64_t)scan_tile * kTile < n_seq) {
            HeadPair sum{0, -1};
            for (int w = 0; w < kWavesPerScanTile; ++w)
                sum = HeadOp()(sum, s_wave[threadIdx.x * kWavesPerScanTile + w]);
            tile_cnt[scan_tile] = sum.cnt;
            tile_head[scan_tile] = sum.head;
        }
    }
}

// Block and offset of every sequence, first position of every block, totals.  Every tile
// adds up the head counts of the tiles before it by itself.
__global__ __launch_bounds__(kThreads) void plan_assign_kernel(
    const uint8_t* __restrict__ mark, const int32_t* __restrict__ order,
    const int64_t* __restrict__ prefix, int32_t n_seq, const int32_t* __restrict__ tile_cnt,
    const int32_t* __restrict__ tile_head, const int32_t* __restrict__ tile_bad,
    int32_t* __restrict__ block_of_seq, int32_t* __restrict__ offset_of_seq,
    int32_t* __restrict__ block_first, PlanResult* __restrict__ result)
{
    // heads in front of this tile and the last of them; the last tile also collects the
    // length checks of all tiles
    HeadPair mine{0, -1};
    int bad = 0;
    const bool last_tile = blockIdx.x == gridDim.x - 1;
    for (int32_t t = (int32_t)threadIdx.x; t < (int32_t)gridDim.x; t += kThreads) {
        if (t < (int32_t)blockIdx.x) mine = HeadOp()(mine, HeadPair{tile_cnt[t], tile_head[t]});
        if (last_tile) bad |= tile_bad[t];
    }
    HeadPair before;
    block_exclusive_scan<HeadPair>(mine, HeadPair{0, -1}, HeadOp(), &before);
    if (last_tile) bad = __syncthreads_or(bad);

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
    run = HeadOp()(before, run);
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
                result->bad_length = bad;
                result->pad_ = 0;
            }
        }
    }
}

// The whole plan of at most kTile sequences in one workgroup: the same steps as the
// kernels above with the prefix sums, jump tables and head marks in LDS and a barrier where
// the tiled path has a kernel boundary.  A thread scans ceil(n_seq / 256) consecutive
// positions, so that small inputs still spread over all threads.
__global__ __launch_bounds__(kThreads) void plan_small_kernel(
    const int32_t* __restrict__ lengths, int32_t n_seq, int32_t t_blk, OrderKey key, int rounds,
    int32_t* __restrict__ order, int32_t* __restrict__ block_of_seq,
    int32_t* __restrict__ offset_of_seq, int32_t* __restrict__ block_first,
    PlanResult* __restrict__ result)
{
    __shared__ int64_t s_prefix[kTile + 1];
    __shared__ int32_t s_jump[2][kTile];          // [0] holds the shuffled lengths first
    __shared__ uint8_t s_mark[kTile];
    const int per_thread = (n_seq + kThreads - 1) / kThreads;
    const int base = (int)threadIdx.x * per_thread;
    const int end = min(base + per_thread, n_seq);

    int bad = 0;
    for (int p = (int)threadIdx.x; p < n_seq; p += kThreads) {
        const int32_t i = order_at((uint32_t)p, (uint32_t)n_seq, key);
        const int32_t len = lengths[i];
        order[p] = i;
        s_jump[0][p] = len;
        bad |= (len < 1) | (len > t_blk);
    }
    bad = __syncthreads_or(bad);
    int64_t sum = 0;
    for (int p = base; p < end; ++p) sum += s_jump[0][p];
    int64_t total;
    int64_t run = block_exclusive_scan<int64_t>(sum, 0, SumI64(), &total);
    for (int p = base; p < end; ++p) {
        s_prefix[p] = run;
        run += s_jump[0][p];
    }
    if (threadIdx.x == 0) s_prefix[n_seq] = total;
    __syncthreads();

    // next[p]: the position that opens the next block if p opens one
    for (int p = (int)threadIdx.x; p < n_seq; p += kThreads) {
        s_jump[0][p] = next_head([&](int32_t q) { return s_prefix[q]; }, p, n_seq, t_blk);
        s_mark[p] = (uint8_t)(p == 0);
    }
    // pointer jumping: 2^rounds >= n_seq
    int cur = 0;
    for (int r = 0; r < rounds; ++r) {
        __syncthreads();
        jump_round<true, kThreads>(s_jump[cur], s_jump[cur ^ 1], s_mark, 0, n_seq);
        cur ^= 1;
    }
    __syncthreads();

    // blocks, offsets, first positions: block and head of every position into the (now free)
    // jump tables, then every thread finishes the positions it ordered itself
    HeadPair v{0, -1};
    for (int p = base; p < end; ++p)
        if (s_mark[p]) { v.cnt += 1; v.head = p; }
    HeadPair all;
    HeadPair at = block_exclusive_scan<HeadPair>(v, HeadPair{0, -1}, HeadOp(), &all);
    for (int p = base; p < end; ++p) {
        if (s_mark[p]) {
            at.cnt += 1;
            at.head = p;
            block_first[at.cnt - 1] = p;
        }
        s_jump[0][p] = at.cnt - 1;
        s_jump[1][p] = at.head;
    }
    __syncthreads();
    for (int p = (int)threadIdx.x; p < n_seq; p += kThreads) {
        const int32_t i = order[p];               // this thread's own store above
        block_of_seq[i] = s_jump[0][p];
        offset_of_seq[i] = (int32_t)(s_prefix[p] - s_prefix[s_jump[1][p]]);
    }
    if (threadIdx.x == 0) {
        block_first[all.cnt] = n_seq;
        result->num_blocks = all.cnt;
        result->total_frames = total;
        result->bad_length = bad;
        result->pad_ = 0;
    }
}

// Workspace layout (every part 16-byte aligned).
struct PlanLayout {
    size_t result, shuffled_len, prefix, next, exit_of, mark, tile_sum, tile_cnt, tile_head, tile_entry,
        tile_bad, bytes;
    int32_t n_tiles;           // scan tiles
    int32_t n_jump_tiles;
};

static PlanLayout plan_layout(int64_t n_seq)
{
    PlanLayout l{};
    const size_t n = (size_t)(n_seq > 0 ? n_seq : 0);
    l.n_tiles = (int32_t)ceil_div((int64_t)n, kTile);
    l.n_jump_tiles = (int32_t)ceil_div((int64_t)n, kJumpTile);
    size_t off = 0;
    auto take = [&off](size_t bytes) { const size_t at = off; off += round_up(bytes, 16); return at; };
    l.result = take(sizeof(PlanResult));
    l.shuffled_len = take(n * 4);
    l.prefix = take((n + 1) * 8);
    l.next = take(n * 4);
    l.exit_of = take(n * 4);
    l.mark = take(n);
    l.tile_sum = take((size_t)l.n_tiles * 8);
    l.tile_cnt = take((size_t)l.n_tiles * 4);
    l.tile_head = take((size_t)l.n_tiles * 4);
    l.tile_entry = take((size_t)l.n_jump_tiles * 4);
    l.tile_bad = take((size_t)l.n_tiles * 4);
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
    // the numbers the host waits for go straight into pinned host memory where there is some,
    // else into the workspace, from where they are copied back
    static_assert(sizeof(PlanResult) <= 64, "the pinned buffer holds 64 bytes");
    PlanResult* pinned = static_cast<PlanResult*>(host_result_buffer());
    PlanResult* result = pinned ? pinned : reinterpret_cast<PlanResult*>(ws + l.result);
    int32_t* shuffled_len = reinterpret_cast<int32_t*>(ws + l.shuffled_len);
    int64_t* prefix = reinterpret_cast<int64_t*>(ws + l.prefix);
    int32_t* next = reinterpret_cast<int32_t*>(ws + l.next);
    int32_t* exit_of = reinterpret_cast<int32_t*>(ws + l.exit_of);
    uint8_t* mark = ws + l.mark;
    int64_t* tile_sum = reinterpret_cast<int64_t*>(ws + l.tile_sum);
    int32_t* tile_cnt = reinterpret_cast<int32_t*>(ws + l.tile_cnt);
    int32_t* tile_head = reinterpret_cast<int32_t*>(ws + l.tile_head);
    int32_t* tile_entry = reinterpret_cast<int32_t*>(ws + l.tile_entry);
    int32_t* tile_bad = reinterpret_cast<int32_t*>(ws + l.tile_bad);

    const int32_t n = (int32_t)n_seq;
    const OrderKey key = make_order_key(n_seq, seed);
    const dim3 block(kThreads);
    const dim3 tiles((uint32_t)l.n_tiles), jump_tiles((uint32_t)l.n_jump_tiles);

    if (n_seq <= kTile) {
        // 2^rounds >= n_seq >= number of heads
        int rounds = 0;
        while (((int64_t)1 << rounds) < n_seq) ++rounds;
        hipLaunchKernelGGL(plan_small_kernel, dim3(1), block, 0, stream, d_lengths, n, t_blk, key,
                           rounds, d_order, d_block_of_seq, d_offset_of_seq, d_block_first, result);
    } else {
        hipLaunchKernelGGL(plan_order_kernel, tiles, block, 0, stream, d_lengths, n, t_blk, key,
                           d_order, shuffled_len, tile_sum, tile_bad);
        hipLaunchKernelGGL(plan_prefix_kernel, tiles, block, 0, stream, shuffled_len, n, tile_sum,
                           prefix);
        hipLaunchKernelGGL(plan_next_kernel, dim3((uint32_t)ceil_div(n_seq, kThreads)), block, 0, stream,
                           prefix, n, t_blk, next);
        // where the orbit of position 0 enters each jump tile: a single tile it enters at 0; up to
        // kWalkTiles tiles every tile finds its own entry; beyond, one thread finds them all
        const bool one_jump_tile = l.n_jump_tiles == 1, tiles_walk = l.n_jump_tiles <= kWalkTiles;
        if (!one_jump_tile)
            hipLaunchKernelGGL(plan_exit_kernel, jump_tiles, dim3(kJumpThreads), 0, stream, next, n, exit_of);
        if (!tiles_walk)
            hipLaunchKernelGGL(plan_chain_kernel, dim3(1), block, 0, stream, exit_of, n, l.n_jump_tiles,
                               tile_entry);
        hipLaunchKernelGGL(plan_mark_kernel, jump_tiles, dim3(kJumpThreads), 0, stream, next,
                           tiles_walk ? nullptr : tile_entry, one_jump_tile ? nullptr : exit_of, n, mark,
                           tile_cnt, tile_head);
        hipLaunchKernelGGL(plan_assign_kernel, tiles, block, 0, stream, mark, d_order, prefix, n,
                           tile_cnt, tile_head, tile_bad, d_block_of_seq, d_offset_of_seq,
                           d_block_first, result);
    }
    if (launch_status() != BLOAD_OK) return BLOAD_EHIP;

    PlanResult host{};
    if (!pinned && !hip_ok(hipMemcpyAsync(&host, result, sizeof(host), hipMemcpyDeviceToHost, stream)))
        return BLOAD_EHIP;
    if (!hip_ok(hipStreamSynchronize(stream))) return BLOAD_EHIP;
    if (pinned) host = *pinned;
    if (host.bad_length) return BLOAD_ELENGTH;
    *h_num_blocks = host.num_blocks;
    *h_total_frames = host.total_frames;
    return BLOAD_OK;
}
