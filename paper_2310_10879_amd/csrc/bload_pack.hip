// bload_pack: gather the frames of every sequence into the dense
// [num_blocks, T_blk, frame] tensor, fill the rest with 0's, and write the
// per-slot form of the start table (BLoad, Methods section).
//
// The kernels are destination driven: a workgroup owns a contiguous piece of
// the packed tensor (a "tile"), looks up which sequences land in it, and
// streams 16-byte vectors from the ragged source to the tile.  Every output
// byte is written by exactly one thread, so no memset pass and no atomics are
// needed.  A first pass (pack_prepare_kernel) turns the plan into a table of
// "runs" in shuffled order -- one 32-byte record per sequence saying where it
// lands and where it comes from, so that the copy kernels need one contiguous
// read per sequence instead of a chain of look-ups through five tables -- and
// finds, for every tile, where in that table its runs begin.
//
// Two tile shapes (takes_wide_tiles chooses, from the frame size and the bytes
// per sequence):
//   wide   a tile is 4 KiB of the packed tensor, one 16-byte vector per thread;
//          best where runs (a sequence's bytes) are long: a tile inside one run
//          is a plain copy with wave-uniform scalar look-ups.  Frames of at
//          least 64 bytes.
//   narrow a tile is 1024 consecutive slots; a tile inside one run or inside a
//          block's padding is written straight away, for any other the runs go
//          into an LDS table, lanes take consecutive 16-byte destination vectors
//          and assemble them from source elements of the widest type that
//          divides the frame.  Small frames, and middle-sized frames of short
//          sequences.  Without its payload part the same kernel writes the start
//          table of large tensors of wide frames, whose 4 KiB tiles then only
//          copy.
// All large outputs leave through streaming stores (see store_slot).
#include "bload_common.hpp"

#include <limits.h>

#include <mutex>

namespace bload {

// Where one sequence goes: the record the copy kernels work from.  Position p of the
// table belongs to shuffled position p; slots are numbered globally (block * T_blk +
// slot in block).  A position that holds no sequence (a worker's share lists only its
// own) has dst = INT64_MAX, which also ends the list.
struct __attribute__((aligned(32))) Run {
    int64_t dst;       // first slot
    int64_t src;       // first source frame
    int32_t len;       // frames
    int32_t seq;       // original sequence index
    int32_t block;     // dst / T_blk
    int32_t pad_;
};
static_assert(sizeof(Run) == 32, "a run is two 16-byte vectors");
constexpr int64_t kNoRun = INT64_MAX;

struct PackArgs {
    const uint8_t* src;
    const Run* runs;          // [n_seq], by shuffled position
    int32_t n_seq;
    int32_t t_blk;
    int64_t frame_bytes;
    int64_t total_slots;      // num_blocks * t_blk
    uint8_t* packed;
    int32_t* seq_id;
    int32_t* frame_idx;
    uint8_t* reset;
    uint8_t* valid;
};

// The sequences ("runs") that overlap one tile, in shuffled order.  Slots are
// numbered globally (block * T_blk + slot in block); dst is relative to the
// tile's first slot and is negative for a run that starts before the tile.
template <int MAXRUNS>
struct RunTable {
    int64_t src[MAXRUNS];      // first source frame of the run
    int32_t dst[MAXRUNS + 1];  // first slot, tile relative; [n] = INT_MAX sentinel
    int16_t end[MAXRUNS];      // one past its last slot, tile relative, cut to [0, MAXRUNS]: 18 bytes per
                               // run keep the table of a 1024-slot tile under an eighth of a CU's LDS
    int32_t seq[MAXRUNS];      // original sequence index
};

// Fill `tab` with the runs that can overlap global slots [gs_lo, gs_hi): the shuffled positions
// first .. last, where `first` is the tile's entry of the prepare pass (the last position of the
// tile's first block that starts at or before gs_lo) and `last` that of the tile behind it (no
// run that starts before gs_hi has a later position).  Runs are sorted by destination, so the
// runs to keep are a prefix of these candidates; candidate k becomes table entry k, and a
// candidate that starts at or behind gs_hi becomes an end mark (as does the entry behind the
// last candidate), so that a search over all candidates finds only runs of the tile.  Called by
// the whole workgroup, all look-ups in flight together; ends with a barrier.  Returns the
// number of candidates.
template <int MAXRUNS>
__device__ __forceinline__ int gather_runs(const Run* __restrict__ runs, int32_t n_seq, int32_t first,
                                           int32_t last, int64_t gs_lo, int64_t gs_hi, RunTable<MAXRUNS>& tab)
{
    const int tid = (int)threadIdx.x;
    const int n_cand = max(0, min(min(last, n_seq - 1) - first + 1, MAXRUNS));
    constexpr int PER = (MAXRUNS + kThreads - 1) / kThreads;
    Run r[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int k = tid + i * kThreads;
        if (k < n_cand) r[i] = runs[(int64_t)first + k];
    }
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int k = tid + i * kThreads;
        if (k < n_cand) {
            const bool take = r[i].dst < gs_hi;
            tab.src[k] = r[i].src;
            tab.dst[k] = take ? (int32_t)(r[i].dst - gs_lo) : INT_MAX;
            tab.end[k] = (int16_t)min(max(r[i].dst - gs_lo + r[i].len, (int64_t)0), (int64_t)MAXRUNS);
            tab.seq[k] = r[i].seq;
        }
    }
    if (tid == 0) tab.dst[n_cand] = INT_MAX;
    __syncthreads();
    return n_cand;
}

// Index of the last run whose first slot is <= slot (tile relative), -1 if none.
template <int MAXRUNS>
__device__ __forceinline__ int run_of_slot(const RunTable<MAXRUNS>& tab, int n, int32_t slot)
{
    int lo = 0, hi = n;                 // first run with dst > slot
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (tab.dst[mid] <= slot) lo = mid + 1; else hi = mid;
    }
    return lo - 1;
}

// ------------------------------------------------------------------- wide
//
// One workgroup writes one small flat piece of the packed tensor and ends:
// workgroups that run at the same time then touch a few compact windows of the
// destination (one per XCD, see xcd_contiguous) and a handful of source
// streams, which is what HBM wants; a workgroup that loops over a large private
// tile does measurably worse.
// To keep so short a workgroup cheap there is no LDS and no barrier here, and
// the lookup of the tile's runs is wave-uniform (a binary search over the
// block's positions followed by a walk over consecutive positions), so it
// runs on the scalar unit with a handful of dependent scalar loads.

constexpr int kWideMinFrame = 64;                   // smallest frame the wide kernel takes
constexpr int kWideTile = 4096;                     // tile used: one 16-byte vector per thread
constexpr int kWideWalkRuns = 2;                    // up to this many runs in a tile are walked one by one
constexpr int kWideRuns = 128;                      // shuffled positions looked up per tile; a power of two
static_assert(kWideTile / kWideMinFrame + 2 <= kWideRuns, "a tile's runs must fit the look-up window");

typedef vec16 __attribute__((aligned(1))) vec16_unaligned;

// floor(x / d) for 0 <= x < 2^52, d >= 1, with inv_d = 1.0 / d: the double
// quotient is within one of the answer, fixed up exactly in integers.
__device__ __forceinline__ int64_t floor_div(int64_t x, int64_t d, double inv_d)
{
    int64_t q = (int64_t)((double)x * inv_d);
    if (q * d > x) --q;
    else if ((q + 1) * d <= x) ++q;
    return q;
}

// Write packed bytes [lo, hi): copies of src[0 ..) (any alignment) or zeros.
// Destination vectors are 16-byte aligned; the ragged ends of the range are
// written byte by byte.  Called by all threads of the workgroup.
template <bool ZERO>
__device__ __forceinline__ void write_range(uint8_t* packed, int64_t lo, int64_t hi,
                                            const uint8_t* src)
{
    const int tid = (int)threadIdx.x;
    int64_t lo_al = (lo + 15) & ~(int64_t)15;
    if (lo_al > hi) lo_al = hi;
    int64_t hi_al = hi & ~(int64_t)15;
    if (hi_al < lo_al) hi_al = lo_al;
    const int head = (int)(lo_al - lo);
    const int tail = (int)(hi - hi_al);
    if (tid < head) packed[lo + tid] = ZERO ? (uint8_t)0 : src[tid];
    if (tid >= kWave && tid - kWave < tail)
        packed[hi_al + (tid - kWave)] = ZERO ? (uint8_t)0 : src[(hi_al - lo) + (tid - kWave)];

    const int nv = (int)((hi_al - lo_al) >> 4);
    vec16* d = reinterpret_cast<vec16*>(packed + lo_al);
    const uint8_t* s = src + (lo_al - lo);
    int v = tid;
    if (ZERO) {
        const vec16 z = {0u, 0u, 0u, 0u};
        for (; v < nv; v += kThreads) store_stream(d + v, z);
    } else {
        for (; v + 3 * kThreads < nv; v += 4 * kThreads) {
            const vec16 x0 = __builtin_nontemporal_load(
                reinterpret_cast<const vec16_unaligned*>(s + 16 * (int64_t)v));
            const vec16 x1 = __builtin_nontemporal_load(
                reinterpret_cast<const vec16_unaligned*>(s + 16 * (int64_t)(v + kThreads)));
            const vec16 x2 = __builtin_nontemporal_load(
                reinterpret_cast<const vec16_unaligned*>(s + 16 * (int64_t)(v + 2 * kThreads)));
            const vec16 x3 = __builtin_nontemporal_load(
                reinterpret_cast<const vec16_unaligned*>(s + 16 * (int64_t)(v + 3 * kThreads)));
            store_stream(d + v, x0);
            store_stream(d + v + kThreads, x1);
            store_stream(d + v + 2 * kThreads, x2);
            store_stream(d + v + 3 * kThreads, x3);
        }
        for (; v < nv; v += kThreads) {
            const vec16 x = __builtin_nontemporal_load(
                reinterpret_cast<const vec16_unaligned*>(s + 16 * (int64_t)v));
            store_stream(d + v, x);
        }
    }
}

// The start-table entry of one slot (frame index -1: padding).  Streamed like the payload: plain
// stores leave these planes (a gigabyte at 10^8 slots) as modified lines in the memory-side
// cache, and a consumer that streams the packed tensor right afterwards then reads about a tenth
// slower (measured: the reduction of 3000 x 320-byte blocks takes 3.98 ms alone and 4.45 ms
// behind a pack that wrote them with plain stores).
__device__ __forceinline__ void store_slot(const PackArgs& a, int64_t slot, int32_t seq, int32_t fid)
{
    __builtin_nontemporal_store(seq, a.seq_id + slot);
    __builtin_nontemporal_store(fid, a.frame_idx + slot);
    __builtin_nontemporal_store((uint8_t)(fid == 0), a.reset + slot);
    __builtin_nontemporal_store((uint8_t)(fid >= 0), a.valid + slot);
}

// Start-table entries of global slots [lo, hi): lane k of the calling wave writes the slots
// lo + k, lo + k + 64, ...  frame0 = frame index of slot lo, or -1 for padding.
__device__ __forceinline__ void write_slots(const PackArgs& a, int64_t lo, int64_t hi, int32_t seq,
                                            int64_t frame0)
{
    for (int64_t k = lane_id(); lo + k < hi; k += kWave) {
        const int64_t g = lo + k;
        const int32_t fid = frame0 < 0 ? -1 : (int32_t)(frame0 + k);
        store_slot(a, g, frame0 < 0 ? -1 : seq, fid);
    }
}

constexpr int kTableSlots = 1024;                   // slots per workgroup of the slot-tile kernel

// Pass 1 (used by both tile shapes, which come after it in this file's launch
// order).  Thread p < n_seq writes the run of shuffled position p.  Thread t < n_tiles
// finds, for tile t, the last shuffled position of the tile's first block whose
// sequence starts at or before the tile's first slot (the block's first sequence
// starts at slot 0, so there is one); it searches the plan's own tables, so the two
// halves do not depend on each other.
__global__ __launch_bounds__(kThreads) void pack_prepare_kernel(
    const int64_t* __restrict__ src_offsets, const int32_t* __restrict__ lengths,
    const int32_t* __restrict__ order, const int32_t* __restrict__ block_of_seq,
    const int32_t* __restrict__ offset_of_seq, const int32_t* __restrict__ block_first,
    int32_t n_seq, int64_t num_blocks, int64_t t_blk, int64_t frame_bytes, int64_t n_tiles,
    int32_t tile_bytes, double inv_frame_bytes, double inv_t_blk, Run* __restrict__ runs,
    int32_t* __restrict__ first_pos, int64_t n_table_tiles, int32_t* __restrict__ first_pos_table)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx < n_seq) {
        Run r{kNoRun, 0, 0, -1, -1, 0};
        const uint32_t i = (uint32_t)order[idx];
        if (i < (uint32_t)n_seq) {
            const int64_t b = block_of_seq[i];
            if (b >= 0 && b < num_blocks) {
                r.dst = b * t_blk + offset_of_seq[i];
                r.src = src_offsets[i];
                r.len = lengths[i];
                r.seq = (int32_t)i;
                r.block = (int32_t)b;
            }
        }
        runs[idx] = r;
    }
    // the last shuffled position of slot gs_lo's block whose sequence starts at or before gs_lo
    auto entry_of = [&](int64_t gs_lo) {
        const int64_t b0 = floor_div(gs_lo, t_blk, inv_t_blk);
        const int32_t rel = (int32_t)(gs_lo - b0 * t_blk);
        int32_t p = min(max(block_first[b0], 0), n_seq);
        int32_t above = min(max(block_first[b0 + 1], p), n_seq);
        while (above - p > 1) {
            const int32_t mid = p + ((above - p) >> 1);
            const uint32_t i = (uint32_t)order[mid];
            if (i < (uint32_t)n_seq && offset_of_seq[i] <= rel) p = mid; else above = mid;
        }
        return p;
    };
    if (idx < n_tiles) first_pos[idx] = entry_of(floor_div(idx * tile_bytes, frame_bytes, inv_frame_bytes));
    // tiles of kTableSlots slots, for the pass that writes the start table of wide frames
    if (idx < n_table_tiles) first_pos_table[idx] = entry_of(idx * kTableSlots);
}

// Pass 2: the copy.  The run table and the tiles' entries come as separate
// __restrict__ pointers so that the compiler knows nothing this kernel stores
// can alias them and keeps their loads on the scalar unit.
__global__ __launch_bounds__(kThreads) void pack_wide_kernel(
    PackArgs a, const Run* __restrict__ runs, const int32_t* __restrict__ first_pos,
    int32_t tile_bytes, double inv_frame_bytes, int32_t writes_table)
{
    const int64_t F = a.frame_bytes;
    const int64_t T = a.t_blk;
    const int32_t n_seq = a.n_seq;
    const int64_t total_bytes = a.total_slots * F;
    const uint32_t tile = xcd_contiguous(blockIdx.x, gridDim.x);
    const int64_t D0 = (int64_t)tile * tile_bytes;
    const int64_t D1 = min(D0 + (int64_t)tile_bytes, total_bytes);
    const bool table_wave = writes_table != 0 && wave_id() == 0;
    int32_t p = min(max(first_pos[tile], 0), n_seq);

    // the common case first: the tile lies inside one run -- one load and one
    // store per thread, plus the start-table entries of the few frames that
    // begin in the tile
    if (p < n_seq && tile_bytes == kThreads * 16) {
        const Run r = runs[p];
        if (r.dst != kNoRun) {
            const int64_t g = r.dst;
            const int64_t len = r.len;
            const int64_t run_lo = g * F;
            if (run_lo <= D0 && run_lo + len * F >= D0 + tile_bytes && D0 + tile_bytes <= total_bytes) {
                const uint8_t* s = a.src + r.src * F + (D0 - run_lo) + 16 * (int64_t)threadIdx.x;
                const vec16 x = __builtin_nontemporal_load(reinterpret_cast<const vec16_unaligned*>(s));
                store_stream(reinterpret_cast<vec16*>(a.packed + D0) + threadIdx.x, x);
                if (table_wave) {
                    // frames t of this run with D0 <= run_lo + t * F < D1
                    for (int64_t t = floor_div(D0 - run_lo + F - 1, F, inv_frame_bytes) + lane_id();
                         run_lo + t * F < D1 && t < len; t += kWave) {
                        store_slot(a, g + t, r.seq, (int32_t)t);
                    }
                }
                return;
            }
            // next most common: the tile lies in the zero tail of the run's block
            if (run_lo + len * F <= D0 && ((int64_t)r.block + 1) * T * F >= D0 + tile_bytes) {
                const vec16 z = {0u, 0u, 0u, 0u};
                store_stream(reinterpret_cast<vec16*>(a.packed + D0) + threadIdx.x, z);
                if (table_wave) {
                    for (int64_t slot = floor_div(D0 + F - 1, F, inv_frame_bytes) + lane_id(); slot * F < D1;
                         slot += kWave) {
                        store_slot(a, slot, -1, -1);
                    }
                }
                return;
            }
        }
    }

    const int64_t gs_lo = floor_div(D0, F, inv_frame_bytes);              // first slot touched
    const int64_t gs_hi = floor_div(D1 + F - 1, F, inv_frame_bytes);      // one past the last
    // slots whose first byte lies in this tile get their start-table entry here
    const int64_t m_lo = gs_lo + ((gs_lo * F < D0) ? 1 : 0);
    const int64_t m_hi = min(gs_hi, a.total_slots);

    // A tile that few runs touch walks them one after the other (their look-ups are scalar
    // loads, the whole workgroup copies each run's part).  The shuffled position in front of
    // the next tile bounds the number of runs from above.
    const int32_t p_next = (tile + 1 < gridDim.x) ? min(max(first_pos[tile + 1], 0), n_seq) : n_seq - 1;
    if (p_next - p + 1 <= kWideWalkRuns) {
        // runs in destination order from there on, zeros in the gaps (block tails)
        int64_t cursor = D0;          // payload bytes written so far
        int64_t mcursor = m_lo;       // start-table slots written so far
        for (; p < n_seq; ++p) {
            const Run r = runs[p];
            const int64_t g = r.dst;
            if (g >= gs_hi) break;                    // also the end of the list (kNoRun)
            const int64_t len = r.len;
            if (g + len <= gs_lo) continue;           // ends before the tile: the tile starts in padding
            const int64_t run_lo = g * F;
            const int64_t lo = max(max(run_lo, D0), cursor);
            const int64_t hi = min(run_lo + len * F, D1);
            if (hi > lo) {
                if (lo > cursor) write_range<true>(a.packed, cursor, lo, nullptr);
                write_range<false>(a.packed, lo, hi, a.src + r.src * F + (lo - run_lo));
                cursor = hi;
            }
            if (table_wave) {
                const int64_t s_lo = max(g, mcursor), s_hi = min(g + len, m_hi);
                if (s_lo > mcursor) write_slots(a, mcursor, s_lo, -1, -1);
                if (s_hi > s_lo) { write_slots(a, s_lo, s_hi, r.seq, s_lo - g); mcursor = s_hi; }
            }
        }
        if (cursor < D1) write_range<true>(a.packed, cursor, D1, nullptr);
        if (table_wave && mcursor < m_hi) write_slots(a, mcursor, m_hi, -1, -1);
        return;
    }

    // Every other tile: the runs that touch it are looked up side by side (thread k takes the
    // k-th shuffled position from p on), so that the cost does not grow with their number, and
    // every thread then finds the run of its own 16 bytes.  A frame of kWideMinFrame bytes or
    // more puts at most kWideTile / kWideMinFrame + 2 runs into a tile.
    __shared__ int64_t s_run_lo[kWideRuns + 1];     // first packed byte of the run; INT64_MAX: no run
    __shared__ int64_t s_run_hi[kWideRuns];         // one past its last packed byte
    __shared__ int64_t s_run_src[kWideRuns];        // source byte that goes to s_run_lo
    __shared__ int32_t s_run_seq[kWideRuns];
    const int tid = (int)threadIdx.x;
    if (tid <= kWideRuns) {
        int64_t lo = INT64_MAX, hi = 0, from = 0;
        int32_t seq = -1;
        const int64_t pos = (int64_t)p + tid;
        if (tid < kWideRuns && pos < n_seq) {
            const Run r = runs[pos];
            if (r.dst < gs_hi) {
                lo = r.dst * F;
                hi = lo + (int64_t)r.len * F;
                from = r.src * F;
                seq = r.seq;
            }
        }
        s_run_lo[tid] = lo;
        if (tid < kWideRuns) {
            s_run_hi[tid] = hi;
            s_run_src[tid] = from;
            s_run_seq[tid] = seq;
        }
    }
    __syncthreads();
    // last gathered run that starts at or before packed byte x, -1 if none
    // (a binary search over the first `span` entries, span = a power of two that covers them)
    int span = 1;
    while (span < min(p_next - p + 2, kWideRuns)) span <<= 1;
    auto run_at = [&](int64_t x) {
        int k = -1;
        for (int step = span >> 1; step >= 1; step >>= 1)
            if (s_run_lo[k + step] <= x) k += step;
        if (s_run_lo[k + 1] <= x) ++k;
        return k;
    };

    for (int64_t x0 = D0 + 16 * (int64_t)tid; x0 < D1; x0 += 16 * (int64_t)kThreads) {
        int k = run_at(x0);
        const int64_t next_lo = s_run_lo[k + 1];
        const int64_t lo = k >= 0 ? s_run_lo[k] : 0, hi = k >= 0 ? s_run_hi[k] : 0;
        vec16* dst = reinterpret_cast<vec16*>(a.packed + x0);
        if (x0 + 16 <= D1 && x0 + 16 <= hi) {                           // inside one run
            const uint8_t* from = a.src + s_run_src[k] + (x0 - lo);
            store_stream(dst, __builtin_nontemporal_load(reinterpret_cast<const vec16_unaligned*>(from)));
        } else if (x0 + 16 <= D1 && x0 >= hi && x0 + 16 <= next_lo) {   // inside a block's zero tail
            const vec16 z = {0u, 0u, 0u, 0u};
            store_stream(dst, z);
        } else {                                                        // a border inside: byte by byte
            for (int j = 0; j < 16 && x0 + j < D1; ++j) {
                const int64_t x = x0 + j;
                while (s_run_lo[k + 1] <= x) ++k;
                uint8_t v = 0;
                if (k >= 0 && x < s_run_hi[k]) v = a.src[s_run_src[k] + (x - s_run_lo[k])];
                a.packed[x] = v;
            }
        }
    }
    if (table_wave) {
        for (int64_t slot = m_lo + lane_id(); slot < m_hi; slot += kWave) {
            const int64_t x = slot * F;
            const int k = run_at(x);
            int32_t seq = -1, fid = -1;
            if (k >= 0 && x < s_run_hi[k]) {
                seq = s_run_seq[k];
                fid = (int32_t)(slot - floor_div(s_run_lo[k], F, inv_frame_bytes));
            }
            store_slot(a, slot, seq, fid);
        }
    }
}

// ----------------------------------------------------------------- narrow

constexpr int kNarrowSlots = kTableSlots;            // slots per workgroup
constexpr int kNarrowMaxRuns = kNarrowSlots + 2;

// The run a lane is currently reading from, kept in registers and advanced
// as the lane walks over consecutive slots.
template <int MAXRUNS>
struct RunCursor {
    const RunTable<MAXRUNS>& tab;
    int r;
    int32_t dst, end, next, seq;
    int64_t src;

    __device__ __forceinline__ RunCursor(const RunTable<MAXRUNS>& t, int n, int32_t slot)
        : tab(t)
    {
        r = run_of_slot(t, n, slot);
        load();
    }
    __device__ __forceinline__ void load()
    {
        next = tab.dst[r + 1];
        if (r >= 0) { dst = tab.dst[r]; end = tab.end[r]; seq = tab.seq[r]; src = tab.src[r]; }
        else        { dst = 0; end = 0; seq = -1; src = 0; }
    }
    // frame index of `slot` inside the current run, or -1 on padding
    __device__ __forceinline__ int32_t seek(int32_t slot)
    {
        while (slot >= next) { ++r; load(); }
        return (r >= 0 && slot < end) ? slot - dst : -1;
    }
};

// What a tile of kNarrowSlots slots is, as far as the run its entry names can tell.
enum NarrowKind : int { kTileGeneral = 0, kTileOneRun = 1, kTilePadding = 2, kTileAbsent = 3 };

// The start-table entries of a whole tile that lies inside one run (`r`), or inside the padding
// behind a block's last run (`r` null): four slots per lane, without a look at any table.
__device__ __forceinline__ void narrow_uniform_table(const PackArgs& a, int64_t g0, const Run* r)
{
    const int64_t g = g0 + 4 * (int)threadIdx.x;
    vec16 vs = {~0u, ~0u, ~0u, ~0u}, vf = vs;
    uint32_t rs = 0, vl = 0;
    if (r) {
        const uint32_t fid = (uint32_t)(g - r->dst);           // >= 0: the run begins at or before the tile
        vs = vec16{(uint32_t)r->seq, (uint32_t)r->seq, (uint32_t)r->seq, (uint32_t)r->seq};
        vf = vec16{fid, fid + 1u, fid + 2u, fid + 3u};
        rs = fid == 0u ? 1u : 0u;
        vl = 0x01010101u;
    }
    store_stream(reinterpret_cast<vec16*>(a.seq_id + g), vs);
    store_stream(reinterpret_cast<vec16*>(a.frame_idx + g), vf);
    __builtin_nontemporal_store(rs, reinterpret_cast<uint32_t*>(a.reset + g));
    __builtin_nontemporal_store(vl, reinterpret_cast<uint32_t*>(a.valid + g));
}

// The payload of such a tile: per step one 16-byte vector per lane.
__device__ __forceinline__ void narrow_uniform_payload(const PackArgs& a, int64_t g0, const Run* r)
{
    const int tid = (int)threadIdx.x;
    const int64_t F = a.frame_bytes;
    vec16* dst = reinterpret_cast<vec16*>(a.packed + g0 * F);      // 16-byte aligned: g0 is a multiple of 1024
    const int32_t nvec = (int32_t)(kNarrowSlots * F / 16);
    if (r) {
        const uint8_t* from = a.src + (r->src + (g0 - r->dst)) * F;
        for (int32_t v = tid; v < nvec; v += kThreads)
            store_stream(dst + v, __builtin_nontemporal_load(reinterpret_cast<const vec16_unaligned*>(from) + v));
    } else {
        const vec16 z = {0u, 0u, 0u, 0u};
        for (int32_t v = tid; v < nvec; v += kThreads) store_stream(dst + v, z);
    }
}

// A 16-byte vector put together from elements of type E (1, 2, 4 or 16 bytes).  Element numbers
// are compile-time constants where it is used, so the vector stays in registers.
template <typename E>
struct Assembled {
    vec16 vec = {0u, 0u, 0u, 0u};
    __device__ __forceinline__ void set(int e, E v)
    {
        vec[e * (int)sizeof(E) / 4] |= (uint32_t)v << (8 * (e * (int)sizeof(E) % 4));
    }
    __device__ __forceinline__ E get(int e) const
    {
        return (E)(vec[e * (int)sizeof(E) / 4] >> (8 * (e * (int)sizeof(E) % 4)));
    }
};
template <>
struct Assembled<vec16> {
    vec16 vec = {0u, 0u, 0u, 0u};
    __device__ __forceinline__ void set(int, vec16 v) { vec = v; }
    __device__ __forceinline__ vec16 get(int) const { return vec; }
};

// One tile of kNarrowSlots slots (or the shorter last one) that needs its runs looked up: the
// candidates `first` .. `last` of the run table are gathered into `tab` first.  Called by the
// whole workgroup.
template <typename E, bool FUSED, bool PAYLOAD, bool TABLE>
__device__ __forceinline__ void narrow_general_tile(const PackArgs& a, const Run* __restrict__ runs,
                                                    RunTable<kNarrowMaxRuns>& tab, int64_t g0, int64_t g1,
                                                    int32_t first, int32_t last)
{
    const int tid = (int)threadIdx.x;
    const int nslot = (int)(g1 - g0);
    const int n = gather_runs(runs, a.n_seq, first, last, g0, g1, tab);

    // start table (and, FUSED, the payload): 4 consecutive slots per lane -> 16-byte / 4-byte stores
    for (int q = tid; (TABLE || FUSED) && 4 * q < nslot; q += kThreads) {
        const int32_t s0 = 4 * q;
        RunCursor<kNarrowMaxRuns> cur(tab, n, s0);
        int32_t sid[4], fid[4];
        int64_t from[4];                 // source frame of each slot (FUSED only)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            fid[j] = (s0 + j < nslot) ? cur.seek(s0 + j) : -1;
            sid[j] = fid[j] >= 0 ? cur.seq : -1;
            from[j] = cur.src + fid[j];
        }
        if (FUSED && s0 + 4 <= nslot) {
            const uint32_t* src32 = reinterpret_cast<const uint32_t*>(a.src);
            vec16 pv;
            if (fid[0] >= 0 && sid[3] == sid[0] && fid[3] == fid[0] + 3) {
                // one run: 16 contiguous source bytes (4-byte aligned)
                typedef vec16 __attribute__((aligned(4))) vec16_a4;
                pv = __builtin_nontemporal_load(reinterpret_cast<const vec16_a4*>(src32 + from[0]));
            } else {
                uint32_t e0 = 0u, e1 = 0u, e2 = 0u, e3 = 0u;
                if (fid[0] >= 0) e0 = src32[from[0]];
                if (fid[1] >= 0) e1 = src32[from[1]];
                if (fid[2] >= 0) e2 = src32[from[2]];
                if (fid[3] >= 0) e3 = src32[from[3]];
                pv = vec16{e0, e1, e2, e3};
            }
            store_stream(reinterpret_cast<vec16*>(a.packed + (g0 + s0) * 4), pv);
        }
        if (!TABLE) continue;
        const int64_t g = g0 + s0;
        if (s0 + 4 <= nslot) {
            const vec16 vs = {(uint32_t)sid[0], (uint32_t)sid[1], (uint32_t)sid[2], (uint32_t)sid[3]};
            const vec16 vf = {(uint32_t)fid[0], (uint32_t)fid[1], (uint32_t)fid[2], (uint32_t)fid[3]};
            store_stream(reinterpret_cast<vec16*>(a.seq_id + g), vs);
            store_stream(reinterpret_cast<vec16*>(a.frame_idx + g), vf);
            uint32_t rs = 0, vl = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                rs |= (uint32_t)(fid[j] == 0) << (8 * j);
                vl |= (uint32_t)(fid[j] >= 0) << (8 * j);
            }
            __builtin_nontemporal_store(rs, reinterpret_cast<uint32_t*>(a.reset + g));
            __builtin_nontemporal_store(vl, reinterpret_cast<uint32_t*>(a.valid + g));
        } else {
            for (int j = 0; s0 + j < nslot; ++j) {
                store_slot(a, g + j, sid[j], fid[j]);
            }
        }
    }

    if (!PAYLOAD) return;
    // payload: one 16-byte destination vector per lane and step, assembled
    // from elements of type E (k elements per frame)
    constexpr int EPV = 16 / (int)sizeof(E);
    const int done_slots = FUSED ? (nslot & ~3) : 0;            // already written above
    const int32_t k = (int32_t)(a.frame_bytes / (int64_t)sizeof(E));
    const int32_t tile_elems = nslot * k;                       // < 1024 * 512
    const int32_t nvec = (tile_elems + EPV - 1) / EPV;
    const E* src = reinterpret_cast<const E*>(a.src);
    uint8_t* dst_tile = a.packed + g0 * a.frame_bytes;          // 16-byte aligned
    for (int32_t v = (FUSED ? done_slots / 4 : 0) + tid; v < nvec; v += kThreads) {
        const int32_t w = v * EPV;
        int32_t slot = w / k;
        int32_t j = w - slot * k;
        RunCursor<kNarrowMaxRuns> cur(tab, n, slot);
        const int nvalid = min(EPV, tile_elems - w);
        Assembled<E> u;
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            E val{};
            if (e < nvalid) {
                const int32_t t = cur.seek(slot);
                if (t >= 0) val = src[(cur.src + t) * k + j];
                if (++j == k) { j = 0; ++slot; }
            }
            u.set(e, val);
        }
        if (nvalid == EPV) {
            store_stream(reinterpret_cast<vec16*>(dst_tile) + v, u.vec);
        } else {
#pragma unroll
            for (int e = 0; e < EPV; ++e)
                if (e < nvalid) reinterpret_cast<E*>(dst_tile)[w + e] = u.get(e);
        }
    }
}

// FUSED (4-byte frames, e.g. tokens): the four slots of a lane's start-table
// quad are also exactly one 16-byte vector of payload, so both are written in
// the same pass and the payload pass is skipped.
//
// PAYLOAD false: only the start table is written; TABLE false: only the payload.  Large tensors
// of 4-byte frames are packed in two such passes, and the start table of large tensors of wide
// frames, whose payload the 4 KiB tiles copy, by the first of them: five output streams written
// at once reach 5.1-5.2 TB/s on this GPU, the payload alone 6.0 and the four planes of the table
// alone 6.2 (plain streaming kernels with this traffic, 2^30 tokens: 3.46 ms in one pass, 1.17 +
// 1.73 ms in two).
//
// GROUP consecutive tiles per workgroup.  What decides a tile's kind hangs on two look-ups, one
// after the other (the tile's entry, then the run it names), and the payload on a third: with
// several tiles per workgroup the look-ups of a stage are asked for together, and so is the
// payload of all tiles that lie inside one run, so that a wave has GROUP times the bytes in
// flight per wait.  Tiles that need their runs gathered follow one by one.
template <typename E, bool FUSED, bool PAYLOAD = true, bool TABLE = true, int GROUP = 1>
__global__ __launch_bounds__(kThreads) void pack_narrow_kernel(PackArgs a, const Run* __restrict__ runs,
                                                               const int32_t* __restrict__ first_pos,
                                                               uint32_t n_tiles)
{
    static_assert(PAYLOAD || !FUSED, "the fused form is about the payload");
    static_assert(PAYLOAD || TABLE, "a pass writes something");
    __shared__ RunTable<kNarrowMaxRuns> tab;
    const int tid = (int)threadIdx.x;
    const uint32_t tile0 = xcd_contiguous(blockIdx.x, gridDim.x) * (uint32_t)GROUP;

    // entry[u]: where tile tile0 + u starts in the run table; behind the last tile: the last run
    int32_t entry[GROUP + 1];
#pragma unroll
    for (int u = 0; u <= GROUP; ++u) {
        const uint32_t t = tile0 + (uint32_t)u;
        entry[u] = first_pos[min(t, n_tiles - 1u)];
    }
#pragma unroll
    for (int u = 0; u <= GROUP; ++u)
        entry[u] = tile0 + (uint32_t)u < n_tiles ? min(max(entry[u], 0), a.n_seq) : a.n_seq - 1;

    // The two most common tiles where sequences are long need no table: a tile inside one run,
    // and a tile inside the padding behind its block's last run.  The tile's entry names the
    // last run of the tile's first block that begins at or before the tile; that record alone
    // tells (runs of a block follow each other without a gap).  Wave-uniform look-ups, no LDS,
    // no barrier: every wave decides alone and all decide alike.
    Run r[GROUP];
#pragma unroll
    for (int u = 0; u < GROUP; ++u) r[u] = runs[min(entry[u], a.n_seq - 1)];
    int kind[GROUP];
#pragma unroll
    for (int u = 0; u < GROUP; ++u) {
        const uint32_t t = tile0 + (uint32_t)u;
        const int64_t g0 = (int64_t)t * kNarrowSlots, g1 = g0 + kNarrowSlots;
        kind[u] = kTileGeneral;
        if (t >= n_tiles) {
            kind[u] = kTileAbsent;
        } else if (g1 <= a.total_slots && entry[u] < a.n_seq && r[u].dst != kNoRun) {
            if (r[u].dst <= g0 && r[u].dst + r[u].len >= g1) kind[u] = kTileOneRun;
            else if (r[u].dst + r[u].len <= g0 && ((int64_t)r[u].block + 1) * a.t_blk >= g1) kind[u] = kTilePadding;
        }
    }

    if (PAYLOAD && FUSED) {
        // 4-byte frames: a tile's payload is one 16-byte vector per lane
        vec16 pv[GROUP];
#pragma unroll
        for (int u = 0; u < GROUP; ++u) {
            pv[u] = vec16{0u, 0u, 0u, 0u};
            if (kind[u] == kTileOneRun) {
                const int64_t g0 = (int64_t)(tile0 + (uint32_t)u) * kNarrowSlots;
                const uint8_t* from = a.src + (r[u].src + (g0 - r[u].dst)) * 4;
                pv[u] = __builtin_nontemporal_load(reinterpret_cast<const vec16_unaligned*>(from) + tid);
            }
        }
#pragma unroll
        for (int u = 0; u < GROUP; ++u) {
            if (kind[u] == kTileOneRun || kind[u] == kTilePadding) {
                const int64_t g0 = (int64_t)(tile0 + (uint32_t)u) * kNarrowSlots;
                store_stream(reinterpret_cast<vec16*>(a.packed + g0 * 4) + tid, pv[u]);
            }
        }
    } else if (PAYLOAD) {
#pragma unroll
        for (int u = 0; u < GROUP; ++u) {
            const int64_t g0 = (int64_t)(tile0 + (uint32_t)u) * kNarrowSlots;
            if (kind[u] == kTileOneRun) narrow_uniform_payload(a, g0, &r[u]);
            else if (kind[u] == kTilePadding) narrow_uniform_payload(a, g0, nullptr);
        }
    }
    if (TABLE) {
#pragma unroll
        for (int u = 0; u < GROUP; ++u) {
            const int64_t g0 = (int64_t)(tile0 + (uint32_t)u) * kNarrowSlots;
            if (kind[u] == kTileOneRun) narrow_uniform_table(a, g0, &r[u]);
            else if (kind[u] == kTilePadding) narrow_uniform_table(a, g0, nullptr);
        }
    }

    bool table_in_use = false;
#pragma unroll
    for (int u = 0; u < GROUP; ++u) {
        if (kind[u] != kTileGeneral) continue;
        const int64_t g0 = (int64_t)(tile0 + (uint32_t)u) * kNarrowSlots;
        if (table_in_use) __syncthreads();           // the tile before is done with the gathered runs
        narrow_general_tile<E, FUSED, PAYLOAD, TABLE>(a, runs, tab, g0, min(g0 + kNarrowSlots, a.total_slots),
                                                      entry[u], entry[u + 1]);
        table_in_use = true;
    }
}

// ------------------------------------------------------------------ check
//
// Are the tables a plan: every rule is local to one shuffled position (or one block), so
// one thread tests one of each; the smallest failing index is kept with an atomic minimum.
__global__ __launch_bounds__(kThreads) void pack_check_kernel(
    const int64_t* __restrict__ src_offsets, const int32_t* __restrict__ lengths,
    const int32_t* __restrict__ order, const int32_t* __restrict__ block_of_seq,
    const int32_t* __restrict__ offset_of_seq, const int32_t* __restrict__ block_first,
    int32_t n_seq, int32_t num_blocks, int32_t t_blk, int64_t total_frames,
    unsigned long long* __restrict__ first_bad)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    bool bad = false;
    // block idx: its range of positions
    if (idx < num_blocks) {
        const int64_t lo = block_first[idx], hi = block_first[idx + 1];
        bad |= lo < 0 || hi < lo || hi > n_seq || (idx == 0 && lo != 0);
    }
    // position idx: its sequence
    const int64_t listed = min(max((int64_t)block_first[num_blocks], (int64_t)0), (int64_t)n_seq);
    if (idx < listed) {
        const uint32_t i = (uint32_t)order[idx];
        if (i >= (uint32_t)n_seq) {
            bad = true;
        } else {
            const int64_t b = block_of_seq[i], off = offset_of_seq[i], len = lengths[i];
            const int64_t from = src_offsets[i];
            bad |= len < 1 || off < 0 || off + len > t_blk;
            bad |= from < 0 || from + len > total_frames || src_offsets[i + 1] - from != len;
            if (b < 0 || b >= num_blocks) {
                bad = true;
            } else {
                const int64_t lo = block_first[b], hi = block_first[b + 1];
                if (lo < 0 || idx < lo || idx >= hi) {
                    bad = true;
                } else if (idx == lo) {
                    bad |= off != 0;
                } else {
                    const uint32_t before = (uint32_t)order[idx - 1];
                    bad |= before >= (uint32_t)n_seq ||
                           (before < (uint32_t)n_seq &&
                            off != (int64_t)offset_of_seq[before] + (int64_t)lengths[before]);
                }
            }
        }
    }
    if (bad) atomicMin(first_bad, (unsigned long long)idx);
}

__global__ void pack_check_clear_kernel(unsigned long long* first_bad) { *first_bad = ~0ull; }

}  // namespace bload

using namespace bload;

// Which tile shape packs faster, from what the host knows.  The 4 KiB tiles win where runs
// (a sequence's bytes) are long: a tile inside one run is a plain copy.  The 1024-slot tiles
// amortise their run table better where many short runs meet, and copy 16 bytes per lane when
// frames are multiples of 16 bytes and the source is aligned.  Measured crossovers, in bytes
// per run (bounded from above here by packed bytes / sequences).
static bool takes_wide_tiles(int64_t frame_bytes, int64_t total_bytes, int64_t n_seq, bool src_aligned16)
{
    if (frame_bytes < kWideMinFrame) return false;
    if (frame_bytes >= 512) return true;
    const int64_t run_bytes = total_bytes / (n_seq > 0 ? n_seq : 1);
    const bool narrow_copies_vectors = frame_bytes % 16 == 0 && src_aligned16;
    return run_bytes >= (narrow_copies_vectors ? 24 * 1024 : 4 * 1024);
}

extern "C" int32_t bload_pack_tile_bytes(int64_t n_seq, int64_t num_blocks, int32_t t_blk,
                                         int64_t frame_bytes, int32_t src_aligned_16)
{
    if (n_seq < 0 || num_blocks <= 0 || t_blk < 1 || frame_bytes < 1) return 0;
    const int64_t total_slots = num_blocks * (int64_t)t_blk;
    if (total_slots >= ((int64_t)1 << 40) || total_slots > (((int64_t)1 << 52) - 1) / frame_bytes) return 0;
    return takes_wide_tiles(frame_bytes, total_slots * frame_bytes, n_seq, src_aligned_16 != 0) ? kWideTile : 0;
}

namespace {

// Workspace: the run table, then one int32 per tile.
struct PackLayout {
    bool wide;
    int64_t tiles;
    int64_t table_tiles;       // slot tiles of the separate start-table pass (wide frames, large tensors), else 0
    size_t runs_off, first_off, table_off, bytes;
};

// From this many slots on, the start table of wide frames is written by a pass of its own, in
// slot tiles with full-width stores: the few entries per 4 KiB tile, written by that tile's first
// wave, are 2 % of the bytes and cost 5 % of the time (10^8 slots of 320 bytes: 9.64 ms, 9.11 ms
// without them, 9.36 ms with the pass).  About 3 ns per 1000 slots: below a couple of million
// slots the pass saves less than its launch costs, and the one pass stays.
constexpr int64_t kTablePassFromSlots = (int64_t)1 << 21;
// Tiles per workgroup in the passes that large tensors get (pack_narrow_kernel's GROUP).  Measured on
// 0.8-1.3 * 10^9 token slots of four length mixes: two tiles 1-3.5 % faster than one, four between 3 %
// slower and 2 % faster, eight 40 % slower.
constexpr int kPassGroup = 2;

// Sizes the caller cannot know in advance (which tile shape the lengths will choose) are
// taken at their larger value when `for_query`.
bool pack_layout(int64_t n_seq, int64_t num_blocks, int32_t t_blk, int64_t frame_bytes,
                 bool src_aligned16, bool for_query, PackLayout* l)
{
    const int64_t total_slots = num_blocks * (int64_t)t_blk;
    if (total_slots >= ((int64_t)1 << 40) || total_slots > (((int64_t)1 << 52) - 1) / frame_bytes) return false;
    const int64_t total_bytes = total_slots * frame_bytes;
    const int64_t wide_tiles = ceil_div(total_bytes, kWideTile), narrow_tiles = ceil_div(total_slots, kNarrowSlots);
    if (for_query) {
        // frames that may take either shape get room for the 4 KiB tiles, which are more
        l->wide = frame_bytes >= kWideMinFrame;
        l->tiles = l->wide ? (wide_tiles > narrow_tiles ? wide_tiles : narrow_tiles) : narrow_tiles;
    } else {
        l->wide = takes_wide_tiles(frame_bytes, total_bytes, n_seq, src_aligned16);
        l->tiles = l->wide ? wide_tiles : narrow_tiles;
    }
    l->table_tiles = l->wide && total_slots >= kTablePassFromSlots ? narrow_tiles : 0;
    l->runs_off = 0;
    l->first_off = round_up((size_t)n_seq * sizeof(Run), 32);
    l->table_off = l->first_off + round_up((size_t)l->tiles * sizeof(int32_t), 16);
    l->bytes = l->table_off + round_up((size_t)l->table_tiles * sizeof(int32_t), 16);
    return true;
}

// Argument checks shared by the entry points that pack.
bload_status pack_check_args(const void* d_src, const int64_t* d_src_offsets, const int32_t* d_lengths,
                             const int32_t* d_order, const int32_t* d_block_of_seq,
                             const int32_t* d_offset_of_seq, const int32_t* d_block_first, int64_t n_seq,
                             int64_t num_blocks, int32_t t_blk, int64_t frame_bytes, void* d_packed,
                             int32_t* d_seq_id, int32_t* d_frame_idx, uint8_t* d_reset, uint8_t* d_valid)
{
    if (!d_src || !d_src_offsets || !d_lengths || !d_order || !d_block_of_seq ||
        !d_offset_of_seq || !d_block_first || !d_packed || !d_seq_id || !d_frame_idx ||
        !d_reset || !d_valid)
        return BLOAD_EINVAL;
    const int64_t total_slots = num_blocks * (int64_t)t_blk;
    if (total_slots >= ((int64_t)1 << 40) || frame_bytes >= ((int64_t)1 << 31) ||
        total_slots > INT64_MAX / frame_bytes / 2 || total_slots * frame_bytes >= ((int64_t)1 << 52))
        return BLOAD_EOVERFLOW;
    if (!aligned_to(d_packed, 16) || !aligned_to(d_seq_id, 16) || !aligned_to(d_frame_idx, 16) ||
        !aligned_to(d_reset, 16) || !aligned_to(d_valid, 16) || !aligned_to(d_src_offsets, 8) ||
        !aligned_to(d_lengths, 4) || !aligned_to(d_order, 4) || !aligned_to(d_block_of_seq, 4) ||
        !aligned_to(d_offset_of_seq, 4) || !aligned_to(d_block_first, 4))
        return BLOAD_EALIGN;
    return BLOAD_OK;
}

// Enqueue the two passes.  `ws` holds l.bytes bytes, 32-byte aligned or better.
bload_status pack_enqueue(const PackLayout& l, const void* d_src, const int64_t* d_src_offsets,
                          const int32_t* d_lengths, const int32_t* d_order, const int32_t* d_block_of_seq,
                          const int32_t* d_offset_of_seq, const int32_t* d_block_first, int64_t n_seq,
                          int64_t num_blocks, int32_t t_blk, int64_t frame_bytes, void* d_packed,
                          int32_t* d_seq_id, int32_t* d_frame_idx, uint8_t* d_reset, uint8_t* d_valid,
                          uint8_t* ws, hipStream_t stream)
{
    if (l.tiles > INT32_MAX || l.table_tiles > INT32_MAX) return BLOAD_EOVERFLOW;
    Run* runs = reinterpret_cast<Run*>(ws + l.runs_off);
    int32_t* first_pos = reinterpret_cast<int32_t*>(ws + l.first_off);
    int32_t* first_pos_table = reinterpret_cast<int32_t*>(ws + l.table_off);
    PackArgs a;
    a.src = static_cast<const uint8_t*>(d_src);
    a.runs = runs;
    a.n_seq = (int32_t)n_seq;
    a.t_blk = t_blk;
    a.frame_bytes = frame_bytes;
    a.total_slots = num_blocks * (int64_t)t_blk;
    a.packed = static_cast<uint8_t*>(d_packed);
    a.seq_id = d_seq_id;
    a.frame_idx = d_frame_idx;
    a.reset = d_reset;
    a.valid = d_valid;

    // pass 1 (both tile shapes): the run table, and where each tile starts in it.  The
    // narrow tiles are 1024 slots, which the kernel takes as "1024 bytes of 1-byte frames".
    const int64_t unit_bytes = l.wide ? frame_bytes : 1;
    const int32_t tile_units = l.wide ? kWideTile : kNarrowSlots;
    const double inv_unit = 1.0 / (double)unit_bytes, inv_t = 1.0 / (double)t_blk;
    const int64_t prepare_threads = l.tiles > n_seq ? l.tiles : n_seq;       // table_tiles <= tiles
    hipLaunchKernelGGL(pack_prepare_kernel, dim3((uint32_t)ceil_div(prepare_threads, kThreads)),
                       dim3(kThreads), 0, stream, d_src_offsets, d_lengths, d_order, d_block_of_seq,
                       d_offset_of_seq, d_block_first, (int32_t)n_seq, num_blocks, (int64_t)t_blk, unit_bytes,
                       l.tiles, tile_units, inv_unit, inv_t, runs, first_pos, l.table_tiles, first_pos_table);
    const dim3 grid((uint32_t)l.tiles), block(kThreads);
    const uint32_t n_tiles = (uint32_t)l.tiles;
    if (l.wide) {
        hipLaunchKernelGGL(pack_wide_kernel, grid, block, 0, stream, a, runs, first_pos, kWideTile, inv_unit,
                           l.table_tiles == 0 ? 1 : 0);
        if (l.table_tiles > 0)
            hipLaunchKernelGGL((pack_narrow_kernel<uint8_t, false, false, true, kPassGroup>),
                               dim3((uint32_t)ceil_div(l.table_tiles, kPassGroup)), block, 0, stream, a, runs,
                               first_pos_table, (uint32_t)l.table_tiles);
        return launch_status();
    }
    // slot tiles: one pass; 4-byte frames (whose payload and table share a loop, so that one kernel writes
    // five streams at once) from kTablePassFromSlots slots on: the payload and the start table in a pass
    // each over the same tiles.  Measured on 1.3 * 10^9 token slots: 3.98 -> 3.72 ms; frames of 6 and 8
    // bytes, whose one pass already writes the table first and the payload after it, lose 5-7 % to the
    // second pass's look-ups and keep the one pass.
    if (frame_bytes % 16 == 0 && aligned_to(d_src, 16)) {
        hipLaunchKernelGGL((pack_narrow_kernel<vec16, false>), grid, block, 0, stream, a, runs, first_pos, n_tiles);
    } else if (frame_bytes == 4 && aligned_to(d_src, 4)) {
        if (a.total_slots >= kTablePassFromSlots) {
            const dim3 groups((uint32_t)ceil_div(l.tiles, kPassGroup));
            hipLaunchKernelGGL((pack_narrow_kernel<uint32_t, true, true, false, kPassGroup>), groups, block, 0, stream,
                               a, runs, first_pos, n_tiles);
            hipLaunchKernelGGL((pack_narrow_kernel<uint8_t, false, false, true, kPassGroup>), groups, block, 0, stream,
                               a, runs, first_pos, n_tiles);
        } else {
            hipLaunchKernelGGL((pack_narrow_kernel<uint32_t, true>), grid, block, 0, stream, a, runs, first_pos, n_tiles);
        }
    } else if (frame_bytes % 4 == 0 && aligned_to(d_src, 4)) {
        hipLaunchKernelGGL((pack_narrow_kernel<uint32_t, false>), grid, block, 0, stream, a, runs, first_pos, n_tiles);
    } else if (frame_bytes % 2 == 0 && aligned_to(d_src, 2)) {
        hipLaunchKernelGGL((pack_narrow_kernel<uint16_t, false>), grid, block, 0, stream, a, runs, first_pos, n_tiles);
    } else {
        hipLaunchKernelGGL((pack_narrow_kernel<uint8_t, false>), grid, block, 0, stream, a, runs, first_pos, n_tiles);
    }
    return launch_status();
}

}  // namespace

extern "C" size_t bload_pack_workspace_bytes(int64_t n_seq, int64_t num_blocks, int32_t t_blk,
                                             int64_t frame_bytes)
{
    if (n_seq <= 0 || n_seq > BLOAD_MAX_SEQ || num_blocks <= 0 || t_blk < 1 || frame_bytes < 1) return 0;
    PackLayout l;
    if (!pack_layout(n_seq, num_blocks, t_blk, frame_bytes, true, true, &l)) return 0;
    return l.bytes;
}

extern "C" bload_status bload_pack(const void* d_src, const int64_t* d_src_offsets,
                                   const int32_t* d_lengths, const int32_t* d_order,
                                   const int32_t* d_block_of_seq, const int32_t* d_offset_of_seq,
                                   const int32_t* d_block_first, int64_t n_seq, int64_t num_blocks,
                                   int32_t t_blk, int64_t frame_bytes, void* d_packed,
                                   int32_t* d_seq_id, int32_t* d_frame_idx, uint8_t* d_reset,
                                   uint8_t* d_valid, void* d_workspace, size_t workspace_bytes,
                                   void* hip_stream)
{
    if (n_seq < 0 || num_blocks < 0 || t_blk < 1 || frame_bytes < 1) return BLOAD_EINVAL;
    if (n_seq > BLOAD_MAX_SEQ || num_blocks > n_seq) return n_seq > BLOAD_MAX_SEQ ? BLOAD_EOVERFLOW
                                                                                 : BLOAD_EINVAL;
    if (n_seq == 0 || num_blocks == 0) return BLOAD_OK;
    const bload_status st = pack_check_args(d_src, d_src_offsets, d_lengths, d_order, d_block_of_seq,
                                            d_offset_of_seq, d_block_first, n_seq, num_blocks, t_blk,
                                            frame_bytes, d_packed, d_seq_id, d_frame_idx, d_reset, d_valid);
    if (st != BLOAD_OK) return st;
    PackLayout l;
    if (!pack_layout(n_seq, num_blocks, t_blk, frame_bytes, aligned_to(d_src, 16), false, &l))
        return BLOAD_EOVERFLOW;
    if (!d_workspace) return BLOAD_EINVAL;
    if (!aligned_to(d_workspace, 32)) return BLOAD_EALIGN;
    if (workspace_bytes < l.bytes) return BLOAD_EWORKSPACE;
    return pack_enqueue(l, d_src, d_src_offsets, d_lengths, d_order, d_block_of_seq, d_offset_of_seq,
                        d_block_first, n_seq, num_blocks, t_blk, frame_bytes, d_packed, d_seq_id,
                        d_frame_idx, d_reset, d_valid, static_cast<uint8_t*>(d_workspace),
                        static_cast<hipStream_t>(hip_stream));
}

// ---------------------------------------------------- bload_pack_noalloc
//
// bload_pack for callers that cannot bring a workspace: the run table and the tiles'
// entries live in a fixed array in device memory that is part of the loaded library.
// Every GPU the library runs on holds its own copy of the array, at its own address,
// until the process ends; the address is asked for once per device.

constexpr size_t kStaticRunBytes = (size_t)BLOAD_PACK_NOALLOC_MAX_SEQ * sizeof(Run);
constexpr size_t kStaticBytes = kStaticRunBytes + (size_t)BLOAD_PACK_NOALLOC_MAX_TILES * sizeof(int32_t);
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_of_device[kMaxDevices] = {};

// Device address of `scratch` on the current device.
bload_status static_scratch(uint8_t** out)
{
    int dev = -1;
    if (!hip_ok(hipGetDevice(&dev))) return BLOAD_EHIP;
    if (dev < 0 || dev >= kMaxDevices) return BLOAD_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_of_device[dev]) {
        void* ptr = nullptr;
        if (!hip_ok(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch))) || !ptr) return BLOAD_EHIP;
        g_scratch_of_device[dev] = ptr;
    }
    *out = static_cast<uint8_t*>(g_scratch_of_device[dev]);
    return BLOAD_OK;
}

}  // namespace

extern "C" bload_status bload_pack_noalloc(const void* d_src, const int64_t* d_src_offsets,
                                           const int32_t* d_lengths, const int32_t* d_order,
                                           const int32_t* d_block_of_seq, const int32_t* d_offset_of_seq,
                                           const int32_t* d_block_first, int64_t n_seq,
                                           int64_t num_blocks, int32_t t_blk, int64_t frame_bytes,
                                           void* d_packed, int32_t* d_seq_id, int32_t* d_frame_idx,
                                           uint8_t* d_reset, uint8_t* d_valid, void* hip_stream)
{
    if (n_seq < 0 || num_blocks < 0 || t_blk < 1 || frame_bytes < 1) return BLOAD_EINVAL;
    if (n_seq > BLOAD_MAX_SEQ || num_blocks > n_seq) return n_seq > BLOAD_MAX_SEQ ? BLOAD_EOVERFLOW
                                                                                 : BLOAD_EINVAL;
    if (n_seq == 0 || num_blocks == 0) return BLOAD_OK;
    const bload_status st = pack_check_args(d_src, d_src_offsets, d_lengths, d_order, d_block_of_seq,
                                            d_offset_of_seq, d_block_first, n_seq, num_blocks, t_blk,
                                            frame_bytes, d_packed, d_seq_id, d_frame_idx, d_reset, d_valid);
    if (st != BLOAD_OK) return st;
    PackLayout l;
    if (!pack_layout(n_seq, num_blocks, t_blk, frame_bytes, aligned_to(d_src, 16), false, &l))
        return BLOAD_EOVERFLOW;
    // the fixed array holds this many runs and tiles, no more
    if (n_seq > BLOAD_PACK_NOALLOC_MAX_SEQ || l.tiles + l.table_tiles + 4 > BLOAD_PACK_NOALLOC_MAX_TILES)
        return BLOAD_EOVERFLOW;
    l.first_off = kStaticRunBytes;
    l.table_off = l.first_off + round_up((size_t)l.tiles * sizeof(int32_t), 16);
    uint8_t* ws = nullptr;
    const bload_status got = static_scratch(&ws);
    if (got != BLOAD_OK) return got;
    return pack_enqueue(l, d_src, d_src_offsets, d_lengths, d_order, d_block_of_seq, d_offset_of_seq,
                        d_block_first, n_seq, num_blocks, t_blk, frame_bytes, d_packed, d_seq_id,
                        d_frame_idx, d_reset, d_valid, ws, static_cast<hipStream_t>(hip_stream));
}

extern "C" bload_status bload_pack_check(const int64_t* d_src_offsets, const int32_t* d_lengths,
                                         const int32_t* d_order, const int32_t* d_block_of_seq,
                                         const int32_t* d_offset_of_seq, const int32_t* d_block_first,
                                         int64_t n_seq, int64_t num_blocks, int32_t t_blk,
                                         int64_t total_frames, int64_t* h_first_bad, void* d_workspace,
                                         size_t workspace_bytes, void* hip_stream)
{
    if (h_first_bad) *h_first_bad = -1;
    if (n_seq < 0 || num_blocks < 0 || t_blk < 1 || total_frames < 0) return BLOAD_EINVAL;
    if (n_seq > BLOAD_MAX_SEQ) return BLOAD_EOVERFLOW;
    if (num_blocks > n_seq) return BLOAD_EINVAL;
    if (n_seq == 0 || num_blocks == 0) return BLOAD_OK;
    if (!d_src_offsets || !d_lengths || !d_order || !d_block_of_seq || !d_offset_of_seq ||
        !d_block_first || !d_workspace)
        return BLOAD_EINVAL;
    if (!aligned_to(d_src_offsets, 8) || !aligned_to(d_lengths, 4) || !aligned_to(d_order, 4) ||
        !aligned_to(d_block_of_seq, 4) || !aligned_to(d_offset_of_seq, 4) ||
        !aligned_to(d_block_first, 4) || !aligned_to(d_workspace, 16))
        return BLOAD_EALIGN;
    if (workspace_bytes < 16) return BLOAD_EWORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    unsigned long long* first_bad = static_cast<unsigned long long*>(d_workspace);
    hipLaunchKernelGGL(pack_check_clear_kernel, dim3(1), dim3(1), 0, stream, first_bad);
    hipLaunchKernelGGL(pack_check_kernel, dim3((uint32_t)ceil_div(n_seq, kThreads)), dim3(kThreads), 0,
                       stream, d_src_offsets, d_lengths, d_order, d_block_of_seq, d_offset_of_seq,
                       d_block_first, (int32_t)n_seq, (int32_t)num_blocks, t_blk, total_frames, first_bad);
    if (launch_status() != BLOAD_OK) return BLOAD_EHIP;
    unsigned long long host = 0;
    if (!hip_ok(hipMemcpyAsync(&host, first_bad, sizeof(host), hipMemcpyDeviceToHost, stream)))
        return BLOAD_EHIP;
    if (!hip_ok(hipStreamSynchronize(stream))) return BLOAD_EHIP;
    if (host == ~0ull) return BLOAD_OK;
    if (h_first_bad) *h_first_bad = (int64_t)host;
    return BLOAD_EINVAL;
}
