// bload_segment_reduce: per-sequence sum / mean over the packed blocks, using
// only the packed tensor and the per-slot start table (BLoad, Methods section:
// the table of starting indices lets a consumer that carries state from frame
// to frame drop it where a new sequence begins).
//
// A segment is a maximal run of valid slots inside one block that begins at a
// start flag, at the block's first slot or behind a padding slot, and contains
// no other start flag.
// Time is cut into chunks; every chunk reduces the pieces of segments that lie
// in it.  A piece that is a whole segment goes straight to the output.  A
// piece cut by a chunk border goes to a partial buffer: "head" partial = the
// piece that continues a segment begun in an earlier chunk, "tail" partial =
// the piece that begins a segment continued in the next chunk.  A second
// small kernel adds tail + following heads in time order.  Fixed chunking and
// fixed order make the float32 result bit-reproducible.
//
// Two layouts of the work:
//   wide   (a frame is >= 64 bytes): lanes across the features of a frame, each
//          row of lanes (at most one wave) walks one chunk of time serially
//          with several loads in flight, restarting its accumulators at every
//          start flag.
//   narrow (small frames, e.g. one token): lanes across time, 16 consecutive
//          slots per lane, segmented scan over the workgroup with the segment
//          breaks as heads and a carry between lanes and waves.
#include "bload_common.hpp"

#include <hip/hip_fp16.h>
#include <limits.h>

#include <algorithm>

namespace bload {

constexpr int kHeadNone = 0, kHeadClosed = 1, kHeadThrough = 2;

struct ChunkDesc {
    int32_t head_state;   // kHead*: is there a piece continuing an earlier segment, and does
                          // it run through the whole chunk into the next one
    int32_t cnt_head;     // frames in that piece
    int32_t cnt_tail;     // frames in the piece that continues into the next chunk, 0 if none
    int32_t seq_tail;     // sequence id of that piece
};

struct ReduceArgs {
    const uint8_t* packed;
    const int32_t* seq_id;
    const uint8_t* reset;
    const uint8_t* valid;
    int64_t num_blocks;
    int64_t total_slots;
    int64_t total_chunks;
    int32_t t_blk;
    int32_t feat_dim;
    int32_t n_seq;
    int32_t mean;            // 1: divide by the frame count
    // narrow: a block is cut into `n_chunks` tiles (t_blk >= the tile), or a tile holds
    // `blocks_per_tile` whole blocks (t_blk < the tile); magic_t_blk = min(ceil(2^32 / t_blk),
    // 2^32 - 1) then divides positions inside a tile by t_blk (to within one, fixed up)
    int32_t blocks_per_tile;
    uint32_t magic_t_blk;
    void* out;               // [n_seq, feat_dim] float or int64
    // chunking
    int32_t chunk;           // slots per chunk
    int32_t n_chunks;        // wide: chunks per block
    int32_t row_lanes_log2;  // wide: lanes per row = 1 << this
    int32_t n_vec;           // wide: lanes needed to cover one frame
    int32_t feat_tiles;      // wide: workgroups side by side over one frame
    // partial buffers (null when no chunk border can cut a segment)
    ChunkDesc* desc;         // [total_chunks]
    void* head_part;         // [total_chunks, feat_dim] accumulators
    void* tail_part;         // [total_chunks, feat_dim]
};

// ---- element access -----------------------------------------------------------

template <typename ElemT> struct Elem;
template <> struct Elem<uint8_t> {
    typedef float Acc;
    // a piece of a chunk holds fewer than 2^15 frames of at most 255: every float sum of
    // them is a whole number below 2^24, i.e. exact, and needs no compensation
    static constexpr bool kCompensate = false;
    __device__ static float get(uint8_t v) { return (float)v; }
};
struct half_bits { uint16_t bits; };           // IEEE binary16 storage
template <> struct Elem<half_bits> {
    typedef float Acc;
    static constexpr bool kCompensate = true;
    __device__ static float get(half_bits v) { return __half2float(__ushort_as_half(v.bits)); }
};
template <> struct Elem<float> {
    typedef float Acc;
    static constexpr bool kCompensate = true;
    __device__ static float get(float v) { return v; }
};
template <> struct Elem<int32_t> {
    typedef long long Acc;
    static constexpr bool kCompensate = false;
    __device__ static long long get(int32_t v) { return (long long)v; }
};

// VEC elements of one lane: a 16-byte vector (VEC = 16 / sizeof(ElemT)) or one element.
template <typename ElemT, int VEC>
struct LaneData {
    union { vec16 v; ElemT e[VEC > 1 ? VEC : 1]; } u;
    __device__ __forceinline__ void load(const uint8_t* p)
    {
        if (VEC > 1) u.v = load_stream(reinterpret_cast<const vec16*>(p));
        else u.e[0] = *reinterpret_cast<const ElemT*>(p);
    }
};

template <typename Acc> struct OutOf;
template <> struct OutOf<float> { typedef float T; };
template <> struct OutOf<long long> { typedef long long T; };

// A running sum that many terms are added to, one after the other.  Integers are
// exact.  A float sum (COMPENSATED) carries the rounding error of every addition
// along (Kahan's compensated summation), so that its error stays at about two
// units in the last place of the sum of the |terms| however many there are,
// instead of growing with their number.  Once the sum has left the finite range
// the compensation is dropped, so that infinities add up as in plain arithmetic.
template <typename Acc, bool COMPENSATED> struct Running {
    Acc sum;
    __device__ __forceinline__ void clear() { sum = 0; }
    __device__ __forceinline__ void add(Acc term) { sum += term; }
};
template <> struct Running<float, true> {
    float sum, lost;
    __device__ __forceinline__ void clear() { sum = 0.0f; lost = 0.0f; }
    __device__ __forceinline__ void add(float term)
    {
        const float y = term - lost;
        const float t = sum + y;
        const float l = (t - sum) - y;
        lost = __builtin_isfinite(t) ? l : 0.0f;
        sum = t;
    }
};

template <typename Acc>
__device__ __forceinline__ Acc finish(Acc sum, int32_t cnt, int mean)
{
    return sum;
}
template <>
__device__ __forceinline__ float finish<float>(float sum, int32_t cnt, int mean)
{
    return mean ? sum / (float)cnt : sum;
}

// ------------------------------------------------------------------- wide

constexpr int kWideUnroll = 8;
constexpr int kWideFlagBytes = 32768;      // LDS budget for the staged flags: also the longest chunk
static_assert((int64_t)kWideFlagBytes * 255 < ((int64_t)1 << 24), "uint8 pieces must sum exactly in float");

// First slot s in [t, len) whose staged flags say "valid" (WANT_VALID) or "not a
// plain continuation: padding or a start flag" (!WANT_VALID); len if none.  The
// lanes of a row (a whole wave, or an aligned part of one) test one slot
// each per step and vote; every lane of the row gets the same answer.  WAVE_ROW:
// the row is the whole wave, and everything here but the tested slot is wave-uniform.
template <bool WANT_VALID, bool WAVE_ROW>
__device__ __forceinline__ int32_t next_slot(const uint8_t* flags, int32_t t, int32_t len,
                                             int row_lanes_log2)
{
    const int width = WAVE_ROW ? kWave : (1 << row_lanes_log2);
    const int lane = lane_id();
    const int base = WAVE_ROW ? 0 : lane & ~(width - 1);
    const uint64_t row_mask = WAVE_ROW ? ~0ull : ((1ull << width) - 1ull) << base;
    for (; t < len; t += width) {
        const int32_t s = t + (lane - base);
        bool hit = false;
        if (s < len) {
            const uint8_t f = flags[s];
            hit = WANT_VALID ? (f & 1) != 0 : (f & 3) != 1;
        }
        const uint64_t vote = __ballot(hit) & row_mask;
        if (vote) return t + (__ffsll((unsigned long long)vote) - 1 - base);
    }
    return len;
}

// Elements of LDS scratch per lane for the transposed stores: the lane's VEC values plus
// padding against bank conflicts (a multiple of 4 for floats, which move 16 bytes at a time).
template <typename Acc, int VEC>
__host__ __device__ constexpr int kScratchStride() { return sizeof(Acc) == 4 ? VEC + 4 : VEC + 1; }

// Store the VEC accumulators of every lane of a row to dst[feat0 ...].  A lane
// holds VEC consecutive features, so storing straight from the registers
// writes 16-byte pieces 16 * VEC bytes apart; when a whole wave belongs to one
// row the values go through the wave's LDS scratch instead and leave as runs
// of 64 consecutive elements.  `scratch` is null for rows narrower than a wave.
template <typename Acc, int VEC>
__device__ __forceinline__ void store_row(Acc* dst_row, int64_t feat0, const Acc (&v)[VEC],
                                          bool lane_stores, Acc* scratch, int64_t wave_feat0,
                                          int32_t feat_dim)
{
    if (VEC == 1 || scratch == nullptr) {
        if (lane_stores) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) dst_row[feat0 + k] = v[k];
        }
        return;
    }
    const int lane = lane_id();
    constexpr int S = kScratchStride<Acc, VEC>();
    // element e of the wave's 64 * VEC span lives in lane e / VEC, register e % VEC
    if constexpr (sizeof(Acc) == 4 && VEC % 4 == 0) {
      if ((reinterpret_cast<uintptr_t>(dst_row) & 15) == 0) {
        // four floats at a time: VEC / 4 stores of 1 KiB per wave
        typedef float float4v __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int k = 0; k < VEC; k += 4) {
            const float4v q = {(float)v[k], (float)v[k + 1], (float)v[k + 2], (float)v[k + 3]};
            *reinterpret_cast<float4v*>(reinterpret_cast<float*>(scratch) + lane * S + k) = q;
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < VEC / 4; ++j) {
            const int e = j * kWave * 4 + lane * 4;
            const float4v q = *reinterpret_cast<const float4v*>(reinterpret_cast<const float*>(scratch) +
                                                                (e / VEC) * S + (e % VEC));
            if (wave_feat0 + e < feat_dim)
                *reinterpret_cast<float4v*>(reinterpret_cast<float*>(dst_row) + wave_feat0 + e) = q;
        }
        __builtin_amdgcn_wave_barrier();
        return;
      }
    }
#pragma unroll
    for (int k = 0; k < VEC; ++k) scratch[lane * S + k] = v[k];
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
        const int e = j * kWave + lane;
        const Acc x = scratch[(e / VEC) * S + (e % VEC)];
        if (wave_feat0 + e < feat_dim) dst_row[wave_feat0 + e] = x;
    }
    __builtin_amdgcn_wave_barrier();
}

// WAVE_ROW: a row of lanes is exactly one wave.  Its chunk, the pieces found in it and the
// addresses of the frames are then the same for all lanes of the wave, and saying so (the row
// index goes through readfirstlane) lets the compiler keep them in scalar registers and address
// the loads as scalar base + lane offset.
template <typename ElemT, int VEC, bool WAVE_ROW>
__global__ __launch_bounds__(kThreads) void reduce_wide_kernel(ReduceArgs a)
{
    typedef typename Elem<ElemT>::Acc Acc;
    extern __shared__ uint8_t s_flags[];   // rows x (chunk + 2): bit0 valid, bit1 reset
    const int tid = (int)threadIdx.x;
    const int C = a.chunk, stride = C + 2;
    const int rows = kThreads >> a.row_lanes_log2;
    // consecutive workgroups take the lane-slices of one frame range, so that
    // workgroups running side by side read neighbouring memory
    const int feat_tile = (int)(blockIdx.x % (uint32_t)a.feat_tiles);
    const int64_t q_base = (int64_t)(blockIdx.x / (uint32_t)a.feat_tiles) * rows;
    const int64_t T = a.t_blk;

    // stage the flags of this workgroup's chunks, plus the slot before and the slot
    // after each chunk (0 outside the block): row r holds slots t0-1 .. t0+len
    for (int r = 0; r < rows; ++r) {
        const int64_t q = q_base + r;
        if (q >= a.total_chunks) break;
        const int64_t b = q / a.n_chunks;
        const int32_t t0 = (int32_t)(q - b * a.n_chunks) * C;
        const int32_t len = min(C, a.t_blk - t0);
        const int64_t g = b * T + t0;
        for (int t = tid - 1; t <= len; t += kThreads) {
            uint8_t f = 0;
            if (t0 + t >= 0 && t0 + t < a.t_blk)
                f = (uint8_t)((a.valid[g + t] ? 1 : 0) | (a.reset[g + t] ? 2 : 0));
            s_flags[r * stride + 1 + t] = f;
        }
    }
    __syncthreads();

    const int row = WAVE_ROW ? __builtin_amdgcn_readfirstlane(tid >> 6) : tid >> a.row_lanes_log2;
    const int col = WAVE_ROW ? lane_id() : tid & ((1 << a.row_lanes_log2) - 1);
    const int64_t q = q_base + row;
    if (q >= a.total_chunks) return;
    // which lane-slice of the frame; the surplus lanes of a row stay alive (they
    // take part in the votes of next_slot), read what the last lane reads, and store nothing
    const int fv_raw = feat_tile * (1 << a.row_lanes_log2) + col;
    const bool lane_stores = fv_raw < a.n_vec;
    const int fv = lane_stores ? fv_raw : a.n_vec - 1;

    const int64_t b = q / a.n_chunks;
    const int32_t t0 = (int32_t)(q - b * a.n_chunks) * C;
    const int32_t len = min(C, a.t_blk - t0);
    const int64_t g = b * T + t0;
    const uint8_t* flags = s_flags + row * stride + 1;      // flags[-1] = the slot before the chunk
    const int64_t frame_bytes = (int64_t)a.feat_dim * (int64_t)sizeof(ElemT);
    const uint8_t* chunk_src = a.packed + g * frame_bytes;                 // the chunk's first frame
    const uint32_t lane_off = (uint32_t)fv * VEC * (uint32_t)sizeof(ElemT);  // the lane's place in a frame
    const int64_t feat0 = (int64_t)fv * VEC;
    const bool writes_desc = (col == 0 && feat_tile == 0 && a.desc != nullptr);
    typedef typename OutOf<Acc>::T Out;
    Out* out = static_cast<Out*>(a.out);
    Acc* head_part = static_cast<Acc*>(a.head_part);
    Acc* tail_part = static_cast<Acc*>(a.tail_part);

    // per-wave LDS scratch for the transposed stores (behind the flags), when a
    // wave lies inside one row
    Acc* scratch = nullptr;
    const int64_t wave_feat0 = (int64_t)(fv_raw - lane_id()) * VEC;   // first feature of the wave
    if (VEC > 1 && WAVE_ROW) {
        const size_t flag_bytes = ((size_t)rows * stride + 15) & ~(size_t)15;
        scratch = reinterpret_cast<Acc*>(s_flags + flag_bytes) + (size_t)wave_id() * kWave * kScratchStride<Acc, VEC>();
    }

    Running<Acc, Elem<ElemT>::kCompensate> run[VEC];
    Acc acc[VEC];
    ChunkDesc desc{kHeadNone, 0, 0, -1};

    // The chunk is a sequence of pieces: maximal runs of valid slots that hold
    // no start flag after their first slot.  Find a piece [t, e) from the
    // staged flags, sum it with unconditional loads, hand the sum on.  The
    // frames of a piece are added eight at a time as a balanced tree, and the
    // sums of the eights go into a compensated running sum: the float32 result
    // is within a few units in the last place of sum |x| at any piece length.
    int32_t t = 0;
    for (;;) {
        t = next_slot<true, WAVE_ROW>(flags, t, len, a.row_lanes_log2);    // next valid slot
        if (t >= len) break;
        // a segment starts at a start flag, at the block's first slot, or behind padding;
        // a valid first slot of the chunk that does none of these continues the segment
        // of the chunk before
        const bool head_open = t == 0 && !(flags[0] & 2) && (flags[-1] & 1);
        const int32_t e = next_slot<false, WAVE_ROW>(flags, t + 1, len, a.row_lanes_log2);  // padding or a start
#pragma unroll
        for (int k = 0; k < VEC; ++k) run[k].clear();
        const uint8_t* p = chunk_src + (int64_t)t * frame_bytes;          // frame of slot s, lane 0
        int32_t s = t;
        static_assert(kWideUnroll == 8, "the tree below adds eight frames");
        for (; s + kWideUnroll <= e; s += kWideUnroll) {
            LaneData<ElemT, VEC> x[kWideUnroll];
#pragma unroll
            for (int u = 0; u < kWideUnroll; ++u) x[u].load(p + (int64_t)u * frame_bytes + lane_off);
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                Acc v[kWideUnroll];
#pragma unroll
                for (int u = 0; u < kWideUnroll; ++u) v[u] = Elem<ElemT>::get(x[u].u.e[k]);
                run[k].add(((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7])));
            }
            p += (int64_t)kWideUnroll * frame_bytes;
        }
        if (s < e) {
            // the last, partial batch: all loads are issued at once as well (those
            // past the piece re-read its last slot and count as 0)
            const int32_t left = e - s;
            LaneData<ElemT, VEC> x[kWideUnroll];
#pragma unroll
            for (int u = 0; u < kWideUnroll; ++u)
                x[u].load(p + (int64_t)min(u, left - 1) * frame_bytes + lane_off);
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                Acc v[kWideUnroll];
#pragma unroll
                for (int u = 0; u < kWideUnroll; ++u) v[u] = u < left ? Elem<ElemT>::get(x[u].u.e[k]) : (Acc)0;
                run[k].add(((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7])));
            }
        }
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc[k] = run[k].sum;
        const int32_t cnt = e - t;
        // the segment ends here unless the piece runs to the chunk's end and the
        // slot after the chunk (flags[len], 0 past the block) continues it
        const bool closed = e < len || (flags[len] & 3) != 1;
        if (head_open) {
            if (head_part) store_row<Acc, VEC>(head_part + q * a.feat_dim, feat0, acc, lane_stores, scratch, wave_feat0, a.feat_dim);
            desc.head_state = closed ? kHeadClosed : kHeadThrough;
            desc.cnt_head = cnt;
        } else {
            const int32_t seq = a.seq_id[g + t];
            if (closed) {
                if ((uint32_t)seq < (uint32_t)a.n_seq) {
#pragma unroll
                    for (int k = 0; k < VEC; ++k) acc[k] = finish<Acc>(acc[k], cnt, a.mean);
                    store_row<Acc, VEC>(out + (int64_t)seq * a.feat_dim, feat0, acc, lane_stores, scratch, wave_feat0, a.feat_dim);
                }
            } else {
                if (tail_part) store_row<Acc, VEC>(tail_part + q * a.feat_dim, feat0, acc, lane_stores, scratch, wave_feat0, a.feat_dim);
                desc.cnt_tail = cnt;
                desc.seq_tail = seq;
            }
        }
        t = e;
    }
    if (writes_desc) a.desc[q] = desc;
}

// ----------------------------------------------------------------- narrow
//
// Lanes across time: a workgroup takes 4096 consecutive slots (a "tile": a piece
// of one block, or several whole blocks), a lane 16 consecutive slots.  From the
// flags every lane builds two 16-bit masks: valid, and "break" (a slot that cannot
// continue the segment of the slot before it: padding, a start flag, a block's
// first slot, or a slot that follows padding).  Sums are a segmented scan with the
// breaks as heads: a lane contributes the sum of its slots from its last break
// on (`tail`: all its slots if it has none); the scan runs across the wave without
// LDS (DPP) and across the four waves through LDS, and gives every lane the sum of
// the segment that is open in front of it.  A lane keeps one more sum, of its
// slots in front of its first break (`head`), and not its 16 elements: a piece
// that ends in the lane is carry + head, or tail; only a piece between two breaks
// of one lane -- a segment of fewer than 16 slots -- is read again.  Frame counts
// need no scan: a segment's frames are consecutive, so its count is (end position
// - position of its break + 1).  Integer sums are exact, float sums add only the
// segment's own terms (no cancellation against neighbouring segments).

constexpr int kSlotsPerLane = 16;
constexpr int kNarrowTile = kThreads * kSlotsPerLane;      // 4096 slots per workgroup

// Running state of a segmented sum: `any` = a break was seen.
template <typename Acc>
struct SegState { Acc sum; uint32_t any; };

template <typename Acc>
struct SegCombine {
    __device__ __forceinline__ SegState<Acc> operator()(SegState<Acc> left, SegState<Acc> right) const
    {
        SegState<Acc> r;
        r.sum = right.any ? right.sum : left.sum + right.sum;
        r.any = left.any | right.any;
        return r;
    }
};

template <typename Acc>
struct PlainSum {
    __device__ __forceinline__ Acc operator()(Acc left, Acc right) const { return left + right; }
};
template <typename Acc>
struct PlainMove {
    template <int CTRL, int ROW_MASK>
    __device__ __forceinline__ Acc at(Acc x) const { return dpp_move<CTRL, ROW_MASK>(x, (Acc)0); }
};

template <typename Acc>
struct SegMove {
    template <int CTRL, int ROW_MASK>
    __device__ __forceinline__ SegState<Acc> at(SegState<Acc> s) const
    {
        return SegState<Acc>{dpp_move<CTRL, ROW_MASK>(s.sum, (Acc)0), dpp_move<CTRL, ROW_MASK>(s.any, 0u)};
    }
};

// Bit j of the result: byte j of the 16 flag bytes is non-zero.
__device__ __forceinline__ uint32_t nonzero_bytes16(vec16 w)
{
    // 0x80 in every non-zero byte; a dot product with byte weights 1, 2, 4, 8 (16 ... 128 for the
    // next four bytes) then puts one bit per byte side by side, seven places up
    uint32_t t[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) t[k] = (((w[k] & 0x7f7f7f7fu) + 0x7f7f7f7fu) | w[k]) & 0x80808080u;
    const uint32_t lo = __builtin_amdgcn_udot4(t[1], 0x80402010u, __builtin_amdgcn_udot4(t[0], 0x08040201u, 0u, false), false);
    const uint32_t hi = __builtin_amdgcn_udot4(t[3], 0x80402010u, __builtin_amdgcn_udot4(t[2], 0x08040201u, 0u, false), false);
    return (lo >> 7) | ((hi >> 7) << 8);
}

typedef vec16 __attribute__((aligned(1))) vec16_any;      // a 16-byte vector at any address

// Where a workgroup's tile lies.  Tiles never straddle a block: a tile is a piece of one block
// (blocks of at least a tile's length) or a whole number of blocks.
struct NarrowTile {
    int64_t g0;            // first slot
    int32_t n;             // slots in the tile
    int32_t rem0;          // position of the tile's first slot inside its block
};

__device__ __forceinline__ NarrowTile narrow_tile(const ReduceArgs& a, int64_t q)
{
    NarrowTile t;
    if (a.t_blk >= kNarrowTile) {
        const int64_t b = a.n_chunks == 1 ? q : (int64_t)((uint32_t)q / (uint32_t)a.n_chunks);
        const int32_t c = (int32_t)(q - b * a.n_chunks);
        t.rem0 = c * kNarrowTile;
        t.g0 = b * (int64_t)a.t_blk + t.rem0;
        t.n = min(kNarrowTile, a.t_blk - t.rem0);
    } else {
        const int64_t b0 = q * a.blocks_per_tile;
        t.rem0 = 0;
        t.g0 = b0 * (int64_t)a.t_blk;
        t.n = (int32_t)min((int64_t)a.blocks_per_tile, a.num_blocks - b0) * a.t_blk;
    }
    return t;
}

// What a lane knows about its 16 slots after reading the flags.
struct LaneFlags {
    uint32_t vmask;        // bit j: slot j is valid
    uint32_t bmask;        // bit j: slot j is a break
    uint32_t ends;         // bit j: a segment ends at slot j
    int32_t j_last;        // index of the tile's last slot in this lane (may lie outside 0..15)
    bool tail_open;        // the tile's last slot is here and its segment goes on into the next tile
};

// The flag bytes of a lane as they come from memory, and what the whole wave is, as far as a
// look at whole words can tell.
struct LaneFlagBytes {
    vec16 valid, reset;    // zero where the lane has not all its 16 slots in the tile
    bool wave_blank;       // the wave holds nothing but padding
    bool wave_plain;       // the wave holds nothing but valid slots without a start flag
};

__device__ __forceinline__ LaneFlagBytes narrow_flag_bytes(const ReduceArgs& a, const NarrowTile& tile)
{
    constexpr int SPL = kSlotsPerLane;
    static_assert(SPL == 16, "the flags of a lane are one 16-byte vector per plane");
    const int pos0 = (int)threadIdx.x * SPL;
    const int32_t left = tile.n - pos0;
    LaneFlagBytes b;
    b.valid = vec16{0u, 0u, 0u, 0u};
    b.reset = vec16{0u, 0u, 0u, 0u};
    if (left >= SPL) {
        b.valid = __builtin_nontemporal_load(reinterpret_cast<const vec16_any*>(a.valid + tile.g0 + pos0));
        b.reset = __builtin_nontemporal_load(reinterpret_cast<const vec16_any*>(a.reset + tile.g0 + pos0));
    }
    // Two kinds of waves are common in packed blocks and need no byte-by-byte look at their
    // flags: nothing but padding (block tails), and nothing but valid slots without a start flag
    // (the inside of long sequences).  Both tests are wave-uniform.
    const uint32_t v_any = b.valid[0] | b.valid[1] | b.valid[2] | b.valid[3];
    const uint32_t v_all = b.valid[0] & b.valid[1] & b.valid[2] & b.valid[3];
    const uint32_t r_any = b.reset[0] | b.reset[1] | b.reset[2] | b.reset[3];
    const bool lane_blank = left >= SPL ? v_any == 0u : left <= 0;
    // (a non-zero byte in the AND of the four words means four non-zero bytes)
    const bool lane_plain = left >= SPL && r_any == 0u &&
                            ((((v_all & 0x7f7f7f7fu) + 0x7f7f7f7fu) | v_all) & 0x80808080u) == 0x80808080u;
    b.wave_blank = __ballot(lane_blank) == ~0ull;
    b.wave_plain = __ballot(lane_plain) == ~0ull;
    return b;
}

// Derives the masks of the lane's slots from its flag bytes and those of its neighbours.
// Called by every thread of the workgroup (the lanes of a wave exchange their border slots).
__device__ __forceinline__ LaneFlags narrow_lane_flags(const ReduceArgs& a, const NarrowTile& tile,
                                                       const LaneFlagBytes& bytes)
{
    constexpr int SPL = kSlotsPerLane;
    constexpr uint32_t ALL = (1u << SPL) - 1u;
    const int tid = (int)threadIdx.x;
    const int lane = lane_id();
    const uint32_t T = (uint32_t)a.t_blk;
    const int pos0 = tid * SPL;
    const int32_t left = tile.n - pos0;                  // slots from this lane's first one to the tile's end
    const int64_t s0 = tile.g0 + pos0;
    LaneFlags r;

    // position of the lane's first slot inside its block, and of the slot behind its last one
    uint32_t rem0 = (uint32_t)tile.rem0 + (uint32_t)pos0;
    if (T < (uint32_t)kNarrowTile) {
        rem0 -= __umulhi((uint32_t)pos0, a.magic_t_blk) * T;        // pos0 mod T, possibly one T too many
        if (rem0 >= T) rem0 -= T;
    }
    uint32_t rem_next = rem0 + (uint32_t)SPL;
    while (rem_next >= T) rem_next -= T;                 // at most once unless t_blk < 16

    // the slots in front of and behind the lanes of this wave, where they belong to the same block
    uint8_t before_valid = 0, after_valid = 0, after_reset = 0;
    if (lane == 0 && rem0 != 0 && left > 0) before_valid = a.valid[s0 - 1];
    if (lane == kWave - 1 && rem_next != 0 && left >= SPL) { after_valid = a.valid[s0 + SPL]; after_reset = a.reset[s0 + SPL]; }

    uint32_t vmask = 0, rmask = 0;
    if (bytes.wave_blank) {
        // vmask = rmask = 0
    } else if (bytes.wave_plain) {
        vmask = ALL;
    } else if (left >= SPL) {
        vmask = nonzero_bytes16(bytes.valid);
        rmask = nonzero_bytes16(bytes.reset);
    } else if (left > 0) {
        // the tile ends inside this lane: slot by slot (those past the end re-read its last slot)
#pragma unroll
        for (int j = 0; j < SPL; ++j) {
            vmask |= (uint32_t)(a.valid[s0 + min(j, left - 1)] != 0) << j;
            rmask |= (uint32_t)(a.reset[s0 + min(j, left - 1)] != 0) << j;
        }
        vmask &= (1u << left) - 1u;
        rmask &= (1u << left) - 1u;
    }
    // first slots of blocks among the lane's slots: `gap` = slots to the next block start
    uint32_t smask = 0;
    for (uint32_t gap = rem0 == 0 ? 0u : T - rem0; gap < (uint32_t)SPL; gap += T) smask |= 1u << gap;
    // validity of the slot before this lane's first one
    uint32_t prev_valid = dpp_move<kDppWaveShr1>((vmask >> (SPL - 1)) & 1u, 0u);
    if (lane == 0) prev_valid = (uint32_t)(before_valid != 0);
    const uint32_t after_pad = ~((vmask << 1) | prev_valid);          // bit j: slot j-1 is not valid
    const uint32_t bmask = (~vmask | rmask | smask | after_pad) & ALL;
    // is the slot after this lane's last one a break
    uint32_t next_first = dpp_move<kDppWaveShl1>(bmask & 1u, 0u);
    if (lane == kWave - 1) {
        next_first = 1u;
        if (rem_next != 0 && left >= SPL)
            next_first = (!after_valid || after_reset || !((vmask >> (SPL - 1)) & 1u)) ? 1u : 0u;
    }
    const uint32_t next_brk = (bmask >> 1) | (next_first << (SPL - 1));
    r.vmask = vmask;
    r.bmask = bmask;
    r.ends = vmask & next_brk;
    r.j_last = left - 1;
    r.tail_open = r.j_last >= 0 && r.j_last < SPL && ((vmask >> r.j_last) & 1u) &&
                  !((next_brk >> r.j_last) & 1u);
    return r;
}

// LDS staging of the payload of one workgroup: the NV 16-byte vectors of a lane lie together,
// vector k of lane l in place k ^ (l / (16 / NV)) of the lane's NV, so that the 16 lanes which
// one pass of a 16-byte LDS access serves touch every bank once, both when a lane writes vector
// l of a row and when it reads its own vectors.
template <typename ElemT>
struct NarrowStage {
    static constexpr int NV = kSlotsPerLane * (int)sizeof(ElemT) / 16;     // vectors per lane
    static_assert(NV == 1 || NV == 2 || NV == 4, "the bank swizzle below is written for 1, 2 or 4 vectors");
    static constexpr int kVectors = NV > 1 ? kThreads * NV : 1;
    // place of vector k of lane l (l counted within the wave) in the wave's part of the stage
    __device__ static __forceinline__ int at(int l, int k) { return l * NV + (k ^ ((l / (16 / NV)) & (NV - 1))); }
};

// The payload of a wave whose 1024 elements are contiguous (a frame is one element, every lane
// has all its slots): read as whole 1 KiB rows, lane l taking vector l of each row, because 64
// lanes that each read their own 64 bytes would touch four times as many cache lines per load.
// `issue` only starts the loads (so that the work on the flags runs while they are in flight),
// `finish` hands every vector to the lane it belongs to, through LDS.
template <typename ElemT>
struct NarrowRows {
    static constexpr int NV = NarrowStage<ElemT>::NV;
    vec16 v[NV > 0 ? NV : 1];

    __device__ __forceinline__ void issue(const ReduceArgs& a, int64_t wave_s0)
    {
        const vec16_any* row = reinterpret_cast<const vec16_any*>(a.packed + wave_s0 * (int64_t)sizeof(ElemT));
#pragma unroll
        for (int k = 0; k < NV; ++k) v[k] = __builtin_nontemporal_load(row + k * kWave + lane_id());
    }
    __device__ __forceinline__ void finish(vec16* stage, ElemT (&raw)[kSlotsPerLane])
    {
        const int lane = lane_id();
        vec16* mine = stage + (int)(threadIdx.x - lane) * NV;                // the wave's part
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int row_at = k * kWave + lane;             // vector `row_at` of the wave belongs to lane row_at / NV
            mine[NarrowStage<ElemT>::at(row_at / NV, row_at % NV)] = v[k];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        union { vec16 q[NV > 0 ? NV : 1]; ElemT e[kSlotsPerLane]; } u;
#pragma unroll
        for (int k = 0; k < NV; ++k) u.q[k] = mine[NarrowStage<ElemT>::at(lane, k)];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < kSlotsPerLane; ++j) raw[j] = u.e[j];
    }
    // Element j of the lane once more, from the stage (which keeps the wave's rows until the
    // workgroup ends): for the few lanes that need single elements again.
    __device__ __forceinline__ static ElemT again(const vec16* stage, int j)
    {
        constexpr int EPV = 16 / (int)sizeof(ElemT);
        const int lane = lane_id();
        const vec16* mine = stage + (int)(threadIdx.x - lane) * NV;
        return reinterpret_cast<const ElemT*>(mine + NarrowStage<ElemT>::at(lane, j / EPV))[j % EPV];
    }
};

// The lane's 16 elements of feature d where they do not come as rows; only those of valid slots
// mean anything.  ONE: a frame is one element, so they are contiguous and come as 16-byte
// vectors.  Otherwise one load per slot, all issued together.  `left` = slots from the lane's
// first one to the tile's end.
template <typename ElemT, bool ONE>
__device__ __forceinline__ void narrow_load(const ReduceArgs& a, int64_t s0, int32_t left, int d,
                                            ElemT (&raw)[kSlotsPerLane])
{
    constexpr int SPL = kSlotsPerLane;
    constexpr int NV = NarrowStage<ElemT>::NV;
    if (ONE && left >= SPL) {
        union { vec16 v[NV > 0 ? NV : 1]; ElemT e[SPL]; } u;
        const vec16_any* from = reinterpret_cast<const vec16_any*>(a.packed + s0 * (int64_t)sizeof(ElemT));
#pragma unroll
        for (int k = 0; k < NV; ++k) u.v[k] = __builtin_nontemporal_load(from + k);
#pragma unroll
        for (int j = 0; j < SPL; ++j) raw[j] = u.e[j];
    } else if (left > 0) {
        // slots past the tile's end re-read its last slot (their valid bits are 0)
        const int64_t stride = (int64_t)(ONE ? 1 : a.feat_dim) * (int64_t)sizeof(ElemT);
        const uint8_t* from = a.packed + (s0 * (ONE ? 1 : a.feat_dim) + d) * (int64_t)sizeof(ElemT);
#pragma unroll
        for (int j = 0; j < SPL; ++j) raw[j] = *reinterpret_cast<const ElemT*>(from + min(j, left - 1) * stride);
    } else {
#pragma unroll
        for (int j = 0; j < SPL; ++j) raw[j] = ElemT{};
    }
}

// x where bit j of `mask` is set, 0 (of the accumulator's type) elsewhere
__device__ __forceinline__ float masked(float x, uint32_t mask, int j)
{
    return __int_as_float(__float_as_int(x) & (int32_t)__builtin_amdgcn_sbfe(mask, j, 1));
}
__device__ __forceinline__ long long masked(long long x, uint32_t mask, int j)
{
    return (long long)((int32_t)x & (int32_t)__builtin_amdgcn_sbfe(mask, j, 1));     // x holds an int32 here
}

// Hand one finished piece on: to the output row of its sequence, or to the
// partial buffers when the tile border cuts its segment.  `seq` is the sequence
// id at the first slot of the piece when the segment starts in this tile
// (`started`), as in the wide layout.
template <typename Acc>
__device__ __forceinline__ void narrow_emit(const ReduceArgs& a, int64_t q, int d, int32_t seq,
                                            bool is_end, bool started, Acc sum, int32_t cnt,
                                            ChunkDesc* s_desc)
{
    typedef typename OutOf<Acc>::T Out;
    const int D = a.feat_dim;
    if (is_end && started) {
        if ((uint32_t)seq < (uint32_t)a.n_seq)
            static_cast<Out*>(a.out)[(int64_t)seq * D + d] = finish<Acc>(sum, cnt, a.mean);
    } else if (!started) {
        // continues a segment of the previous tile; closed here or running through
        if (a.head_part) static_cast<Acc*>(a.head_part)[q * D + d] = sum;
        if (d == 0) {
            s_desc->head_state = is_end ? kHeadClosed : kHeadThrough;
            s_desc->cnt_head = cnt;
        }
    } else {
        if (a.tail_part) static_cast<Acc*>(a.tail_part)[q * D + d] = sum;
        if (d == 0) {
            s_desc->cnt_tail = cnt;
            s_desc->seq_tail = seq;
        }
    }
}

template <typename ElemT, bool ONE>
__global__ __launch_bounds__(kThreads) void reduce_narrow_kernel(ReduceArgs a)
{
    typedef typename Elem<ElemT>::Acc Acc;
    constexpr int NW = kThreads / kWave;
    constexpr int SPL = kSlotsPerLane;
    __shared__ Acc s_wave_sum[NW];                     // the wave's sum behind its last break (all of it if none)
    __shared__ uint32_t s_wave_any[NW];                // the wave holds a break
    __shared__ unsigned long long s_wave_breaks[NW];   // which lanes of the wave hold a break
    __shared__ int32_t s_last_break[kThreads];         // position of a lane's last break (lanes that have one)
    __shared__ int32_t s_break_seq[kThreads];          // and the sequence id found there
    __shared__ vec16 s_stage[ONE ? NarrowStage<ElemT>::kVectors : 1];
    __shared__ ChunkDesc s_desc;

    const int tid = (int)threadIdx.x;
    const int lane = lane_id(), wave = wave_id();
    const int64_t q = blockIdx.x;
    const NarrowTile tile = narrow_tile(a, q);
    const int64_t g0 = tile.g0;
    const int pos0 = tid * SPL;
    const int64_t s0 = g0 + pos0;
    if (tid == 0) s_desc = ChunkDesc{kHeadNone, 0, 0, -1};
    const LaneFlagBytes bytes = narrow_flag_bytes(a, tile);
    // a wave without a valid slot reads no payload; a wave that lies whole in the tile asks for
    // its rows now, before the flags are looked at
    const bool wave_valid = !bytes.wave_blank;
    const int32_t left = tile.n - pos0;
    const bool by_rows = ONE && NarrowStage<ElemT>::NV > 1 && left - (kWave - 1 - lane) * SPL >= SPL;
    NarrowRows<ElemT> rows;
    if (wave_valid && by_rows) rows.issue(a, s0 - lane * SPL);
    const LaneFlags f = narrow_lane_flags(a, tile, bytes);
    const uint32_t bmask = f.bmask;
    const unsigned long long wave_breaks = __ballot(bmask != 0);
    const int last_break = bmask ? 31 - __clz((int)bmask) : 0;
    const int first_break = bmask ? __ffs((int)bmask) - 1 : SPL;
    // the sequence that starts at the lane's last break: asked for now, so that the answer is
    // there when a lane further on (or this one) closes that segment
    int32_t own_seq = -1;
    if (bmask && ((f.vmask >> last_break) & 1u)) own_seq = a.seq_id[s0 + last_break];
    if (lane == 0) s_wave_breaks[wave] = wave_breaks;
    const uint32_t from_last_break = f.vmask & (~0u << last_break);   // the lane's part of the open segment
    const uint32_t to_first_break = f.vmask & ((1u << first_break) - 1u);   // its part of the segment it inherits
    const bool finishes = f.ends != 0 || f.tail_open;                 // a piece ends in this lane
    int32_t prev_start = -1;           // position of the last break in front of this lane, -1: none in the tile
    int32_t prev_seq = -1;             // and the sequence id found there

    const int n_feat = ONE ? 1 : a.feat_dim;
    for (int d = 0; d < n_feat; ++d) {
        SegState<Acc> scan, carry;
        Acc tail = 0;                  // the lane's slots from its last break on (all of them if it has none)
        Acc head = 0;                  // the lane's slots in front of its first break
        if (!wave_valid) {
            // nothing but padding: every slot is a break, nothing to add
            scan = SegState<Acc>{0, 1u};
            carry = SegState<Acc>{0, lane == 0 ? 0u : 1u};
        } else {
            ElemT raw[SPL];
            if (by_rows) rows.finish(s_stage, raw);
            else narrow_load<ElemT, ONE>(a, s0, left, d, raw);
            if (wave_breaks == 0) {
                // no break in the whole wave (so every slot is valid): plain sums
#pragma unroll
                for (int j = 0; j < SPL; ++j) tail += Elem<ElemT>::get(raw[j]);
                scan = SegState<Acc>{wave_scan(tail, PlainSum<Acc>(), PlainMove<Acc>()), 0u};
                carry = SegState<Acc>{dpp_move<kDppWaveShr1>(scan.sum, (Acc)0), 0u};
            } else {
#pragma unroll
                for (int j = 0; j < SPL; ++j) {
                    tail += masked((Acc)Elem<ElemT>::get(raw[j]), from_last_break, j);
                    head += masked((Acc)Elem<ElemT>::get(raw[j]), to_first_break, j);
                }
                scan = wave_scan(SegState<Acc>{tail, bmask != 0 ? 1u : 0u}, SegCombine<Acc>(), SegMove<Acc>());
                carry = SegMove<Acc>().template at<kDppWaveShr1, 0xF>(scan);      // the lanes before this one
            }
        }
        if (d > 0) __syncthreads();                  // the previous feature's wave sums are consumed
        if (lane == kWave - 1) { s_wave_sum[wave] = scan.sum; s_wave_any[wave] = scan.any; }
        if (d == 0 && bmask) { s_last_break[tid] = pos0 + last_break; s_break_seq[tid] = own_seq; }
        __syncthreads();
        if (!finishes) continue;

        // the segments that end in this lane, and the open tail of the tile
        SegState<Acc> before{0, 0};
        for (int w = 0; w < wave; ++w)
            before = SegCombine<Acc>()(before, SegState<Acc>{s_wave_sum[w], s_wave_any[w]});
        carry = SegCombine<Acc>()(before, carry);
        if (d == 0) {
            const unsigned long long lower = wave_breaks & ((1ull << lane) - 1ull);
            int holder = lower ? wave * kWave + 63 - __clzll((long long)lower) : -1;
            for (int w = wave - 1; w >= 0 && holder < 0; --w) {
                const unsigned long long b = s_wave_breaks[w];
                if (b) holder = w * kWave + 63 - __clzll((long long)b);
            }
            if (holder >= 0) { prev_start = s_last_break[holder]; prev_seq = s_break_seq[holder]; }
        }
        // One piece per end (usually one per lane).  The piece that closes what the lanes before
        // left open ends in front of the lane's first break: carry + head.  The piece that the
        // lane's last break opened ends at its last slot: tail (plus the carry if the lane has no
        // break at all).  A piece between two breaks of the lane is read again, slot by slot: from
        // the LDS stage where the wave's rows went through it (workload of 10^6 token sequences:
        // 1.24 -> 1.15 ms against reading them from memory), else from memory.
        uint32_t todo = f.ends | (f.tail_open ? 1u << f.j_last : 0u);
        while (todo) {
            const int j = 31 - __clz((int)todo);                          // last one first
            todo &= ~(1u << j);
            const uint32_t upto = bmask & ((2u << j) - 1u);               // breaks at or before j
            const int lb = upto ? 31 - __clz((int)upto) : -1;
            Acc sum;
            if (lb < 0) {
                sum = carry.sum + (bmask ? head : tail);
            } else if (lb == last_break) {
                sum = tail;
            } else {
                sum = 0;
                if (by_rows) {
                    for (int k = lb; k <= j; ++k) sum += Elem<ElemT>::get(NarrowRows<ElemT>::again(s_stage, k));
                } else {
                    const int64_t stride = (int64_t)(ONE ? 1 : a.feat_dim) * (int64_t)sizeof(ElemT);
                    const uint8_t* from = a.packed + ((s0 + lb) * (ONE ? 1 : a.feat_dim) + d) * (int64_t)sizeof(ElemT);
                    for (int k = lb; k <= j; ++k, from += stride) sum += Elem<ElemT>::get(*reinterpret_cast<const ElemT*>(from));
                }
            }
            const int32_t start = lb >= 0 ? pos0 + lb : prev_start;
            const int32_t cnt = start >= 0 ? pos0 + j - start + 1 : pos0 + j + 1;
            const int32_t seq = lb < 0 ? prev_seq : (lb == last_break ? own_seq : a.seq_id[s0 + lb]);
            narrow_emit<Acc>(a, q, d, seq, (f.ends >> j) & 1u, start >= 0, sum, cnt, &s_desc);
        }
    }
    __syncthreads();
    if (tid == 0 && a.desc) a.desc[q] = s_desc;
}

// ----------------------------------------------------------------- stitch

// Segments cut by chunk borders: tail piece + the head pieces of the following
// chunks, added in time order.  One thread per (chunk, feature): a workgroup
// takes 256 features of one chunk, or, for frames of fewer than 256 features,
// all features of `chunks_per_wg` consecutive chunks.
template <typename Acc>
__global__ __launch_bounds__(kThreads) void reduce_stitch_kernel(ReduceArgs a, int32_t feat_tiles,
                                                                 int32_t chunks_per_wg)
{
    typedef typename OutOf<Acc>::T Out;
    int64_t q, d;
    if (chunks_per_wg > 1) {
        const int32_t r = (int32_t)threadIdx.x / a.feat_dim;
        if (r >= chunks_per_wg) return;
        q = (int64_t)blockIdx.x * chunks_per_wg + r;
        d = (int32_t)threadIdx.x - r * a.feat_dim;
        if (q >= a.total_chunks) return;
    } else {
        q = (int64_t)blockIdx.x / feat_tiles;
        d = ((int64_t)blockIdx.x % feat_tiles) * kThreads + threadIdx.x;
    }
    const ChunkDesc first = a.desc[q];
    if (first.cnt_tail <= 0 || d >= a.feat_dim) return;
    const Acc* head_part = static_cast<const Acc*>(a.head_part);
    const Acc* tail_part = static_cast<const Acc*>(a.tail_part);
    Running<Acc, sizeof(Acc) == 4> sum;
    sum.clear();
    sum.add(tail_part[q * a.feat_dim + d]);
    int64_t cnt = first.cnt_tail;
    for (int64_t q2 = q + 1; q2 < a.total_chunks; ++q2) {
        const ChunkDesc nd = a.desc[q2];
        if (nd.head_state == kHeadNone) break;
        sum.add(head_part[q2 * a.feat_dim + d]);
        cnt += nd.cnt_head;
        if (nd.head_state != kHeadThrough) break;
    }
    if ((uint32_t)first.seq_tail < (uint32_t)a.n_seq)
        static_cast<Out*>(a.out)[(int64_t)first.seq_tail * a.feat_dim + d] =
            finish<Acc>(sum.sum, (int32_t)cnt, a.mean);
}

// ------------------------------------------------------------------- host

struct ReducePlan {
    bool wide;
    int vec;                 // wide: elements per lane (16 / elem size, or 1)
    int row_lanes_log2;
    int n_vec;
    int32_t chunk, n_chunks;
    int32_t blocks_per_tile;  // narrow, t_blk < the tile: whole blocks per tile
    int64_t total_chunks;
    bool partials;           // can a chunk border cut a segment
    size_t desc_off, head_off, tail_off, bytes;
};

static int elem_size(bload_dtype dtype) { return dtype == BLOAD_U8 ? 1 : dtype == BLOAD_F16 ? 2 : 4; }

static ReducePlan reduce_plan(int64_t num_blocks, int32_t t_blk, int64_t feat_dim, bload_dtype dtype)
{
    ReducePlan p{};
    const int es = elem_size(dtype);
    const int64_t frame_bytes = feat_dim * es;
    const size_t acc = dtype == BLOAD_I32 ? 8 : 4;
    const bool vectors = frame_bytes % 16 == 0 && frame_bytes >= 64;
    p.wide = vectors || feat_dim >= 64;
    if (p.wide) {
        p.vec = vectors ? 16 / es : 1;
        p.n_vec = (int)ceil_div(feat_dim, p.vec);
        // a row is at most one wave wide: the last lane-slice of a frame then idles at most 63
        // lanes, and the four waves of a workgroup walk four different chunks
        p.row_lanes_log2 = 0;
        while ((1 << p.row_lanes_log2) < p.n_vec && p.row_lanes_log2 < 6) ++p.row_lanes_log2;
        const int rows = kThreads >> p.row_lanes_log2;
        const int64_t feat_tiles = ceil_div(p.n_vec, 1 << p.row_lanes_log2);
        // Enough chunks per block for ~1024 workgroups (four per compute unit, as many as are
        // resident at once), each at least 64 slots long.  No more: reads at full rate need few
        // waves in flight, while every chunk border costs partial sums, and writes mixed into the
        // read stream cost far more than their bytes.
        int64_t want = ceil_div((int64_t)1024 * rows, num_blocks * feat_tiles);
        const int64_t most = t_blk / 64 > 0 ? t_blk / 64 : 1;
        if (want > most) want = most;
        if (want < 1) want = 1;
        // Whole blocks that already make more workgroups than are resident at once (2048) run in
        // a few long rounds, and the last one leaves the chip half empty for a long time: then
        // chunks of at least 512 slots towards 12288 workgroups (34576 blocks of 3000 slots x 320
        // bytes: 3.98 ms in whole blocks, 3.89 in two chunks per block, 3.85 in three, 3.87 in
        // four, 3.91 in five).
        const int64_t whole_block_groups = num_blocks * feat_tiles / rows;
        if (want == 1 && whole_block_groups >= 2048 && whole_block_groups < 12288) {
            want = ceil_div((int64_t)12288, whole_block_groups);
            const int64_t most_long = t_blk / 512 > 0 ? t_blk / 512 : 1;
            if (want > most_long) want = most_long;
        }
        int64_t chunk = ceil_div(t_blk, want);
        const int64_t lds_cap = kWideFlagBytes / rows - 2;
        if (chunk > lds_cap) chunk = lds_cap;
        p.chunk = (int32_t)chunk;
        p.n_chunks = (int32_t)ceil_div(t_blk, chunk);
        p.total_chunks = num_blocks * p.n_chunks;
        p.partials = p.n_chunks > 1;
    } else {
        // tiles never straddle a block: pieces of one block, or several whole blocks
        p.chunk = kNarrowTile;
        if (t_blk >= kNarrowTile) {
            p.n_chunks = (int32_t)ceil_div(t_blk, kNarrowTile);
            p.blocks_per_tile = 1;
            p.total_chunks = num_blocks * p.n_chunks;
        } else {
            p.n_chunks = 1;
            p.blocks_per_tile = kNarrowTile / t_blk;
            p.total_chunks = ceil_div(num_blocks, p.blocks_per_tile);
        }
        // only a block cut into several tiles can have a segment across a tile border
        p.partials = p.n_chunks > 1;
    }
    if (p.partials) {
        size_t off = 0;
        p.desc_off = off; off += round_up((size_t)p.total_chunks * sizeof(ChunkDesc), 16);
        p.head_off = off; off += round_up((size_t)p.total_chunks * (size_t)feat_dim * acc, 16);
        p.tail_off = off; off += round_up((size_t)p.total_chunks * (size_t)feat_dim * acc, 16);
        p.bytes = off;
    }
    return p;
}

template <typename ElemT>
static void launch_wide(const ReducePlan& p, const ReduceArgs& a, hipStream_t stream)
{
    const int rows = kThreads >> p.row_lanes_log2;
    const dim3 grid((uint32_t)(ceil_div(p.total_chunks, rows) * a.feat_tiles));
    size_t lds = (size_t)rows * (size_t)(p.chunk + 2);
    if (p.vec > 1 && p.row_lanes_log2 >= 6)     // + the per-wave scratch of the transposed stores
        lds = round_up(lds, 16) + (size_t)(kThreads / kWave) * kWave *
                                      kScratchStride<typename Elem<ElemT>::Acc, 16 / (int)sizeof(ElemT)>() *
                                      sizeof(typename Elem<ElemT>::Acc);
    constexpr int kVec = 16 / (int)sizeof(ElemT);
    const bool wave_row = p.row_lanes_log2 == 6;
    if (p.vec > 1 && wave_row)
        hipLaunchKernelGGL((reduce_wide_kernel<ElemT, kVec, true>), grid, dim3(kThreads), lds, stream, a);
    else if (p.vec > 1)
        hipLaunchKernelGGL((reduce_wide_kernel<ElemT, kVec, false>), grid, dim3(kThreads), lds, stream, a);
    else if (wave_row)
        hipLaunchKernelGGL((reduce_wide_kernel<ElemT, 1, true>), grid, dim3(kThreads), lds, stream, a);
    else
        hipLaunchKernelGGL((reduce_wide_kernel<ElemT, 1, false>), grid, dim3(kThreads), lds, stream, a);
}

template <typename ElemT>
static void launch_reduce(const ReducePlan& p, const ReduceArgs& a, hipStream_t stream)
{
    typedef typename Elem<ElemT>::Acc Acc;
    if (p.wide) {
        launch_wide<ElemT>(p, a, stream);
    } else {
        if (a.feat_dim == 1)
            hipLaunchKernelGGL((reduce_narrow_kernel<ElemT, true>), dim3((uint32_t)p.total_chunks),
                               dim3(kThreads), 0, stream, a);
        else
            hipLaunchKernelGGL((reduce_narrow_kernel<ElemT, false>), dim3((uint32_t)p.total_chunks),
                               dim3(kThreads), 0, stream, a);
    }
    if (p.partials) {
        const int32_t feat_tiles = (int32_t)ceil_div(a.feat_dim, kThreads);
        const int32_t chunks_per_wg = a.feat_dim >= kThreads ? 1 : kThreads / a.feat_dim;
        const int64_t groups = chunks_per_wg > 1 ? ceil_div(p.total_chunks, chunks_per_wg)
                                                 : p.total_chunks * feat_tiles;
        hipLaunchKernelGGL(reduce_stitch_kernel<Acc>, dim3((uint32_t)groups), dim3(kThreads), 0, stream,
                           a, feat_tiles, chunks_per_wg);
    }
}

}  // namespace bload

using namespace bload;

extern "C" size_t bload_segment_reduce_workspace_bytes(int64_t num_blocks, int32_t t_blk,
                                                       int64_t feat_dim, bload_dtype dtype)
{
    if (num_blocks <= 0 || t_blk < 1 || feat_dim < 1 || (int)dtype < 0 || (int)dtype > 3) return 0;
    return reduce_plan(num_blocks, t_blk, feat_dim, dtype).bytes;
}

extern "C" bload_status bload_segment_reduce(const void* d_packed, const int32_t* d_seq_id,
                                             const uint8_t* d_reset, const uint8_t* d_valid,
                                             int64_t num_blocks, int32_t t_blk, int64_t feat_dim,
                                             bload_dtype dtype, bload_op op, int64_t n_seq,
                                             void* d_out, void* d_workspace, size_t workspace_bytes,
                                             void* hip_stream)
{
    if (num_blocks < 0 || t_blk < 1 || feat_dim < 1 || n_seq < 0) return BLOAD_EINVAL;
    if ((int)dtype < 0 || (int)dtype > 3 || (int)op < 0 || (int)op > 1) return BLOAD_EINVAL;
    if (dtype == BLOAD_I32 && op == BLOAD_MEAN) return BLOAD_EINVAL;
    if (n_seq > BLOAD_MAX_SEQ || feat_dim >= ((int64_t)1 << 28)) return BLOAD_EOVERFLOW;
    if (num_blocks == 0 || n_seq == 0) return BLOAD_OK;
    if (!d_packed || !d_seq_id || !d_reset || !d_valid || !d_out) return BLOAD_EINVAL;
    const int64_t total_slots = num_blocks * (int64_t)t_blk;
    if (total_slots >= ((int64_t)1 << 40)) return BLOAD_EOVERFLOW;
    if (!aligned_to(d_packed, 16) || !aligned_to(d_seq_id, 4) || !aligned_to(d_reset, 16) ||
        !aligned_to(d_valid, 16) || !aligned_to(d_out, 8))
        return BLOAD_EALIGN;

    const ReducePlan p = reduce_plan(num_blocks, t_blk, feat_dim, dtype);
    if (p.total_chunks * ceil_div(feat_dim, kThreads) > INT32_MAX) return BLOAD_EOVERFLOW;
    if (p.wide && ceil_div(p.total_chunks, kThreads >> p.row_lanes_log2) *
                      ceil_div(p.n_vec, 1 << p.row_lanes_log2) > INT32_MAX)
        return BLOAD_EOVERFLOW;
    if (p.partials) {
        if (!d_workspace) return BLOAD_EINVAL;
        if (!aligned_to(d_workspace, 16)) return BLOAD_EALIGN;
        if (workspace_bytes < p.bytes) return BLOAD_EWORKSPACE;
    }

    ReduceArgs a{};
    a.packed = static_cast<const uint8_t*>(d_packed);
    a.seq_id = d_seq_id;
    a.reset = d_reset;
    a.valid = d_valid;
    a.num_blocks = num_blocks;
    a.total_slots = total_slots;
    a.total_chunks = p.total_chunks;
    a.t_blk = t_blk;
    a.feat_dim = (int32_t)feat_dim;
    a.n_seq = (int32_t)n_seq;
    a.mean = op == BLOAD_MEAN ? 1 : 0;
    a.blocks_per_tile = p.blocks_per_tile;
    a.magic_t_blk = (uint32_t)std::min<uint64_t>((((uint64_t)1 << 32) + (uint64_t)t_blk - 1) / (uint64_t)t_blk, 0xFFFFFFFFull);
    a.out = d_out;
    a.chunk = p.chunk;
    a.n_chunks = p.n_chunks;
    a.row_lanes_log2 = p.row_lanes_log2;
    a.n_vec = p.n_vec;
    a.feat_tiles = p.wide ? (int32_t)ceil_div(p.n_vec, 1 << p.row_lanes_log2) : 1;
    if (p.partials) {
        uint8_t* ws = static_cast<uint8_t*>(d_workspace);
        a.desc = reinterpret_cast<ChunkDesc*>(ws + p.desc_off);
        a.head_part = ws + p.head_off;
        a.tail_part = ws + p.tail_off;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    switch (dtype) {
        case BLOAD_U8: launch_reduce<uint8_t>(p, a, stream); break;
        case BLOAD_F16: launch_reduce<half_bits>(p, a, stream); break;
        case BLOAD_F32: launch_reduce<float>(p, a, stream); break;
        case BLOAD_I32: launch_reduce<int32_t>(p, a, stream); break;
    }
    return launch_status();
}
