// bload_segment_scan: the recurrent consumer of the start table (BLoad, Methods section and
// the figure of the DDS model: what frame n-1 produced is part of the input of frame n, and
// the table says where that carried state belongs to another sequence and is dropped).
// Per feature:  h = x at the first frame of a sequence,  h = decay * h + x afterwards;
// padding slots yield 0.  Output float32 [B, t_blk, feat_dim].
//
// HBM bound, and write heavy (4 output bytes per element).  The recurrence runs along time,
// so parallelism comes from blocks, features and chunks of time.  A slot that is padding or
// starts a sequence ("boundary") depends on nothing before it; only a sequence that runs
// across a chunk border hands a state on.  Three kernels, all deterministic:
//   scan_tail_kernel   per chunk (but the block's last): the state it would hand on if it
//                      received none - the recurrence from the chunk's last boundary (or its
//                      first slot) to its end - and whether it holds a boundary at all
//   scan_chain_kernel  per block and feature, along the chunks: state handed to chunk c+1 =
//                      the tail state of chunk c, plus decay^chunk * (state handed to c) when
//                      chunk c holds no boundary
//   scan_apply_kernel  per chunk: the recurrence over its own slots from the state handed in
// Every slot is read and written once by scan_apply; scan_tail re-reads only the open ends
// of the chunks.  With one chunk per block only scan_apply runs.
//
// A row of lanes (16 input bytes per lane where the frame allows it, taken as quads of 4
// elements laid out so that every load and store instruction of the row is contiguous; else
// one element per lane) covers the features; a wavefront holds 64 / row-width rows, each on
// a chunk of its own.  All loads of a step (8 slots) are issued together; a step of nothing but
// padding issues none.
#include "bload_common.hpp"

#include <hip/hip_fp16.h>
#include <math.h>

namespace bload {

constexpr int kScanBatch = 8;          // slots per step and row: their loads are in flight together
constexpr uint32_t kScanAll = (1u << kScanBatch) - 1u;
static_assert(kScanBatch % 8 == 0 && kScanBatch <= 24, "flags come eight to a load");

struct ScanArgs {
    const uint8_t* packed;
    const uint8_t* reset;
    const uint8_t* valid;
    float* out;
    float* carry;                      // [B, chunks_per_block - 1, feat_dim]: tail states, then states handed on
    uint8_t* has_boundary;             // [B, chunks_per_block - 1]
    int64_t num_blocks;
    int64_t total_slots;               // num_blocks * t_blk
    int32_t t_blk;
    int32_t feat_dim;
    int32_t chunk;                     // slots per chunk
    int32_t chunks_per_block;
    int32_t row_lanes;                 // lanes per row: a power of two <= 64
    int32_t feat_tiles;                // rows needed to cover the features (1 unless row_lanes == 64)
    int32_t n_vec;                     // quads (4 elements) of a frame, or elements where a frame
                                       // is not a whole number of 16-byte pieces
    float decay;
    float decay_chunk;                 // decay ^ chunk
};

template <typename ElemT> struct ScanElem;
template <> struct ScanElem<uint8_t> {
    __device__ static float get(uint8_t v) { return (float)v; }
};
struct scan_half { uint16_t bits; };   // IEEE binary16 storage
template <> struct ScanElem<scan_half> {
    __device__ static float get(scan_half v) { return __half2float(__ushort_as_half(v.bits)); }
};
template <> struct ScanElem<float> {
    __device__ static float get(float v) { return v; }
};

typedef float float4v __attribute__((ext_vector_type(4)));

// Four consecutive elements ("quad") as loaded: 4, 8 or 16 bytes in one instruction.
typedef unsigned int vec8 __attribute__((ext_vector_type(2)));
template <int BYTES> struct ScanBits;
template <> struct ScanBits<4> { typedef unsigned int T; };
template <> struct ScanBits<8> { typedef vec8 T; };
template <> struct ScanBits<16> { typedef vec16 T; };
template <typename ElemT> union ScanQuad {
    typename ScanBits<sizeof(ElemT) * 4>::T bits;
    ElemT e[4];
};

// Flags of the 8 consecutive slots from global slot g on (`plane` covers `total` slots): bit u set
// iff the flag of slot g + u is non-zero; slots at or behind `total` read as 0.  One 8-byte load
// that never leaves the plane; a non-zero byte becomes a 1, and two byte-wise dot products with
// the weights 1, 2, 4, ... gather the eight 1s into eight bits.  TINY: the plane holds fewer than
// 8 slots, which are read one by one.
template <bool TINY>
__device__ __forceinline__ uint32_t scan_flags8(const uint8_t* __restrict__ plane, int64_t g, int64_t total)
{
    typedef uint64_t word_any __attribute__((aligned(1)));
    uint64_t w;
    if (!TINY) {
        const int64_t from = min(g, total - 8);
        w = *reinterpret_cast<const word_any*>(plane + from) >> (8 * (int)(g - from));
    } else {
        w = 0;
        for (int u = 0; u < 8; ++u)
            if (g + u < total) w |= (uint64_t)plane[g + u] << (8 * u);
    }
    const uint32_t lo = (uint32_t)w, hi = (uint32_t)(w >> 32);
    const uint32_t lo1 = ((((lo & 0x7f7f7f7fu) + 0x7f7f7f7fu) | lo) >> 7) & 0x01010101u;
    const uint32_t hi1 = ((((hi & 0x7f7f7f7fu) + 0x7f7f7f7fu) | hi) >> 7) & 0x01010101u;
    return __builtin_amdgcn_udot4(hi1, 0x80402010u, __builtin_amdgcn_udot4(lo1, 0x08040201u, 0u, false), false);
}

// Flags of the kScanBatch slots from slot t of a block on (g = the same slot counted over all
// blocks), and which of them are boundaries: padding, a start flag, the block's first slot, or
// the slot after padding.  Slots behind the block's end read as 0.  `before`: was slot t - 1 valid.
struct ScanFlags { uint32_t valid, boundary; };
template <bool TINY>
__device__ __forceinline__ ScanFlags scan_flags(const uint8_t* __restrict__ valid,
                                                const uint8_t* __restrict__ reset, int64_t g, int64_t total,
                                                int32_t t, int32_t T, uint32_t before)
{
    const uint32_t in_range = T - t >= kScanBatch ? kScanAll : (1u << (T - t)) - 1u;
    uint32_t vm = 0, rm = 0;
#pragma unroll
    for (int part = 0; part < kScanBatch; part += 8) {
        if (part == 0 || t + part < T) {
            vm |= scan_flags8<TINY>(valid, g + part, total) << part;
            rm |= scan_flags8<TINY>(reset, g + part, total) << part;
        }
    }
    vm &= in_range;
    const uint32_t prev_valid = (vm << 1) | before;
    return ScanFlags{vm, in_range & (~vm | rm | ~prev_valid | (t == 0 ? 1u : 0u))};
}

// What a lane works on.  It holds QUADS quads of a frame: quad g of lane r in a row of
// `row_lanes` lanes is quad number tile_base + g * row_lanes + r, so that each load and each
// store instruction of a row covers one contiguous stretch of the frame.
template <typename ElemT, int QUADS, bool VEC, bool TINY>
struct ScanLane {
    static constexpr int EPL = VEC ? QUADS * 4 : 1;      // elements per lane
    bool idle;
    int64_t block;
    int32_t chunk;
    int32_t t0, t1;                    // the chunk's slots inside the block
    int64_t first_elem;                // first element of the lane inside a frame
    int32_t quad_stride;               // elements between the lane's quads
    bool quad_on[QUADS];

    __device__ __forceinline__ ScanLane(const ScanArgs& a, int32_t chunks_used)
    {
        const int lane = lane_id();
        const int rows_per_wave = kWave / a.row_lanes;
        const int64_t wave = (int64_t)xcd_contiguous(blockIdx.x, gridDim.x) * (kThreads / kWave) + wave_id();
        const int32_t feat_tile = (int32_t)(wave % a.feat_tiles);
        const int64_t item = (wave / a.feat_tiles) * rows_per_wave + lane / a.row_lanes;
        const int32_t r = lane & (a.row_lanes - 1);
        const int32_t first = VEC ? feat_tile * a.row_lanes * QUADS + r : feat_tile * a.row_lanes + r;
        idle = item >= a.num_blocks * chunks_used || first >= a.n_vec;
        block = idle ? 0 : item / chunks_used;
        chunk = idle ? 0 : (int32_t)(item - block * chunks_used);
        t0 = chunk * a.chunk;
        t1 = min(a.t_blk, t0 + a.chunk);
        if (t0 >= a.t_blk) idle = true;
        first_elem = (int64_t)first * (VEC ? 4 : 1);
        quad_stride = a.row_lanes * 4;
#pragma unroll
        for (int g = 0; g < QUADS; ++g) quad_on[g] = !VEC || first + g * a.row_lanes < a.n_vec;
    }

    // kScanBatch slots from t on: the recurrence goes on in h; the first `keep` slots are handed
    // to `emit(u, g, quad)`.  `at`: the lane's first byte of slot t.  FULL: all kScanBatch slots
    // lie in the block and all are kept, which spares every clamp and test; otherwise slots
    // behind the block's end re-read its last slot.  A batch of nothing but padding (block
    // tails) costs no read: every state ends there and every output is 0.  h = decay * h + x is
    // one fused multiply-add (one rounding), the state of a boundary slot being replaced by 0
    // first (never multiplied: it may be infinite).
    template <bool FULL, typename Emit>
    __device__ __forceinline__ void step(const ScanArgs& a, const uint8_t* __restrict__ at, int32_t t,
                                         ScanFlags f, float (&h)[EPL], int keep, Emit emit) const
    {
        const int64_t frame_bytes = (int64_t)a.feat_dim * (int64_t)sizeof(ElemT);
        if (f.valid == 0) {
#pragma unroll
            for (int k = 0; k < EPL; ++k) h[k] = 0.0f;
            const float4v zero = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int u = 0; u < kScanBatch; ++u) {
#pragma unroll
                for (int g = 0; g < (VEC ? QUADS : 1); ++g)
                    if ((FULL || u < keep) && quad_on[g]) emit(u, g, zero);
            }
            return;
        }
        const int32_t last = a.t_blk - 1 - t;              // the block's last slot, counted from t
        if (VEC) {
            ScanQuad<ElemT> x[kScanBatch][QUADS];
#pragma unroll
            for (int u = 0; u < kScanBatch; ++u) {
                const uint8_t* frame = at + (int64_t)(FULL ? u : min(u, last)) * frame_bytes;
#pragma unroll
                for (int g = 0; g < QUADS; ++g) {
                    const int64_t off = quad_on[g] ? (int64_t)g * quad_stride * (int64_t)sizeof(ElemT) : 0;
                    x[u][g].bits = __builtin_nontemporal_load(
                        reinterpret_cast<const typename ScanBits<sizeof(ElemT) * 4>::T*>(frame + off));
                }
            }
#pragma unroll
            for (int u = 0; u < kScanBatch; ++u) {
                const bool is_valid = (f.valid >> u) & 1u, starts = (f.boundary >> u) & 1u;
#pragma unroll
                for (int g = 0; g < QUADS; ++g) {
                    float4v o;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float xv = is_valid ? ScanElem<ElemT>::get(x[u][g].e[j]) : 0.0f;
                        h[g * 4 + j] = __builtin_fmaf(a.decay, starts ? 0.0f : h[g * 4 + j], xv);
                        o[j] = h[g * 4 + j];
                    }
                    if ((FULL || u < keep) && quad_on[g]) emit(u, g, o);
                }
            }
        } else {
            ElemT x[kScanBatch];
#pragma unroll
            for (int u = 0; u < kScanBatch; ++u)
                x[u] = *reinterpret_cast<const ElemT*>(at + (int64_t)(FULL ? u : min(u, last)) * frame_bytes);
#pragma unroll
            for (int u = 0; u < kScanBatch; ++u) {
                const bool is_valid = (f.valid >> u) & 1u, starts = (f.boundary >> u) & 1u;
                const float xv = is_valid ? ScanElem<ElemT>::get(x[u]) : 0.0f;
                h[0] = __builtin_fmaf(a.decay, starts ? 0.0f : h[0], xv);
                float4v o = {h[0], 0.0f, 0.0f, 0.0f};
                if (FULL || u < keep) emit(u, 0, o);
            }
        }
    }

    // The recurrence over the slots [from, t1) of the lane's block from the state in h, batch by
    // batch.  `emit(t, n, u, g, quad)`: slot t + u of a batch of n slots that begins at slot t.
    template <typename Emit>
    __device__ __forceinline__ void recur(const ScanArgs& a, int32_t from, int32_t t1, float (&h)[EPL], Emit emit) const
    {
        const int64_t frame_bytes = (int64_t)a.feat_dim * (int64_t)sizeof(ElemT);
        const int64_t slot0 = block * a.t_blk;
        const uint8_t* at = a.packed + ((slot0 + from) * a.feat_dim + first_elem) * (int64_t)sizeof(ElemT);
        uint32_t before = from > 0 ? (a.valid[slot0 + from - 1] != 0) : 0u;
        for (int32_t t = from; t < t1; t += kScanBatch, at += (int64_t)kScanBatch * frame_bytes) {
            const ScanFlags f = scan_flags<TINY>(a.valid, a.reset, slot0 + t, a.total_slots, t, a.t_blk, before);
            const int n = min(kScanBatch, t1 - t);
            auto out = [&](int u, int g, float4v o) { emit(t, n, u, g, o); };
            if (n == kScanBatch) step<true>(a, at, t, f, h, n, out);
            else step<false>(a, at, t, f, h, n, out);
            before = (f.valid >> (n - 1)) & 1u;
        }
    }
};

// The state a chunk hands on when it receives none, and whether it holds a boundary.
template <typename ElemT, int QUADS, bool VEC, bool TINY>
__global__ __launch_bounds__(kThreads) void scan_tail_kernel(ScanArgs a)
{
    typedef ScanLane<ElemT, QUADS, VEC, TINY> Lane;
    const Lane me(a, a.chunks_per_block - 1);                 // the block's last chunk hands nothing on
    if (me.idle) return;
    const int64_t slot0 = me.block * a.t_blk;

    // the chunk's last boundary
    int32_t last = -1;
    uint32_t before = me.t0 > 0 ? (a.valid[slot0 + me.t0 - 1] != 0) : 0u;
    for (int32_t t = me.t0; t < me.t1; t += kScanBatch) {
        const ScanFlags f = scan_flags<TINY>(a.valid, a.reset, slot0 + t, a.total_slots, t, a.t_blk, before);
        const int n = min(kScanBatch, me.t1 - t);
        const uint32_t mine = f.boundary & ((1u << n) - 1u);
        if (mine) last = t + 31 - __builtin_clz(mine);
        before = (f.valid >> (n - 1)) & 1u;
    }

    // the recurrence from there (from the chunk's first slot if there is none) to the chunk's end
    const int32_t from = last >= 0 ? last : me.t0;
    float h[Lane::EPL];
#pragma unroll
    for (int k = 0; k < Lane::EPL; ++k) h[k] = 0.0f;
    float* carry = a.carry + (me.block * (a.chunks_per_block - 1) + me.chunk) * (int64_t)a.feat_dim + me.first_elem;
    me.recur(a, from, me.t1, h, [&](int32_t t, int n, int u, int g, float4v o) {
        if (t + n >= me.t1 && u == n - 1) {
            if (VEC) *reinterpret_cast<float4v*>(carry + g * me.quad_stride) = o;
            else carry[0] = o[0];
        }
    });
    if (me.first_elem == 0) a.has_boundary[me.block * (a.chunks_per_block - 1) + me.chunk] = last >= 0;
}

// Along the chunks of a block: what chunk c + 1 is handed = the tail state of chunk c, plus
// decay^chunk times what chunk c was handed if chunk c holds no boundary.  In place.
__global__ __launch_bounds__(kThreads) void scan_chain_kernel(ScanArgs a)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= a.num_blocks * a.feat_dim) return;
    const int64_t block = idx / a.feat_dim, d = idx - block * a.feat_dim;
    const int32_t links = a.chunks_per_block - 1;
    float handed = 0.0f;
    for (int32_t c = 0; c < links; ++c) {
        const int64_t at = (block * links + c) * (int64_t)a.feat_dim + d;
        const float tail = a.carry[at];
        // a state of exactly 0 stays 0 whatever decay^chunk is (it may have overflowed to inf)
        handed = (a.has_boundary[block * links + c] || handed == 0.0f) ? tail : a.decay_chunk * handed + tail;
        a.carry[at] = handed;
    }
}

// The recurrence over a chunk's own slots, from the state handed in.
template <typename ElemT, int QUADS, bool VEC, bool TINY>
__global__ __launch_bounds__(kThreads) void scan_apply_kernel(ScanArgs a)
{
    typedef ScanLane<ElemT, QUADS, VEC, TINY> Lane;
    const Lane me(a, a.chunks_per_block);
    if (me.idle) return;
    float h[Lane::EPL];
#pragma unroll
    for (int k = 0; k < Lane::EPL; ++k) h[k] = 0.0f;
    if (me.chunk > 0) {
        const float* handed = a.carry + (me.block * (a.chunks_per_block - 1) + me.chunk - 1) * (int64_t)a.feat_dim +
                              me.first_elem;
#pragma unroll
        for (int g = 0; g < QUADS; ++g) {
            if (me.quad_on[g]) {
                if (VEC) {
                    const float4v v = *reinterpret_cast<const float4v*>(handed + g * me.quad_stride);
#pragma unroll
                    for (int j = 0; j < 4; ++j) h[g * 4 + j] = v[j];
                } else {
                    h[0] = handed[0];
                }
            }
        }
    }
    float* dst = a.out + me.block * a.t_blk * (int64_t)a.feat_dim + me.first_elem;
    me.recur(a, me.t0, me.t1, h, [&](int32_t t, int, int u, int g, float4v o) {
        float* to = dst + (int64_t)(t + u) * a.feat_dim;
        if (VEC) __builtin_nontemporal_store(o, reinterpret_cast<float4v*>(to + g * me.quad_stride));
        else __builtin_nontemporal_store(o[0], to);
    });
}

struct ScanPlan {
    int32_t epv, n_vec, row_lanes, feat_tiles, chunk, chunks_per_block;
    int64_t rows_per_wave;
    bool tiny;
    size_t carry_bytes, bytes;         // workspace: the states handed on, then the boundary marks
};

static ScanPlan scan_plan(int64_t num_blocks, int32_t t_blk, int64_t feat_dim, size_t elem)
{
    ScanPlan p{};
    // whole 16-byte pieces per frame: a lane takes 16 / elem elements as quads; else one element
    p.epv = (feat_dim * (int64_t)elem) % 16 == 0 ? (int32_t)(16 / elem) : 1;
    p.tiny = num_blocks * t_blk < 8;               // flags cannot be read eight at a time
    if (p.tiny) p.epv = 1;
    p.n_vec = p.epv > 1 ? (int32_t)(feat_dim / 4) : (int32_t)feat_dim;      // quads, or elements
    const int64_t per_lane = p.epv > 1 ? p.epv / 4 : 1;
    p.row_lanes = 1;
    while (p.row_lanes < kWave && p.row_lanes * per_lane < p.n_vec) p.row_lanes *= 2;
    p.feat_tiles = (int32_t)ceil_div(p.n_vec, p.row_lanes * per_lane);
    p.rows_per_wave = kWave / p.row_lanes;
    // enough wavefronts to fill the chip several times over, chunks not shorter than 64 slots
    const int64_t want_waves = 6144;
    int64_t chunks = ceil_div(want_waves * p.rows_per_wave, (num_blocks > 0 ? num_blocks : 1) * p.feat_tiles);
    const int64_t most = t_blk / 64 > 1 ? t_blk / 64 : 1;
    if (chunks > most) chunks = most;
    if (chunks < 1) chunks = 1;
    p.chunk = (int32_t)round_up((size_t)ceil_div(t_blk, chunks), kScanBatch);
    p.chunks_per_block = (int32_t)ceil_div(t_blk, p.chunk);
    const size_t links = (size_t)(num_blocks > 0 ? num_blocks : 0) * (size_t)(p.chunks_per_block - 1);
    p.carry_bytes = round_up(links * (size_t)feat_dim * sizeof(float), 16);
    p.bytes = p.carry_bytes + round_up(links, 16);
    return p;
}

static size_t scan_elem_bytes(bload_dtype dtype)
{
    return dtype == BLOAD_U8 ? 1 : (dtype == BLOAD_F16 ? 2 : 4);
}

template <typename ElemT>
static void scan_launch(const ScanArgs& a, const ScanPlan& p, hipStream_t stream)
{
    constexpr int kQuads = 4 / (int)sizeof(ElemT);           // quads in 16 input bytes
    const dim3 block(kThreads);
    const int waves_per_group = kThreads / kWave;
    if (p.chunks_per_block > 1) {
        const int64_t waves = ceil_div(a.num_blocks * (p.chunks_per_block - 1), p.rows_per_wave) * p.feat_tiles;
        const dim3 grid((uint32_t)ceil_div(waves, waves_per_group));
        if (p.epv > 1) hipLaunchKernelGGL((scan_tail_kernel<ElemT, kQuads, true, false>), grid, block, 0, stream, a);
        else if (!p.tiny) hipLaunchKernelGGL((scan_tail_kernel<ElemT, 1, false, false>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((scan_tail_kernel<ElemT, 1, false, true>), grid, block, 0, stream, a);
        hipLaunchKernelGGL(scan_chain_kernel, dim3((uint32_t)ceil_div(a.num_blocks * a.feat_dim, kThreads)),
                           block, 0, stream, a);
    }
    const int64_t waves = ceil_div(a.num_blocks * p.chunks_per_block, p.rows_per_wave) * p.feat_tiles;
    const dim3 grid((uint32_t)ceil_div(waves, waves_per_group));
    if (p.epv > 1) hipLaunchKernelGGL((scan_apply_kernel<ElemT, kQuads, true, false>), grid, block, 0, stream, a);
    else if (!p.tiny) hipLaunchKernelGGL((scan_apply_kernel<ElemT, 1, false, false>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((scan_apply_kernel<ElemT, 1, false, true>), grid, block, 0, stream, a);
}

}  // namespace bload

using namespace bload;

extern "C" size_t bload_segment_scan_workspace_bytes(int64_t num_blocks, int32_t t_blk, int64_t feat_dim,
                                                     bload_dtype dtype)
{
    if (num_blocks < 0 || t_blk < 1 || feat_dim < 1 || feat_dim > (1 << 28)) return 0;
    if (dtype != BLOAD_U8 && dtype != BLOAD_F16 && dtype != BLOAD_F32) return 0;
    return scan_plan(num_blocks, t_blk, feat_dim, scan_elem_bytes(dtype)).bytes;
}

extern "C" bload_status bload_segment_scan(const void* d_packed, const uint8_t* d_reset,
                                           const uint8_t* d_valid, int64_t num_blocks, int32_t t_blk,
                                           int64_t feat_dim, bload_dtype dtype, float decay,
                                           float* d_out, void* d_workspace, size_t workspace_bytes,
                                           void* hip_stream)
{
    if (num_blocks < 0 || t_blk < 1 || feat_dim < 1 || feat_dim > (1 << 28)) return BLOAD_EINVAL;
    if (dtype != BLOAD_U8 && dtype != BLOAD_F16 && dtype != BLOAD_F32) return BLOAD_EINVAL;
    if (num_blocks == 0) return BLOAD_OK;
    if (!d_packed || !d_reset || !d_valid || !d_out) return BLOAD_EINVAL;
    if (!aligned_to(d_packed, 16) || !aligned_to(d_out, 16)) return BLOAD_EALIGN;
    if (num_blocks * (int64_t)t_blk >= ((int64_t)1 << 40)) return BLOAD_EOVERFLOW;
    const ScanPlan p = scan_plan(num_blocks, t_blk, feat_dim, scan_elem_bytes(dtype));
    if (p.bytes > 0) {
        if (!d_workspace) return BLOAD_EINVAL;
        if (!aligned_to(d_workspace, 16)) return BLOAD_EALIGN;
        if (workspace_bytes < p.bytes) return BLOAD_EWORKSPACE;
    }
    const int64_t most_waves = ceil_div(num_blocks * p.chunks_per_block, p.rows_per_wave) * p.feat_tiles;
    if (ceil_div(most_waves, kThreads / kWave) > 0x7fffffffLL ||
        ceil_div(num_blocks * feat_dim, kThreads) > 0x7fffffffLL)
        return BLOAD_EOVERFLOW;

    ScanArgs a{};
    a.packed = static_cast<const uint8_t*>(d_packed);
    a.reset = d_reset;
    a.valid = d_valid;
    a.out = d_out;
    a.carry = static_cast<float*>(d_workspace);
    a.has_boundary = static_cast<uint8_t*>(d_workspace) + p.carry_bytes;
    a.num_blocks = num_blocks;
    a.total_slots = num_blocks * (int64_t)t_blk;
    a.t_blk = t_blk;
    a.feat_dim = (int32_t)feat_dim;
    a.chunk = p.chunk;
    a.chunks_per_block = p.chunks_per_block;
    a.row_lanes = p.row_lanes;
    a.feat_tiles = p.feat_tiles;
    a.n_vec = p.n_vec;
    a.decay = decay;
    a.decay_chunk = (float)pow((double)decay, (double)p.chunk);

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (dtype == BLOAD_U8) scan_launch<uint8_t>(a, p, stream);
    else if (dtype == BLOAD_F16) scan_launch<scan_half>(a, p, stream);
    else scan_launch<float>(a, p, stream);
    return launch_status();
}
