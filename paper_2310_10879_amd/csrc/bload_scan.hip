// bload_segment_scan: the recurrent consumer of the start table (BLoad, Methods section and
// the figure of the DDS model: what frame n-1 produced is part of the input of frame n, and
// the table says where that carried state belongs to another sequence and is dropped).
// Per feature:  h = x at the first frame of a sequence,  h = decay * h + x afterwards;
// padding slots yield 0.  Output float32 [B, t_blk, feat_dim].
//
// HBM bound, and write heavy (4 output bytes per element).  The recurrence runs along time,
// so parallelism comes from blocks, features and *pieces of time that need no carry-in*:
// a slot that is padding or starts a sequence ("boundary") depends on nothing before it.
// Time is cut into chunks; the worker of a chunk owns the slots from the chunk's first
// boundary up to the first boundary at or behind the chunk's end.  Every slot has exactly
// one owner, is read once and written once, and no worker ever waits for another.
//
// A row of lanes (16 input bytes per lane where the frame allows it, taken as quads of 4
// elements laid out so that every load and store instruction of the row is contiguous; else
// one element per lane) covers the features; a wavefront holds 64 / row-width rows, each on
// a chunk of its own.  All loads of a pass are unconditional and issued together.
#include "bload_common.hpp"

#include <hip/hip_fp16.h>

namespace bload {

constexpr int kScanBatch = 8;          // slots per step and row: their loads are in flight together

struct ScanArgs {
    const uint8_t* packed;
    const uint8_t* reset;
    const uint8_t* valid;
    float* out;
    int64_t items;                     // num_blocks * chunks_per_block
    int32_t t_blk;
    int32_t feat_dim;
    int32_t chunk;                     // slots per chunk
    int32_t chunks_per_block;
    int32_t row_lanes;                 // lanes per row: a power of two <= 64
    int32_t feat_tiles;                // rows needed to cover the features (1 unless row_lanes == 64)
    int32_t n_vec;                     // quads (4 elements) of a frame, or elements where a frame
                                       // is not a whole number of 16-byte pieces
    float decay;
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

// Flags of 8 consecutive slots starting at `t` of a block of `T` slots (`plane` points at
// the block's first flag): bit u set iff the flag of slot t + u is non-zero; slots at or
// behind T read as 0.  One 8-byte load that never leaves the block.
__device__ __forceinline__ uint32_t scan_flags8(const uint8_t* __restrict__ plane, int32_t t, int32_t T)
{
    typedef uint64_t word_any __attribute__((aligned(1)));
    uint64_t w;
    if (T >= 8) {
        const int32_t from = min(t, T - 8);
        w = *reinterpret_cast<const word_any*>(plane + from) >> (8 * (t - from));
    } else {
        w = 0;
        for (int u = 0; u < 8; ++u) w |= (uint64_t)plane[min(t + u, T - 1)] << (8 * u);
        if (T - t < 8) w &= ~0ull >> (8 * (8 - (T - t)));
    }
    // non-zero byte -> its top bit -> one bit per byte
    const uint64_t low7 = 0x7f7f7f7f7f7f7f7full;
    const uint64_t top = ((w & low7) + low7 | w) & ~low7;
    return (uint32_t)(((top >> 7) * 0x0102040810204080ull) >> 56);
}

// A lane holds QUADS quads of a frame: quad g of lane r in a row of `row_lanes` lanes is
// quad number tile_base + g * row_lanes + r, so that each load and each store instruction of
// a row covers one contiguous stretch of the frame.
template <typename ElemT, int QUADS, bool VEC>
__global__ __launch_bounds__(kThreads) void scan_kernel(ScanArgs a)
{
    constexpr int EPL = VEC ? QUADS * 4 : 1;             // elements per lane
    const int lane = lane_id();
    const int rows_per_wave = kWave / a.row_lanes;
    const int64_t wave = (int64_t)blockIdx.x * (kThreads / kWave) + wave_id();
    const int32_t feat_tile = (int32_t)(wave % a.feat_tiles);
    const int64_t item = (wave / a.feat_tiles) * rows_per_wave + lane / a.row_lanes;
    const int32_t r = lane & (a.row_lanes - 1);
    // first quad (VEC) or element of the lane
    const int32_t first = VEC ? feat_tile * a.row_lanes * QUADS + r : feat_tile * a.row_lanes + r;

    bool done = item >= a.items || first >= a.n_vec;
    const int64_t block = done ? 0 : item / a.chunks_per_block;
    const int32_t chunk = done ? 0 : (int32_t)(item - block * a.chunks_per_block);
    const int64_t slot0 = block * a.t_blk;                     // first slot of the block
    const int32_t T = a.t_blk;
    int32_t t = chunk * a.chunk;
    const int32_t t_end = min(T, t + a.chunk);
    if (t >= T) done = true;
    const uint8_t* __restrict__ valid = a.valid + slot0;
    const uint8_t* __restrict__ reset = a.reset + slot0;
    const int64_t frame_bytes = (int64_t)a.feat_dim * (int64_t)sizeof(ElemT);
    const uint8_t* src = a.packed + slot0 * frame_bytes + (int64_t)first * (int64_t)(VEC ? 4 : 1) * (int64_t)sizeof(ElemT);
    float* dst = a.out + slot0 * (int64_t)a.feat_dim + (int64_t)first * (VEC ? 4 : 1);
    bool quad_on[QUADS];
#pragma unroll
    for (int g = 0; g < QUADS; ++g) quad_on[g] = !VEC || first + g * a.row_lanes < a.n_vec;

    bool owning = false;               // past the chunk's first boundary
    uint32_t before = (!done && t > 0) ? (valid[t - 1] != 0) : 0u;    // was the slot in front valid
    float h[EPL];
#pragma unroll
    for (int k = 0; k < EPL; ++k) h[k] = 0.0f;

    // Every pass moves each unfinished row forward (t grows, or the row starts owning), and a
    // row is finished at the latest when t reaches the block's end.
    while (__any(!done)) {
        if (!done) {
            const uint32_t in_range = T - t >= kScanBatch ? 0xffu : (1u << (T - t)) - 1u;
            const uint32_t vm = scan_flags8(valid, t, T);
            const uint32_t rm = scan_flags8(reset, t, T);
            // boundary: padding, a start flag, the block's first slot, or the slot after padding
            const uint32_t prev_valid = (vm << 1) | before;
            const uint32_t boundary = in_range & (~vm | rm | ~prev_valid | (t == 0 ? 1u : 0u));
            // bit u set iff slot t + u lies at or behind the chunk's end
            const int32_t to_end = t_end - t;
            const uint32_t behind = to_end >= kScanBatch ? 0u : (to_end <= 0 ? ~0u : ~0u << to_end);

            int advance;
            if (!owning) {
                const uint32_t mine = boundary & ~behind;
                if (mine) {
                    advance = __builtin_ctz(mine);
                    owning = true;
                } else {
                    advance = kScanBatch;
                    if (t + advance >= t_end) done = true;    // the chunk holds no boundary: nothing to own
                }
            } else {
                const uint32_t stop = boundary & behind;
                const int n = stop ? __builtin_ctz(stop) : min(kScanBatch, T - t);
                // all loads of the pass first, none of them conditional (slots behind the
                // block's end re-read its last slot and are not used)
                if (VEC) {
                    ScanQuad<ElemT> x[kScanBatch][QUADS];
#pragma unroll
                    for (int u = 0; u < kScanBatch; ++u) {
                        const uint8_t* frame = src + (int64_t)min(t + u, T - 1) * frame_bytes;
#pragma unroll
                        for (int g = 0; g < QUADS; ++g) {
                            const int64_t at = quad_on[g] ? (int64_t)g * a.row_lanes * 4 * (int64_t)sizeof(ElemT) : 0;
                            x[u][g].bits = __builtin_nontemporal_load(
                                reinterpret_cast<const typename ScanBits<sizeof(ElemT) * 4>::T*>(frame + at));
                        }
                    }
#pragma unroll
                    for (int u = 0; u < kScanBatch; ++u) {
                        const bool is_valid = (vm >> u) & 1u, starts = (boundary >> u) & 1u;
#pragma unroll
                        for (int g = 0; g < QUADS; ++g) {
                            float4v o;
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const float xv = is_valid ? ScanElem<ElemT>::get(x[u][g].e[j]) : 0.0f;
                                h[g * 4 + j] = (starts ? 0.0f : a.decay * h[g * 4 + j]) + xv;
                                o[j] = h[g * 4 + j];
                            }
                            if (u < n && quad_on[g])
                                __builtin_nontemporal_store(
                                    o, reinterpret_cast<float4v*>(dst + (int64_t)(t + u) * a.feat_dim +
                                                                  (int64_t)g * a.row_lanes * 4));
                        }
                    }
                } else {
                    ElemT x[kScanBatch];
#pragma unroll
                    for (int u = 0; u < kScanBatch; ++u)
                        x[u] = *reinterpret_cast<const ElemT*>(src + (int64_t)min(t + u, T - 1) * frame_bytes);
#pragma unroll
                    for (int u = 0; u < kScanBatch; ++u) {
                        const bool is_valid = (vm >> u) & 1u, starts = (boundary >> u) & 1u;
                        const float xv = is_valid ? ScanElem<ElemT>::get(x[u]) : 0.0f;
                        h[0] = (starts ? 0.0f : a.decay * h[0]) + xv;
                        if (u < n) __builtin_nontemporal_store(h[0], dst + (int64_t)(t + u) * a.feat_dim);
                    }
                }
                advance = n;
                if (stop || t + n >= T) done = true;
            }
            if (advance > 0) before = (vm >> (advance - 1)) & 1u;
            t += advance;
        }
    }
}

struct ScanPlan {
    int32_t epv, n_vec, row_lanes, feat_tiles, chunk, chunks_per_block;
    int64_t waves;
};

static ScanPlan scan_plan(int64_t num_blocks, int32_t t_blk, int64_t feat_dim, size_t elem)
{
    ScanPlan p{};
    // whole 16-byte pieces per frame: a lane takes 16 / elem elements as quads; else one element
    p.epv = (feat_dim * (int64_t)elem) % 16 == 0 ? (int32_t)(16 / elem) : 1;
    p.n_vec = p.epv > 1 ? (int32_t)(feat_dim / 4) : (int32_t)feat_dim;      // quads, or elements
    const int64_t per_lane = p.epv > 1 ? p.epv / 4 : 1;
    p.row_lanes = 1;
    while (p.row_lanes < kWave && p.row_lanes * per_lane < p.n_vec) p.row_lanes *= 2;
    p.feat_tiles = (int32_t)ceil_div(p.n_vec, p.row_lanes * per_lane);
    const int64_t rows_per_wave = kWave / p.row_lanes;
    // enough wavefronts to fill the chip several times over, chunks not shorter than 32 slots
    const int64_t want_waves = 16384;
    int64_t chunks = ceil_div(want_waves * rows_per_wave, num_blocks * p.feat_tiles);
    const int64_t most = t_blk / 32 > 1 ? t_blk / 32 : 1;
    if (chunks > most) chunks = most;
    if (chunks < 1) chunks = 1;
    p.chunk = (int32_t)round_up((size_t)ceil_div(t_blk, chunks), kScanBatch);
    p.chunks_per_block = (int32_t)ceil_div(t_blk, p.chunk);
    p.waves = ceil_div(num_blocks * p.chunks_per_block, rows_per_wave) * p.feat_tiles;
    return p;
}

template <typename ElemT>
static void scan_launch(const ScanArgs& a, const ScanPlan& p, hipStream_t stream)
{
    const dim3 grid((uint32_t)ceil_div(p.waves, kThreads / kWave)), block(kThreads);
    constexpr int kQuads = 4 / (int)sizeof(ElemT);           // quads in 16 input bytes
    if (p.epv > 1) hipLaunchKernelGGL((scan_kernel<ElemT, kQuads, true>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((scan_kernel<ElemT, 1, false>), grid, block, 0, stream, a);
}

}  // namespace bload

using namespace bload;

extern "C" bload_status bload_segment_scan(const void* d_packed, const uint8_t* d_reset,
                                           const uint8_t* d_valid, int64_t num_blocks, int32_t t_blk,
                                           int64_t feat_dim, bload_dtype dtype, float decay,
                                           float* d_out, void* hip_stream)
{
    if (num_blocks < 0 || t_blk < 1 || feat_dim < 1 || feat_dim > (1 << 28)) return BLOAD_EINVAL;
    if (dtype != BLOAD_U8 && dtype != BLOAD_F16 && dtype != BLOAD_F32) return BLOAD_EINVAL;
    if (num_blocks == 0) return BLOAD_OK;
    if (!d_packed || !d_reset || !d_valid || !d_out) return BLOAD_EINVAL;
    if (!aligned_to(d_packed, 16) || !aligned_to(d_out, 16)) return BLOAD_EALIGN;
    if (num_blocks * (int64_t)t_blk >= ((int64_t)1 << 40)) return BLOAD_EOVERFLOW;
    const size_t elem = dtype == BLOAD_U8 ? 1 : (dtype == BLOAD_F16 ? 2 : 4);
    const ScanPlan p = scan_plan(num_blocks, t_blk, feat_dim, elem);
    if (ceil_div(p.waves, kThreads / kWave) > 0x7fffffffLL) return BLOAD_EOVERFLOW;

    ScanArgs a{};
    a.packed = static_cast<const uint8_t*>(d_packed);
    a.reset = d_reset;
    a.valid = d_valid;
    a.out = d_out;
    a.items = num_blocks * p.chunks_per_block;
    a.t_blk = t_blk;
    a.feat_dim = (int32_t)feat_dim;
    a.chunk = p.chunk;
    a.chunks_per_block = p.chunks_per_block;
    a.row_lanes = p.row_lanes;
    a.feat_tiles = p.feat_tiles;
    a.n_vec = p.n_vec;
    a.decay = decay;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (dtype == BLOAD_U8) scan_launch<uint8_t>(a, p, stream);
    else if (dtype == BLOAD_F16) scan_launch<scan_half>(a, p, stream);
    else scan_launch<float>(a, p, stream);
    return launch_status();
}
