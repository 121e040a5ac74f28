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
// A row of lanes (16 input bytes per lane where the frame allows it, else one element)
// covers the features; a wavefront holds 64 / row-width rows, each on a chunk of its own.
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
    int32_t n_vec;                     // lane-sized pieces of a frame
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

// EPV elements of one lane.
template <typename ElemT, int EPV>
struct ScanLane {
    union { vec16 v; ElemT e[EPV]; } u;
    __device__ __forceinline__ void load(const uint8_t* p)
    {
        if (EPV > 1) u.v = load_stream(reinterpret_cast<const vec16*>(p));
        else u.e[0] = *reinterpret_cast<const ElemT*>(p);
    }
};

template <int EPV>
__device__ __forceinline__ void scan_store(float* dst, const float (&h)[EPV])
{
    if (EPV > 1) {
#pragma unroll
        for (int k = 0; k < EPV; k += 4) {
            float4v v = {h[k], h[k + 1], h[k + 2], h[k + 3]};
            __builtin_nontemporal_store(v, reinterpret_cast<float4v*>(dst + k));
        }
    } else {
        __builtin_nontemporal_store(h[0], dst);
    }
}

template <typename ElemT, int EPV>
__global__ __launch_bounds__(kThreads) void scan_kernel(ScanArgs a)
{
    const int lane = lane_id();
    const int rows_per_wave = kWave / a.row_lanes;
    const int64_t wave = (int64_t)blockIdx.x * (kThreads / kWave) + wave_id();
    const int32_t feat_tile = (int32_t)(wave % a.feat_tiles);
    const int64_t item = (wave / a.feat_tiles) * rows_per_wave + lane / a.row_lanes;
    const int32_t fv = feat_tile * a.row_lanes + (lane & (a.row_lanes - 1));

    bool done = item >= a.items || fv >= a.n_vec;
    const int64_t block = done ? 0 : item / a.chunks_per_block;
    const int32_t chunk = done ? 0 : (int32_t)(item - block * a.chunks_per_block);
    const int64_t slot0 = block * a.t_blk;                     // first slot of the block
    const int32_t T = a.t_blk;
    int32_t t = chunk * a.chunk;
    const int32_t t_end = min(T, t + a.chunk);
    if (t >= T) done = true;
    const int64_t frame_bytes = (int64_t)a.feat_dim * (int64_t)sizeof(ElemT);
    const uint8_t* src = a.packed + (int64_t)fv * (EPV * (int64_t)sizeof(ElemT));
    float* dst = a.out + (int64_t)fv * EPV;

    bool owning = false;               // past the chunk's first boundary
    float h[EPV];
#pragma unroll
    for (int k = 0; k < EPV; ++k) h[k] = 0.0f;

    // Every pass moves each unfinished row forward (t grows, or the row starts owning), and a
    // row is finished at the latest when t reaches the block's end.
    while (__any(!done)) {
        if (!done) {
            // flags of the next kScanBatch slots: bit u = slot t + u
            uint32_t in_range = 0, vm = 0, rm = 0;
            const uint32_t before = t > 0 ? (a.valid[slot0 + t - 1] != 0) : 0u;
#pragma unroll
            for (int u = 0; u < kScanBatch; ++u) {
                if (t + u < T) {
                    in_range |= 1u << u;
                    vm |= (uint32_t)(a.valid[slot0 + t + u] != 0) << u;
                    rm |= (uint32_t)(a.reset[slot0 + t + u] != 0) << u;
                }
            }
            // boundary: padding, a start flag, the block's first slot, or the slot after padding
            const uint32_t prev_valid = (vm << 1) | before;
            const uint32_t boundary = in_range & (~vm | rm | ~prev_valid | (t == 0 ? 1u : 0u));
            // bit u set iff slot t + u lies at or behind the chunk's end
            const int32_t to_end = t_end - t;
            const uint32_t behind = to_end >= kScanBatch ? 0u : (to_end <= 0 ? ~0u : ~0u << to_end);

            if (!owning) {
                const uint32_t mine = boundary & ~behind;
                if (mine) {
                    t += __builtin_ctz(mine);
                    owning = true;
                } else {
                    t += kScanBatch;
                    if (t >= t_end) done = true;       // the chunk holds no boundary: nothing to own
                }
            } else {
                const uint32_t stop = boundary & behind;
                const int n = stop ? __builtin_ctz(stop) : min(kScanBatch, T - t);
                ScanLane<ElemT, EPV> x[kScanBatch];
#pragma unroll
                for (int u = 0; u < kScanBatch; ++u)
                    if (u < n && ((vm >> u) & 1u)) x[u].load(src + (slot0 + t + u) * frame_bytes);
#pragma unroll
                for (int u = 0; u < kScanBatch; ++u) {
                    if (u < n) {
                        const bool is_valid = (vm >> u) & 1u, starts = (boundary >> u) & 1u;
#pragma unroll
                        for (int k = 0; k < EPV; ++k) {
                            const float xv = is_valid ? ScanElem<ElemT>::get(x[u].u.e[k]) : 0.0f;
                            h[k] = (starts ? 0.0f : a.decay * h[k]) + xv;
                        }
                        scan_store<EPV>(dst + (slot0 + t + u) * (int64_t)a.feat_dim, h);
                    }
                }
                t += n;
                if (stop || t >= T) done = true;
            }
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
    p.epv = (feat_dim * (int64_t)elem) % 16 == 0 ? (int32_t)(16 / elem) : 1;
    p.n_vec = (int32_t)(feat_dim / p.epv);
    p.row_lanes = 1;
    while (p.row_lanes < kWave && p.row_lanes < p.n_vec) p.row_lanes *= 2;
    p.feat_tiles = (int32_t)ceil_div(p.n_vec, p.row_lanes);
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
    constexpr int kVec = 16 / (int)sizeof(ElemT);
    if (p.epv > 1) hipLaunchKernelGGL((scan_kernel<ElemT, kVec>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((scan_kernel<ElemT, 1>), grid, block, 0, stream, a);
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
