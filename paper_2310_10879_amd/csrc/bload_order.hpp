// The seeded order of the sequences: a keyed bijection of [0, N) shared by the
// planners (BLoad, Methods section: blocks are built from randomly sampled sequences;
// the paper names no generator).  Balanced Feistel network with cycle walking
// (Black & Rogaway 2002); round function MurmurHash3's 32-bit finaliser, round keys
// consecutive outputs of SplitMix64 started at the seed.
#pragma once

#include "bload_common.hpp"

namespace bload {

constexpr int kFeistelRounds = 6;

// What a planner reports to the host: a block at the start of its workspace.
struct PlanResult {
    int64_t num_blocks;
    int64_t total_frames;
    int32_t bad_length;
    int32_t pad_;
};

struct OrderKey {
    uint32_t key[kFeistelRounds];
    int32_t half_bits;                            // 0: identity (n_seq <= 1)
};

// SplitMix64 (Steele, Lea & Flood 2014): k-th output of the stream started at seed.
__host__ __device__ inline uint64_t splitmix64_at(uint64_t seed, uint64_t k)
{
    uint64_t z = seed + (k + 1) * 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

inline OrderKey make_order_key(int64_t n_seq, uint64_t seed)
{
    OrderKey k{};
    if (n_seq <= 1) return k;
    int width = 2;
    while (((uint64_t)1 << width) < (uint64_t)n_seq) width += 2;    // smallest even width
    k.half_bits = width / 2;
    for (int r = 0; r < kFeistelRounds; ++r) k.key[r] = (uint32_t)splitmix64_at(seed, (uint64_t)r);
    return k;
}

// MurmurHash3's 32-bit finaliser.
__device__ __forceinline__ uint32_t fmix32(uint32_t h)
{
    h ^= h >> 16;
    h *= 0x85EBCA6BU;
    h ^= h >> 13;
    h *= 0xC2B2AE35U;
    h ^= h >> 16;
    return h;
}

__device__ __forceinline__ uint32_t feistel(uint32_t x, const OrderKey& k)
{
    const uint32_t mask = (1u << k.half_bits) - 1u;
    uint32_t left = x >> k.half_bits, right = x & mask;
#pragma unroll
    for (int r = 0; r < kFeistelRounds; ++r) {
        const uint32_t t = left ^ (fmix32(right + k.key[r]) & mask);
        left = right;
        right = t;
    }
    return (left << k.half_bits) | right;
}

// Sequence at shuffled position p: walk the Feistel permutation of the
// enclosing power-of-four domain until it lands inside [0, n_seq).
__device__ __forceinline__ int32_t order_at(uint32_t p, uint32_t n_seq, const OrderKey& k)
{
    if (k.half_bits == 0) return (int32_t)p;
    uint32_t y = feistel(p, k);
    while (y >= n_seq) y = feistel(y, k);
    return (int32_t)y;
}

}  // namespace bload
