/*
 * CPU oracle for the BLoad block packer -- TEST INFRASTRUCTURE, not product.
 *
 * A plain, single-threaded, deliberately slow statement of what the packer
 * computes, written from the paper (BLoad, arXiv 2310.10879) and used only to
 * check the HIP library and to time a CPU baseline.  It shares no code with
 * the HIP library and the library never calls it.
 *
 * What each function follows:
 *   - order:   Methods section (the sequences of a block are taken at random):
 *              the paper fixes no generator, so the random order is a keyed
 *              bijection of [0, N) (balanced Feistel network + cycle walking,
 *              Black & Rogaway 2002) whose round function is the MurmurHash3
 *              32-bit finaliser and whose round keys are consecutive outputs
 *              of SplitMix64 (Steele, Lea & Flood 2014) started at the seed.
 *   - plan:    Methods section: blocks of T_max frames built from whole
 *              sequences with T_i <= T_max, closed as near T_max as the
 *              running order allows (next-fit: a sequence that does not fit
 *              the open block closes it and opens the next one).
 *   - pack:    Methods section: the closed block is filled up with 0's; the
 *              table of where each new sequence starts inside its block is
 *              kept per sequence (offset) and per
 *              frame slot (reset flag, sequence id, frame index, valid).
 *   - reduce:  the consumer of that table (Methods section, resetting the
 *              carried state where a new sequence starts), in its simplest
 *              form: a per-sequence sum / mean over time.  Defined on the
 *              ragged source, so it does not depend on plan or pack.
 *   - padding: Problem Statement (padding every sample to the longest one)
 *              and Table 1 ("padding amount").
 *   - shard:   Problem Statement: equal sample counts for all data-parallel workers.
 *   - random fit: the sampler named in the caption of the pseudocode figure.
 *   - plan check: Methods section: a block is whole sequences laid one after
 *              another from its first slot, none beyond its end.
 *
 * Parity pins (tests/test_oracle_*.py): SplitMix64 known answers, invertible
 * finaliser, bijectivity and spread of the order; next-fit invariants, closed
 * forms and a brute-force optimum on tiny inputs; frame-exactly-once decoding
 * of a tagged payload; reductions of payloads with closed-form sums; the
 * paper's printed pad-to-longest count; the plan check accepts every plan the
 * planners make and is compared with a cell-by-cell simulation of the layout on
 * corrupted tables.  The identity of the permutation (which
 * bijection a seed gives) is a free choice of this implementation: "parity unpinned"
 * beyond those properties.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <stdlib.h>

/* ------------------------------------------------------------------ order */

/* SplitMix64 output function. */
static uint64_t oracle_mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* k-th output (k = 0, 1, ...) of the SplitMix64 stream whose state starts at
 * `seed`: the state advances by the golden-ratio increment before each output. */
uint64_t bload_oracle_splitmix64(uint64_t seed, uint64_t k)
{
    return oracle_mix64(seed + (k + 1) * 0x9E3779B97F4A7C15ULL);
}

/* MurmurHash3 32-bit finaliser. */
uint32_t bload_oracle_fmix32(uint32_t h)
{
    h ^= h >> 16;
    h *= 0x85EBCA6BU;
    h ^= h >> 13;
    h *= 0xC2B2AE35U;
    h ^= h >> 16;
    return h;
}

#define ORACLE_FEISTEL_ROUNDS 6

/* One pass of the 6-round balanced Feistel network over 2*half_bits bits. */
static uint32_t oracle_feistel(uint32_t x, int half_bits, const uint32_t* key)
{
    uint32_t mask = ((uint32_t)1 << half_bits) - 1U;
    uint32_t left = x >> half_bits;
    uint32_t right = x & mask;
    for (int r = 0; r < ORACLE_FEISTEL_ROUNDS; ++r) {
        uint32_t f = bload_oracle_fmix32(right + key[r]) & mask;
        uint32_t new_right = left ^ f;
        left = right;
        right = new_right;
    }
    return (left << half_bits) | right;
}

/* order[p] = index of the sequence at shuffled position p. */
void bload_oracle_order(int64_t n, uint64_t seed, int32_t* order)
{
    if (n <= 0) return;
    if (n == 1) { order[0] = 0; return; }
    /* smallest even bit width whose domain holds [0, n) */
    int width = 0;
    while (((uint64_t)1 << width) < (uint64_t)n) ++width;
    if (width < 2) width = 2;
    if (width & 1) ++width;
    int half_bits = width / 2;
    uint32_t key[ORACLE_FEISTEL_ROUNDS];
    for (int r = 0; r < ORACLE_FEISTEL_ROUNDS; ++r)
        key[r] = (uint32_t)bload_oracle_splitmix64(seed, (uint64_t)r);
    for (int64_t p = 0; p < n; ++p) {
        uint32_t y = oracle_feistel((uint32_t)p, half_bits, key);
        while ((uint64_t)y >= (uint64_t)n)          /* cycle walking */
            y = oracle_feistel(y, half_bits, key);
        order[p] = (int32_t)y;
    }
}

/* ------------------------------------------------------------------- plan */

/* Next-fit over the sequences taken in `order`.
 * Returns 0, or 2 if some length is < 1 or > t_blk (then outputs are undefined).
 * block_first has room for n+1 entries; entries [0 .. B] are written. */
int bload_oracle_plan(const int32_t* lengths, int64_t n, int32_t t_blk,
                      const int32_t* order,
                      int32_t* block_of_seq, int32_t* offset_of_seq,
                      int32_t* block_first,
                      int64_t* num_blocks, int64_t* total_frames)
{
    *num_blocks = 0;
    *total_frames = 0;
    for (int64_t i = 0; i < n; ++i)
        if (lengths[i] < 1 || lengths[i] > t_blk) return 2;
    if (n <= 0) return 0;
    int64_t b = 0;
    int64_t fill = 0;
    int64_t total = 0;
    block_first[0] = 0;
    for (int64_t p = 0; p < n; ++p) {
        int32_t i = order[p];
        int64_t len = lengths[i];
        if (fill + len > (int64_t)t_blk) {   /* does not fit: close, open next */
            b += 1;
            fill = 0;
            block_first[b] = (int32_t)p;
        }
        block_of_seq[i] = (int32_t)b;
        offset_of_seq[i] = (int32_t)fill;
        fill += len;
        total += len;
    }
    block_first[b + 1] = (int32_t)n;
    *num_blocks = b + 1;
    *total_frames = total;
    return 0;
}

/* ------------------------------------------------------------------- pack */

/* Blocks [block_lo, block_hi) of the packed tensor and of the four metadata
 * planes; every output pointer addresses the slab's first slot, i.e. slot
 * (block_lo, 0).  Padding: payload bytes 0, seq_id = frame_idx = -1,
 * reset = valid = 0. */
void bload_oracle_pack_blocks(const uint8_t* src, const int64_t* src_offsets,
                              const int32_t* lengths,
                              const int32_t* block_of_seq, const int32_t* offset_of_seq,
                              int64_t n, int32_t t_blk, int64_t frame_bytes,
                              int64_t block_lo, int64_t block_hi,
                              uint8_t* packed, int32_t* seq_id, int32_t* frame_idx,
                              uint8_t* reset, uint8_t* valid)
{
    int64_t slots = (block_hi - block_lo) * (int64_t)t_blk;
    if (slots <= 0) return;
    memset(packed, 0, (size_t)(slots * frame_bytes));
    for (int64_t s = 0; s < slots; ++s) {
        seq_id[s] = -1;
        frame_idx[s] = -1;
        reset[s] = 0;
        valid[s] = 0;
    }
    for (int64_t i = 0; i < n; ++i) {
        int64_t b = block_of_seq[i];
        if (b < block_lo || b >= block_hi) continue;
        for (int64_t t = 0; t < lengths[i]; ++t) {
            int64_t s = (b - block_lo) * (int64_t)t_blk + offset_of_seq[i] + t;
            memcpy(packed + s * frame_bytes,
                   src + (src_offsets[i] + t) * frame_bytes, (size_t)frame_bytes);
            seq_id[s] = (int32_t)i;
            frame_idx[s] = (int32_t)t;
            reset[s] = (uint8_t)(t == 0);
            valid[s] = 1;
        }
    }
}

/* ----------------------------------------------------------------- reduce */

/* IEEE binary16 bit pattern -> double (exact). */
double bload_oracle_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1F;
    int frac = h & 0x3FF;
    double v;
    if (expo == 0) {
        v = (double)frac * (1.0 / 16777216.0);              /* frac * 2^-24 */
    } else if (expo == 31) {
        if (frac == 0) v = 1.0 / 0.0; else v = 0.0 / 0.0;
    } else {
        v = 1.0 + (double)frac * (1.0 / 1024.0);
        int e = expo - 15;
        while (e > 0) { v *= 2.0; --e; }
        while (e < 0) { v *= 0.5; ++e; }
    }
    return sign ? -v : v;
}

/* dtype: 0 = u8, 1 = f16, 2 = f32, 3 = i32.   op: 0 = sum, 1 = mean.
 * out is float[n, feat_dim] for dtypes 0..2 (accumulated in double, rounded
 * once), int64[n, feat_dim] for i32 (exact; mean = sum / L truncated toward
 * zero is not defined here and is refused by returning 1). */
int bload_oracle_segment_reduce(const void* src, const int64_t* src_offsets,
                                const int32_t* lengths, int64_t n, int64_t feat_dim,
                                int dtype, int op, void* out)
{
    if (dtype == 3 && op != 0) return 1;
    if (n <= 0 || feat_dim <= 0) return 0;
    /* one accumulator per feature; frames are added in time order */
    double* acc = (double*)malloc((size_t)feat_dim * sizeof(double));
    int64_t* iacc = (int64_t*)malloc((size_t)feat_dim * sizeof(int64_t));
    if (!acc || !iacc) { free(acc); free(iacc); return 3; }
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t d = 0; d < feat_dim; ++d) { acc[d] = 0.0; iacc[d] = 0; }
        for (int64_t t = 0; t < lengths[i]; ++t) {
            int64_t base = (src_offsets[i] + t) * feat_dim;
            for (int64_t d = 0; d < feat_dim; ++d) {
                int64_t e = base + d;
                if (dtype == 0) acc[d] += (double)((const uint8_t*)src)[e];
                else if (dtype == 1) acc[d] += bload_oracle_half_to_double(((const uint16_t*)src)[e]);
                else if (dtype == 2) acc[d] += (double)((const float*)src)[e];
                else iacc[d] += (int64_t)((const int32_t*)src)[e];
            }
        }
        for (int64_t d = 0; d < feat_dim; ++d) {
            if (dtype == 3) {
                ((int64_t*)out)[i * feat_dim + d] = iacc[d];
            } else {
                double v = acc[d];
                if (op == 1) v /= (double)lengths[i];
                ((float*)out)[i * feat_dim + d] = (float)v;
            }
        }
    }
    free(acc);
    free(iacc);
    return 0;
}

/* ---------------------------------------------------------------- padding */

/* Padding counts, in frames:
 *   pad_longest = N * t_max - sum(L)        (every sample padded to t_max)
 *   pad_blocks  = num_blocks * t_blk - sum(L)  (block packing) */
void bload_oracle_padding(const int32_t* lengths, int64_t n, int64_t t_max,
                          int64_t num_blocks, int64_t t_blk,
                          int64_t* pad_longest, int64_t* pad_blocks)
{
    int64_t total = 0;
    for (int64_t i = 0; i < n; ++i) total += lengths[i];
    *pad_longest = n * t_max - total;
    *pad_blocks = num_blocks * t_blk - total;
}

/* ------------------------------------------------------------------ shard */

/* The share of data-parallel worker `rank` of `world` (Problem Statement: every
 * worker must get the same number of samples, or the gradient exchange stalls):
 * the blocks b with b mod world == rank, renumbered j = b / world, and, for the
 * workers that would otherwise fall one block short, one block of pure padding
 * at the end, so that every worker holds ceil(B / world) blocks.
 *   order_local[n]          visiting order of the worker's sequences, then -1
 *   block_of_seq_local[n]   local block j of sequence i, -1 if i is another worker's
 *   block_first_local[..]   ceil(B / world) + 1 entries
 * Returns the number of sequences of the worker. */
int64_t bload_oracle_plan_shard(const int32_t* order, const int32_t* block_of_seq,
                                const int32_t* block_first, int64_t n, int64_t num_blocks,
                                int32_t rank, int32_t world,
                                int32_t* order_local, int32_t* block_of_seq_local,
                                int32_t* block_first_local)
{
    int64_t blocks_local = (num_blocks + world - 1) / world;
    int64_t n_local = 0;
    for (int64_t i = 0; i < n; ++i) {
        order_local[i] = -1;
        block_of_seq_local[i] = -1;
    }
    for (int64_t j = 0; j < blocks_local; ++j) {
        int64_t b = j * world + rank;
        block_first_local[j] = (int32_t)n_local;
        if (b >= num_blocks) continue;                   /* the padding block */
        for (int64_t p = block_first[b]; p < block_first[b + 1]; ++p) {
            int32_t i = order[p];
            (void)block_of_seq;
            order_local[n_local++] = i;
            block_of_seq_local[i] = (int32_t)j;
        }
    }
    block_first_local[blocks_local] = (int32_t)n_local;
    return n_local;
}

/* ------------------------------------------------- reduce, from the blocks */

/* The same per-sequence sum / mean, but read the way the consumer of the start
 * table reads it (Methods section: reset the carried state where a new sequence
 * starts): walk every block in time, carry a running sum, and restart it at a
 * slot that is valid and (carries a start flag, or is the block's first slot, or
 * follows a padding slot); a padding slot or the end of the block closes the
 * running segment, whose result goes to row seq_id[first slot of the segment].
 * Defined for any flags, not only those a correct pack writes.
 * dtype / op / out as in bload_oracle_segment_reduce; rows that no segment names
 * are left untouched.  Returns the number of segments, or -1 for i32 mean. */
int64_t bload_oracle_segment_reduce_packed(const void* packed, const int32_t* seq_id,
                                           const uint8_t* reset, const uint8_t* valid,
                                           int64_t num_blocks, int32_t t_blk, int64_t feat_dim,
                                           int dtype, int op, int64_t n_seq, void* out)
{
    if (dtype == 3 && op != 0) return -1;
    int64_t segments = 0;
    double* acc = (double*)malloc((size_t)(feat_dim > 0 ? feat_dim : 1) * sizeof(double));
    int64_t* iacc = (int64_t*)malloc((size_t)(feat_dim > 0 ? feat_dim : 1) * sizeof(int64_t));
    if (!acc || !iacc) { free(acc); free(iacc); return -2; }
    for (int64_t b = 0; b < num_blocks; ++b) {
        int open = 0;
        int64_t count = 0;
        int32_t row = -1;
        for (int64_t t = 0; t <= t_blk; ++t) {
            int64_t s = b * (int64_t)t_blk + t;
            int is_valid = t < t_blk && valid[s] != 0;
            int starts = is_valid && (reset[s] != 0 || t == 0 || valid[s - 1] == 0);
            if (open && (!is_valid || starts)) {           /* the running segment ends before s */
                if (row >= 0 && row < n_seq) {
                    for (int64_t d = 0; d < feat_dim; ++d) {
                        if (dtype == 3) {
                            ((int64_t*)out)[row * feat_dim + d] = iacc[d];
                        } else {
                            double v = acc[d];
                            if (op == 1) v /= (double)count;
                            ((float*)out)[row * feat_dim + d] = (float)v;
                        }
                    }
                }
                segments += 1;
                open = 0;
            }
            if (!is_valid) continue;
            if (starts) {
                open = 1;
                count = 0;
                row = seq_id[s];
                for (int64_t d = 0; d < feat_dim; ++d) { acc[d] = 0.0; iacc[d] = 0; }
            }
            count += 1;
            for (int64_t d = 0; d < feat_dim; ++d) {
                int64_t e = s * feat_dim + d;
                if (dtype == 0) acc[d] += (double)((const uint8_t*)packed)[e];
                else if (dtype == 1) acc[d] += bload_oracle_half_to_double(((const uint16_t*)packed)[e]);
                else if (dtype == 2) acc[d] += (double)((const float*)packed)[e];
                else iacc[d] += (int64_t)((const int32_t*)packed)[e];
            }
        }
    }
    free(acc);
    free(iacc);
    return segments;
}

/* ------------------------------------------------------------- random fit */

/* The block builder of the paper's pseudocode figure, whose caption fixes the
 * sampler: it returns a random entry of the length dictionary L_dict among those
 * whose sequence is no longer than the frames remaining in the open block.  A block
 * is closed when no remaining sequence fits (or none remains).
 *
 * What the caption leaves open, as read here:
 *   - "random entry": every remaining sequence that fits is equally likely.  With m
 *     such sequences the draw is k = floor(u * m / 2^64) for a 64-bit uniform u, and
 *     the k-th of them counted through L_dict by ascending length is taken.
 *   - u for the p-th placement (p = 0, 1, ...) is output number 6 + p of the SplitMix64
 *     stream started at the seed (outputs 0..5 key the seeded order).
 *   - L_dict[l] lists the sequences of length l in the seeded order; a draw that lands
 *     in L_dict[l] removes the last remaining entry of that list.  Since the seeded
 *     order is itself a random permutation this picks uniformly inside the class.
 *
 * `seeded` is the seeded order (bload_oracle_order).  Outputs as in bload_oracle_plan:
 * order[p] is the p-th sequence placed.  Returns 0, or 2 on a length outside [1, t_blk]. */
int bload_oracle_plan_random_fit(const int32_t* lengths, int64_t n, int32_t t_blk, uint64_t seed,
                                 const int32_t* seeded, int32_t* order, int32_t* block_of_seq,
                                 int32_t* offset_of_seq, int32_t* block_first,
                                 int64_t* num_blocks, int64_t* total_frames)
{
    *num_blocks = 0;
    *total_frames = 0;
    for (int64_t i = 0; i < n; ++i)
        if (lengths[i] < 1 || lengths[i] > t_blk) return 2;
    if (n <= 0) return 0;

    /* L_dict: entry[first[l] .. first[l] + left[l]) are the remaining sequences of length l */
    int64_t* left = calloc((size_t)t_blk + 2, sizeof(int64_t));
    int64_t* first = calloc((size_t)t_blk + 2, sizeof(int64_t));
    int32_t* entry = malloc((size_t)n * sizeof(int32_t));
    int64_t total = 0;
    for (int64_t i = 0; i < n; ++i) { left[lengths[i]] += 1; total += lengths[i]; }
    for (int64_t l = 1; l <= t_blk; ++l) first[l + 1] = first[l] + left[l];
    for (int64_t l = 0; l <= t_blk; ++l) left[l] = 0;
    for (int64_t p = 0; p < n; ++p) {
        int32_t i = seeded[p];
        int64_t l = lengths[i];
        entry[first[l] + left[l]] = i;
        left[l] += 1;
    }

    int64_t placed = 0;
    int64_t b = 0;
    while (placed < n) {
        int64_t remaining_frames = t_blk;
        block_first[b] = (int32_t)placed;
        for (;;) {
            uint64_t m = 0;                               /* sequences that still fit */
            for (int64_t l = 1; l <= remaining_frames; ++l) m += (uint64_t)left[l];
            if (m == 0) break;
            uint64_t u = bload_oracle_splitmix64(seed, (uint64_t)(6 + placed));
            uint64_t k = (uint64_t)(((unsigned __int128)u * m) >> 64);
            int64_t l = 1;
            while (k >= (uint64_t)left[l]) { k -= (uint64_t)left[l]; ++l; }
            left[l] -= 1;
            int32_t i = entry[first[l] + left[l]];
            order[placed] = i;
            block_of_seq[i] = (int32_t)b;
            offset_of_seq[i] = (int32_t)(t_blk - remaining_frames);
            remaining_frames -= l;
            placed += 1;
        }
        b += 1;
    }
    block_first[b] = (int32_t)n;
    *num_blocks = b;
    *total_frames = total;
    free(left);
    free(first);
    free(entry);
    return 0;
}

/* -------------------------------------------------------- chunk sampling */

/* The second baseline of the Problem Statement (and Table 1's "sampling" column,
 * rows "padding amount" = 0 and "# frames deleted"): every sequence is cut into
 * pieces of t_chunk frames and each piece is a sample of its own; nothing is padded,
 * so whatever does not fill a piece is deleted.
 *   samples = sum over sequences of floor(L / t_chunk)
 *   deleted = sum over sequences of L mod t_chunk */
void bload_oracle_chunk_sampling(const int32_t* lengths, int64_t n, int64_t t_chunk,
                                 int64_t* samples, int64_t* deleted)
{
    int64_t s = 0, d = 0;
    for (int64_t i = 0; i < n; ++i) {
        int64_t whole = 0;
        int64_t left = lengths[i];
        while (left >= t_chunk) { left -= t_chunk; whole += 1; }
        s += whole;
        d += left;
    }
    *samples = s;
    *deleted = d;
}

/* ------------------------------------------------------- recurrent consumer */

static double oracle_element(const void* p, int dtype, int64_t e)
{
    if (dtype == 0) return (double)((const uint8_t*)p)[e];
    if (dtype == 1) return bload_oracle_half_to_double(((const uint16_t*)p)[e]);
    return (double)((const float*)p)[e];
}

/* The use the start table is made for (Methods section; the figure of the DDS model: what
 * frame n-1 produced is part of the input of frame n, and the table says where that carried
 * state belongs to another sequence and must be dropped).  The smallest consumer with such
 * feedback is a first-order linear recurrence per feature,
 *     h_0 = x_0,   h_t = decay * h_{t-1} + x_t      (t = 1 .. L-1, inside one sequence),
 * defined here on the ragged source, so it knows nothing of blocks, plans or flags.
 * out: float[sum(L), feat_dim] in source order, each value computed in double and rounded
 * once.  scale (may be NULL): the same recurrence on |x| with |decay|, the magnitude a
 * rounding-error bound is stated against.  dtype: 0 u8, 1 f16, 2 f32.  Returns 0, 1 on
 * another dtype. */
int bload_oracle_segment_scan(const void* src, const int64_t* src_offsets, const int32_t* lengths,
                              int64_t n, int64_t feat_dim, int dtype, double decay, float* out,
                              float* scale)
{
    if (dtype < 0 || dtype > 2) return 1;
    double mag = decay < 0 ? -decay : decay;
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t d = 0; d < feat_dim; ++d) {
            double h = 0.0, s = 0.0;
            for (int64_t t = 0; t < lengths[i]; ++t) {
                int64_t e = (src_offsets[i] + t) * feat_dim + d;
                double x = oracle_element(src, dtype, e);
                if (t == 0) { h = x; s = x < 0 ? -x : x; }
                else { h = decay * h + x; s = mag * s + (x < 0 ? -x : x); }
                out[e] = (float)h;
                if (scale) scale[e] = (float)s;
            }
        }
    }
    return 0;
}

/* The same recurrence read from the packed blocks through their flags (any flags): the
 * state is dropped at a valid slot that carries a start flag, is a block's first slot or
 * follows an invalid slot; an invalid slot yields 0.  out, scale: float[B, t_blk, feat_dim]. */
int bload_oracle_segment_scan_packed(const void* packed, const uint8_t* reset, const uint8_t* valid,
                                     int64_t num_blocks, int32_t t_blk, int64_t feat_dim, int dtype,
                                     double decay, float* out, float* scale)
{
    if (dtype < 0 || dtype > 2) return 1;
    double mag = decay < 0 ? -decay : decay;
    for (int64_t b = 0; b < num_blocks; ++b) {
        for (int64_t d = 0; d < feat_dim; ++d) {
            double h = 0.0, s = 0.0;
            for (int64_t t = 0; t < t_blk; ++t) {
                int64_t slot = b * (int64_t)t_blk + t;
                int64_t e = slot * feat_dim + d;
                if (!valid[slot]) {
                    out[e] = 0.0f;
                    if (scale) scale[e] = 0.0f;
                    continue;
                }
                int starts = reset[slot] != 0 || t == 0 || valid[slot - 1] == 0;
                double x = oracle_element(packed, dtype, e);
                if (starts) { h = x; s = x < 0 ? -x : x; }
                else { h = decay * h + x; s = mag * s + (x < 0 ? -x : x); }
                out[e] = (float)h;
                if (scale) scale[e] = (float)s;
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------- plan check */

/* Do the tables describe blocks made of whole sequences laid one after another
 * (Methods section)?  Index k is tested as a block (k < num_blocks) and as a
 * shuffled position (k < block_first[num_blocks]); the smallest k at which a
 * rule fails is returned, -1 if none does.
 *   block k:     0 <= block_first[k] <= block_first[k+1] <= n, block_first[0] = 0
 *   position k:  i = order[k] is a sequence; 1 <= L_i; it starts at slot
 *                offset_of_seq[i] >= 0 of block block_of_seq[i] and ends at or
 *                before slot t_blk; k lies in that block's range of positions;
 *                the block's first sequence starts at slot 0, every other one
 *                where the sequence before it ends; its source frames
 *                [src_offsets[i], src_offsets[i] + L_i) lie inside the source and
 *                src_offsets[i+1] = src_offsets[i] + L_i. */
int64_t bload_oracle_plan_check(const int64_t* src_offsets, const int32_t* lengths,
                                const int32_t* order, const int32_t* block_of_seq,
                                const int32_t* offset_of_seq, const int32_t* block_first,
                                int64_t n, int64_t num_blocks, int32_t t_blk, int64_t total_frames)
{
    if (n <= 0 || num_blocks <= 0) return -1;
    int64_t listed = block_first[num_blocks];
    if (listed < 0) listed = 0;
    if (listed > n) listed = n;
    int64_t last = num_blocks > listed ? num_blocks : listed;
    for (int64_t k = 0; k < last; ++k) {
        if (k < num_blocks) {
            int64_t lo = block_first[k], hi = block_first[k + 1];
            if (lo < 0 || hi < lo || hi > n) return k;
            if (k == 0 && lo != 0) return k;
        }
        if (k < listed) {
            int64_t i = order[k];
            if (i < 0 || i >= n) return k;
            int64_t len = lengths[i], off = offset_of_seq[i], b = block_of_seq[i];
            if (len < 1 || off < 0 || off + len > t_blk) return k;
            if (src_offsets[i] < 0 || src_offsets[i] + len > total_frames) return k;
            if (src_offsets[i + 1] != src_offsets[i] + len) return k;
            if (b < 0 || b >= num_blocks) return k;
            if (block_first[b] < 0 || k < block_first[b] || k >= block_first[b + 1]) return k;
            if (k == block_first[b]) {
                if (off != 0) return k;
            } else {
                int64_t before = order[k - 1];
                if (before < 0 || before >= n) return k;
                if (off != (int64_t)offset_of_seq[before] + (int64_t)lengths[before]) return k;
            }
        }
    }
    return -1;
}
