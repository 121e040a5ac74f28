/*
 * bload.h -- C ABI of the BLoad block packer for MI355X (gfx950).
 *
 * BLoad (arXiv 2310.10879) trains on N sequences S_i of H x W x T_i frames
 * with varying T_i (Problem Statement) by concatenating randomly ordered whole
 * sequences into blocks of a fixed length T_blk = T_max, padding each block's
 * tail with 0's, and keeping a table of where each sequence starts inside its
 * block so that a recurrent consumer can reset its carried state there
 * (Methods).  This library is that packer, on the GPU:
 *
 *   bload_plan            order the sequences by seed and assign them to blocks
 *   bload_pack            gather the frames into [num_blocks, T_blk, frame] and
 *                         write the per-slot form of the start table
 *   bload_segment_reduce  per-sequence sum / mean over the packed blocks, using
 *                         only the packed tensor and that per-slot table
 * and, around that path,
 *   bload_plan_random_fit   the plan built with the sampler of the paper's pseudocode
 *   bload_plan_shard        one data-parallel worker's share of a plan
 *   bload_segment_scan      a recurrent consumer that drops its state at sequence starts
 *   bload_strategy_counts   padding / frames deleted under the strategies the paper compares
 *   bload_pack_check        are these tables a plan bload_pack can take
 *   bload_pack_noalloc      bload_pack with its scratch in a fixed array of the library
 *
 * Conventions
 *   - Pointers named d_* are DEVICE pointers (hipMalloc-style memory of the
 *     current device), h_* are HOST pointers.  The caller owns every buffer;
 *     the library allocates nothing and keeps no state between calls (the one
 *     exception, a fixed scratch array, is bload_pack_noalloc's and is described
 *     there).
 *   - A frame is an opaque record of `frame_bytes` bytes (H*W*C*sizeof(elem));
 *     H and W are the same for all sequences of one call.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     bload_pack, bload_segment_reduce and bload_segment_scan only enqueue work
 *     on it (no synchronisation, no allocation: they can be recorded into a HIP
 *     graph); the planners and bload_strategy_counts enqueue, then wait for the
 *     stream, because they return counts to the host.
 *   - Every function returns a bload_status; nothing is thrown.  On any
 *     status other than BLOAD_OK the contents of the output buffers are
 *     unspecified (but nothing outside them is ever written).
 *   - Sizes: 0 <= n_seq <= BLOAD_MAX_SEQ, 1 <= t_blk, 1 <= L_i <= t_blk,
 *     num_blocks * t_blk < 2^40 slots.
 */
#ifndef BLOAD_H
#define BLOAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BLOAD_MAX_SEQ ((int64_t)1 << 27)

typedef enum {
    BLOAD_OK = 0,
    BLOAD_EINVAL = 1,      /* null pointer, negative size, t_blk < 1, frame_bytes < 1,
                              unknown dtype / op, or an unsupported dtype-op pair */
    BLOAD_ELENGTH = 2,     /* some L_i < 1 or L_i > t_blk (the method needs T_i <= T_max) */
    BLOAD_EWORKSPACE = 3,  /* workspace smaller than the *_workspace_bytes() answer */
    BLOAD_EALIGN = 4,      /* a payload / workspace base is not 16-byte aligned (32-byte for
                              bload_pack's workspace), or an int32 / int64 table is not
                              naturally aligned */
    BLOAD_EOVERFLOW = 5,   /* n_seq or num_blocks * t_blk beyond the supported range */
    BLOAD_EHIP = 6         /* a HIP runtime call failed (bload_last_hip_error() says which) */
} bload_status;

typedef enum { BLOAD_U8 = 0, BLOAD_F16 = 1, BLOAD_F32 = 2, BLOAD_I32 = 3 } bload_dtype;
typedef enum { BLOAD_SUM = 0, BLOAD_MEAN = 1 } bload_op;

/* Human-readable name of a status (static storage, never NULL). */
const char* bload_status_string(bload_status status);

/* hipError_t (as int) of the most recent failing HIP call made by this library
 * on the calling thread, 0 if none. */
int bload_last_hip_error(void);

/* ------------------------------------------------------------------ plan --
 * Methods section: blocks of T_max frames are put together from whole sequences,
 * none longer than T_max, taken in random order; each block is closed as near
 * T_max as the visiting order allows; a table keeps where every sequence starts.
 *
 * order:  a permutation of [0, n_seq) fixed by `seed` alone: position p holds
 *         the sequence walk(p), where walk applies a 6-round balanced Feistel
 *         network over the smallest even bit width w >= 2 with 2^w >= n_seq
 *         (round function: MurmurHash3's 32-bit finaliser of right-half +
 *         key_r, masked to w/2 bits; key_r = low 32 bits of the r-th output of
 *         SplitMix64 started at `seed`) and re-applies it until the value is
 *         below n_seq.  n_seq <= 1 gives the identity.
 * assign: next-fit over that order: a sequence goes into the open block if
 *         fill + L <= t_blk, otherwise the block is closed (its tail is
 *         padding) and the sequence opens the next one.
 *
 * d_lengths        in   int32[n_seq]   L_i, in original sequence order
 * d_order          out  int32[n_seq]   order[p] = sequence at shuffled position p
 * d_block_of_seq   out  int32[n_seq]   block of sequence i      (original index)
 * d_offset_of_seq  out  int32[n_seq]   first slot of sequence i inside its block
 *                                      (the paper's start table, per sequence)
 * d_block_first    out  int32[n_seq+1] capacity; entries [0 .. B] are written:
 *                                      first shuffled position of block b, [B] = n_seq
 * h_num_blocks     out  host int64     B
 * h_total_frames   out  host int64     sum of L_i
 * d_workspace           device scratch of >= bload_plan_workspace_bytes(n_seq)
 *                       bytes, 16-byte aligned; contents meaningless afterwards
 *
 * Lengths are checked on the device; a bad one gives BLOAD_ELENGTH.  n_seq = 0
 * gives B = 0, BLOAD_OK, and writes nothing to the device.  Synchronises the
 * stream before returning.  The library keeps 64 bytes of pinned host memory per
 * calling thread (taken at that thread's first call, never freed) into which the
 * device writes B and the frame total; bload_plan_shard uses the same bytes.
 */
size_t bload_plan_workspace_bytes(int64_t n_seq);

bload_status bload_plan(const int32_t* d_lengths, int64_t n_seq, int32_t t_blk, uint64_t seed,
                        int32_t* d_order, int32_t* d_block_of_seq, int32_t* d_offset_of_seq,
                        int32_t* d_block_first,
                        int64_t* h_num_blocks, int64_t* h_total_frames,
                        void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------- plan, random fit --
 * Caption of the pseudocode figure: the block builder asks a sampler for a random
 * entry of the length dictionary L_dict among the sequences no longer than the
 * frames remaining in the open block; a block is closed when none fits.  The
 * reading implemented here:
 *   - every remaining sequence that fits is equally likely: with m of them the
 *     draw is k = floor(u * m / 2^64), u the output number 6 + p of the seed's
 *     SplitMix64 stream for the p-th placement, and the k-th is counted through
 *     L_dict by ascending length;
 *   - L_dict[l] lists the sequences of length l in the seeded order (the order
 *     bload_plan visits them in); a draw landing in L_dict[l] takes its last
 *     remaining entry.
 * Arguments, outputs, workspace rules and error codes are those of bload_plan
 * (d_order[p] is the p-th sequence placed); bload_pack, bload_plan_shard and
 * bload_segment_reduce take the result like a next-fit plan.  Additionally
 * BLOAD_EOVERFLOW when t_blk > BLOAD_RANDOM_FIT_MAX_T_BLK (the per-length counts
 * are kept in on-chip memory).  The draws form a dependent chain that one
 * wavefront walks: the cost grows linearly with n_seq.
 * Synchronises the stream before returning.
 */
#define BLOAD_RANDOM_FIT_MAX_T_BLK 8192

size_t bload_plan_random_fit_workspace_bytes(int64_t n_seq);

bload_status bload_plan_random_fit(const int32_t* d_lengths, int64_t n_seq, int32_t t_blk,
                                   uint64_t seed, int32_t* d_order, int32_t* d_block_of_seq,
                                   int32_t* d_offset_of_seq, int32_t* d_block_first,
                                   int64_t* h_num_blocks, int64_t* h_total_frames,
                                   void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------ plan shard --
 * Problem Statement: under data-parallel training every worker must receive the
 * same number of samples per epoch, otherwise the gradient exchange stalls; the
 * blocks are the samples.  This call derives worker `rank`'s share of a plan:
 * the blocks b with b mod world == rank, renumbered j = b / world, plus one
 * block of pure padding at the end for the workers that would otherwise hold
 * one block less, so that every worker has ceil(B / world) blocks.  The outputs
 * are a plan in the worker's own numbering; bload_pack and bload_segment_reduce
 * take them like the tables of bload_plan (with n_seq unchanged, the worker's
 * block count, and the same d_lengths / d_offset_of_seq / d_src / d_src_offsets).
 *
 * d_order, d_block_of_seq, d_block_first   in   as produced by bload_plan
 * d_order_local          out  int32[n_seq]  the worker's sequences in visiting
 *                                           order, then -1 (= no sequence)
 * d_block_of_seq_local   out  int32[n_seq]  local block of sequence i, -1 when i
 *                                           belongs to another worker
 * d_block_first_local    out  int32[ceil(B / world) + 1]
 * h_num_blocks_local     out  host int64    ceil(B / world)
 * h_n_seq_local          out  host int64    number of sequences of the worker
 * d_workspace                 >= 16 bytes, 16-byte aligned
 *
 * Synchronises the stream before returning (it reports the worker's counts).
 */
bload_status bload_plan_shard(const int32_t* d_order, const int32_t* d_block_of_seq,
                              const int32_t* d_block_first, int64_t n_seq, int64_t num_blocks,
                              int32_t rank, int32_t world,
                              int32_t* d_order_local, int32_t* d_block_of_seq_local,
                              int32_t* d_block_first_local,
                              int64_t* h_num_blocks_local, int64_t* h_n_seq_local,
                              void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------ pack --
 * Methods section: the sequences of a block are laid one after another and the
 * rest of the block is filled with 0's; the start table says where each new
 * sequence begins.
 *
 * d_src          in   bytes[total_frames * frame_bytes]: the ragged source, the
 *                     frames of sequence i stored contiguously from frame
 *                     d_src_offsets[i]; any byte alignment (fastest when it is
 *                     16-byte aligned and frame_bytes is a multiple of 16)
 * d_src_offsets  in   int64[n_seq+1]  first source frame of each sequence;
 *                     src_offsets[i+1] - src_offsets[i] must equal L_i (not checked)
 * d_lengths, d_order, d_block_of_seq, d_offset_of_seq, d_block_first
 *                in   as produced by bload_plan for the same lengths (or a worker's
 *                     share of them from bload_plan_shard; an entry of d_order that
 *                     is not in [0, n_seq) ends the list of sequences)
 * num_blocks     in   B as returned by bload_plan
 * d_packed       out  bytes[B, t_blk, frame_bytes]; slot
 *                     (b, offset_of_seq[i] + t) receives frame t of sequence i,
 *                     every other byte is 0
 * d_seq_id       out  int32[B, t_blk]  original sequence index, -1 on padding
 * d_frame_idx    out  int32[B, t_blk]  frame number inside its sequence, -1 on padding
 * d_reset        out  uint8[B, t_blk]  1 on the first frame of a sequence, else 0
 * d_valid        out  uint8[B, t_blk]  1 on a real frame, 0 on padding
 *                     (all five outputs 16-byte aligned)
 *
 * d_workspace         device scratch of >= bload_pack_workspace_bytes(...) bytes,
 *                     32-byte aligned: one 32-byte record per sequence (where it
 *                     lands, where it comes from) and one int32 per destination
 *                     tile -- 4 KiB of packed tensor (plus, from 2^21 slots on, one
 *                     per 1024 slots for the pass that writes the start table) or
 *                     1024 slots -- saying where the tile starts in the shuffled
 *                     order; contents meaningless afterwards
 *
 * Every byte of the five outputs is written exactly once (no prior memset is
 * needed), and nothing outside them whatever the tables hold.  The tables are
 * trusted otherwise: tables that are not a plan give a meaningless result, and
 * source offsets outside the source are read; bload_pack_check tells.
 * Asynchronous on `hip_stream`.  n_seq = 0 / num_blocks = 0: no-op.
 */
/* Which of its two kernels bload_pack launches for these sizes: 4096 when the packed
 * tensor is cut into tiles of 4096 bytes (pack_wide_kernel), 0 when it is cut into
 * tiles of 1024 slots (pack_narrow_kernel), also for sizes bload_pack refuses.
 * src_aligned_16: whether d_src is 16-byte aligned.  For profiling and reports. */
int32_t bload_pack_tile_bytes(int64_t n_seq, int64_t num_blocks, int32_t t_blk, int64_t frame_bytes,
                              int32_t src_aligned_16);

size_t bload_pack_workspace_bytes(int64_t n_seq, int64_t num_blocks, int32_t t_blk, int64_t frame_bytes);

bload_status bload_pack(const void* d_src, const int64_t* d_src_offsets, const int32_t* d_lengths,
                        const int32_t* d_order, const int32_t* d_block_of_seq,
                        const int32_t* d_offset_of_seq, const int32_t* d_block_first,
                        int64_t n_seq, int64_t num_blocks, int32_t t_blk, int64_t frame_bytes,
                        void* d_packed, int32_t* d_seq_id, int32_t* d_frame_idx,
                        uint8_t* d_reset, uint8_t* d_valid,
                        void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): bload_pack without the
 * workspace argument.  Its scratch -- the same per-sequence records and per-tile
 * entries -- lives in a fixed array of 16 MiB of device memory that belongs to the
 * loaded library; every GPU on which this entry point is used holds one until the
 * process ends.  Limits: n_seq <= BLOAD_PACK_NOALLOC_MAX_SEQ and at most
 * BLOAD_PACK_NOALLOC_MAX_TILES - 4 tile entries (a tile is 4 KiB of packed tensor
 * when bload_pack_tile_bytes() says 4096, with one more entry per 1024 slots from
 * 2^21 slots on, else 1024 slots: just under 8 GiB of packed tensor, or 2^31
 * slots); anything larger is refused with BLOAD_EOVERFLOW before anything is
 * launched.  All other arguments, checks and results are those of bload_pack.
 * The call allocates and frees nothing and does not synchronise.  Nothing in the
 * array has to be cleared between calls (each call rewrites the part it reads),
 * but all calls on one GPU share it: two such calls must not overlap in time on
 * the same GPU (calls on one stream never do; calls on different streams, or from
 * different threads, need an order between them).
 */
#define BLOAD_PACK_NOALLOC_MAX_SEQ ((int64_t)1 << 18)
#define BLOAD_PACK_NOALLOC_MAX_TILES ((int64_t)1 << 21)

bload_status bload_pack_noalloc(const void* d_src, const int64_t* d_src_offsets, const int32_t* d_lengths,
                                const int32_t* d_order, const int32_t* d_block_of_seq,
                                const int32_t* d_offset_of_seq, const int32_t* d_block_first,
                                int64_t n_seq, int64_t num_blocks, int32_t t_blk, int64_t frame_bytes,
                                void* d_packed, int32_t* d_seq_id, int32_t* d_frame_idx,
                                uint8_t* d_reset, uint8_t* d_valid, void* hip_stream);

/* Methods section: whole sequences, one after another from the block's first
 * slot, none split, none beyond the block's end.  This call verifies that the
 * tables handed to bload_pack describe such a layout, without packing anything:
 *   - block_first[0 .. num_blocks] is non-decreasing, starts at 0 and ends at
 *     P <= n_seq; every position p < P holds a sequence index in [0, n_seq);
 *   - the sequence at position p lies in the block whose range contains p, at
 *     offset 0 if it is the block's first and right behind its predecessor
 *     otherwise, and ends at or before slot t_blk;
 *   - 1 <= L_i, and the source range [src_offsets[i], src_offsets[i] + L_i) lies
 *     inside [0, total_frames) and src_offsets[i+1] - src_offsets[i] = L_i,
 * for every sequence listed.  (Together these make the listed sequences distinct.)
 * BLOAD_OK if so, BLOAD_EINVAL if not; *h_first_bad (may be NULL) receives the
 * smallest shuffled position or block at which a rule fails, -1 if none.
 * d_workspace: >= 16 bytes, 16-byte aligned.  Synchronises the stream.
 */
bload_status bload_pack_check(const int64_t* d_src_offsets, const int32_t* d_lengths,
                              const int32_t* d_order, const int32_t* d_block_of_seq,
                              const int32_t* d_offset_of_seq, const int32_t* d_block_first,
                              int64_t n_seq, int64_t num_blocks, int32_t t_blk, int64_t total_frames,
                              int64_t* h_first_bad, void* d_workspace, size_t workspace_bytes,
                              void* hip_stream);

/* -------------------------------------------------------- segment reduce --
 * Methods section: knowing where a new sequence starts lets the consumer drop
 * what it carried from the previous frame.  The simplest such consumer: a
 * running sum over time that is restarted at every start flag and never
 * crosses a block boundary.  It receives no plan tables: segments are found
 * from d_reset / d_valid alone, d_seq_id only names the output row.
 *
 * d_packed   in   [B, t_blk, feat_dim] of `dtype`, 16-byte aligned
 * d_seq_id   in   int32[B, t_blk];  d_reset, d_valid in uint8[B, t_blk]
 * d_out      out  [n_seq, feat_dim]: float32 for U8 / F16 / F32 inputs (float32
 *                 accumulation over chunks of time, chunks added in time order),
 *                 int64 for I32 (exact).  MEAN divides by the segment's frame
 *                 count; I32 supports SUM only.  A segment's row is d_seq_id at
 *                 its first slot: row i is written iff some segment starts with
 *                 seq_id i; ids outside [0, n_seq) are skipped.  float32 sums are
 *                 compensated: whatever the length of a sequence, the result is
 *                 within a few units of float32 roundoff of sum |x| (exact for U8
 *                 while the sum stays below 2^24).
 * d_workspace     device scratch of >= bload_segment_reduce_workspace_bytes(...)
 *                 bytes, 16-byte aligned.
 *
 * Asynchronous on `hip_stream`; same inputs give bit-identical outputs.
 */
size_t bload_segment_reduce_workspace_bytes(int64_t num_blocks, int32_t t_blk, int64_t feat_dim,
                                            bload_dtype dtype);

bload_status bload_segment_reduce(const void* d_packed, const int32_t* d_seq_id,
                                  const uint8_t* d_reset, const uint8_t* d_valid,
                                  int64_t num_blocks, int32_t t_blk, int64_t feat_dim,
                                  bload_dtype dtype, bload_op op, int64_t n_seq, void* d_out,
                                  void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* ---------------------------------------------------------- segment scan --
 * Methods section and the figure of the DDS model: the network feeds what it
 * produced for frame n-1 into frame n, and the start table tells it where that
 * carried state belongs to another sequence and has to be dropped.  This is the
 * smallest consumer with such feedback: per feature a first-order linear
 * recurrence along time,
 *     h = x                   at a slot that starts a sequence
 *     h = decay * h_prev + x  at every other valid slot
 *     h = 0                   at a padding slot,
 * where a slot starts a sequence exactly as for bload_segment_reduce (valid, and
 * carrying a start flag, or first of its block, or behind an invalid slot).
 *
 * d_packed   in   [B, t_blk, feat_dim] of `dtype` (U8, F16 or F32; I32 is
 *                 refused with BLOAD_EINVAL), 16-byte aligned
 * d_reset, d_valid   in   uint8[B, t_blk]
 * decay      in   any float
 * d_out      out  float32[B, t_blk, feat_dim], 16-byte aligned; every element is
 *                 written.  float32 arithmetic in time order inside chunks of time;
 *                 a sequence that crosses a chunk border receives the state in
 *                 front of the chunk as decay^chunk * (state one chunk earlier) +
 *                 (the chunk's own part).  For the k-th frame of a sequence the
 *                 result differs from the exact one by at most (3k + 4) * 2^-24 * S,
 *                 S being the same recurrence run on |x| with |decay|.
 * d_workspace     device scratch of >= bload_segment_scan_workspace_bytes(...)
 *                 bytes, 16-byte aligned (may be NULL when that is 0).
 * Asynchronous on `hip_stream`; same inputs give bit-identical outputs.
 */
size_t bload_segment_scan_workspace_bytes(int64_t num_blocks, int32_t t_blk, int64_t feat_dim,
                                          bload_dtype dtype);

bload_status bload_segment_scan(const void* d_packed, const uint8_t* d_reset,
                                const uint8_t* d_valid, int64_t num_blocks, int32_t t_blk,
                                int64_t feat_dim, bload_dtype dtype, float decay, float* d_out,
                                void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------- strategy counts --
 * Problem Statement and Table 1 (rows "padding amount" and "# frames deleted"):
 * what the strategies compared there cost on a given set of lengths, counted in
 * frames, without materialising anything.
 *   pad to the longest  every sequence padded to t_max:  n_seq * t_max - sum(L)
 *   chunk sampling      every sequence cut into pieces of t_chunk frames, each a
 *                       sample of its own, nothing padded: sum(floor(L / t_chunk))
 *                       samples, sum(L mod t_chunk) frames deleted
 *   block packing       num_blocks * t_blk - sum(L), for the plan's num_blocks
 * ("mix pad" of Table 1 is not defined in the paper and is not counted.)
 *
 * d_lengths   in   int32[n_seq], every L >= 0
 * t_max       in   pad-to-longest target; <= 0 means "the longest sequence found"
 * t_chunk     in   >= 1
 * num_blocks, t_blk   in   as returned by / given to a planner (0, 0 to skip)
 * h_counts    out  host struct, see below
 * d_workspace      >= 64 bytes, 16-byte aligned
 *
 * Synchronises the stream before returning.
 */
typedef struct bload_strategy_counts_t {
    int64_t total_frames;       /* sum(L) */
    int64_t longest;            /* max(L), 0 when n_seq == 0 */
    int64_t pad_to_longest;     /* frames of padding when every sequence is padded */
    int64_t pad_blocks;         /* frames of padding in the packed blocks */
    int64_t chunk_samples;      /* pieces of t_chunk frames */
    int64_t chunk_deleted;      /* frames that fill no piece */
} bload_strategy_counts_t;

bload_status bload_strategy_counts(const int32_t* d_lengths, int64_t n_seq, int32_t t_max,
                                   int32_t t_chunk, int64_t num_blocks, int32_t t_blk,
                                   bload_strategy_counts_t* h_counts, void* d_workspace,
                                   size_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* BLOAD_H */
