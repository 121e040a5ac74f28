/* Driver for tests/test_oracle_sanitize.py: runs every oracle function on a small input
 * under AddressSanitizer / UndefinedBehaviorSanitizer (host code only).  Exits 0 when the
 * invariants hold; the sanitizers abort the process on any bad access. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void bload_oracle_order(int64_t n, uint64_t seed, int32_t* order);
int bload_oracle_plan(const int32_t* lengths, int64_t n, int32_t t_blk, const int32_t* order,
                      int32_t* block_of_seq, int32_t* offset_of_seq, int32_t* block_first,
                      int64_t* num_blocks, int64_t* total_frames);
void bload_oracle_pack_blocks(const uint8_t* src, const int64_t* src_offsets, const int32_t* lengths,
                              const int32_t* block_of_seq, const int32_t* offset_of_seq, int64_t n,
                              int32_t t_blk, int64_t frame_bytes, int64_t block_lo, int64_t block_hi,
                              uint8_t* packed, int32_t* seq_id, int32_t* frame_idx, uint8_t* reset,
                              uint8_t* valid);
int bload_oracle_segment_reduce(const void* src, const int64_t* src_offsets, const int32_t* lengths,
                                int64_t n, int64_t feat_dim, int dtype, int op, void* out);
int64_t bload_oracle_segment_reduce_packed(const void* packed, const int32_t* seq_id,
                                           const uint8_t* reset, const uint8_t* valid,
                                           int64_t num_blocks, int32_t t_blk, int64_t feat_dim,
                                           int dtype, int op, int64_t n_seq, void* out);
int64_t bload_oracle_plan_shard(const int32_t* order, const int32_t* block_of_seq,
                                const int32_t* block_first, int64_t n, int64_t num_blocks,
                                int32_t rank, int32_t world, int32_t* order_local,
                                int32_t* block_of_seq_local, int32_t* block_first_local);
int64_t bload_oracle_plan_check(const int64_t* src_offsets, const int32_t* lengths, const int32_t* order,
                                const int32_t* block_of_seq, const int32_t* offset_of_seq,
                                const int32_t* block_first, int64_t n, int64_t num_blocks, int32_t t_blk,
                                int64_t total_frames);

int main(void)
{
    enum { N = 257, T = 19, D = 3 };
    int32_t* lengths = malloc(N * sizeof(int32_t));
    int64_t* so = malloc((N + 1) * sizeof(int64_t));
    int64_t total = 0;
    for (int i = 0; i < N; ++i) { lengths[i] = 1 + (int32_t)((i * 7919u) % T); so[i] = total; total += lengths[i]; }
    so[N] = total;
    int32_t* src = malloc((size_t)total * D * sizeof(int32_t));
    for (int64_t e = 0; e < total * D; ++e) src[e] = (int32_t)(e % 1000) - 500;

    int32_t* order = malloc(N * sizeof(int32_t));
    int32_t* block_of = malloc(N * sizeof(int32_t));
    int32_t* offset_of = malloc(N * sizeof(int32_t));
    int32_t* block_first = malloc((N + 1) * sizeof(int32_t));
    int64_t B = 0, frames = 0;
    bload_oracle_order(N, 12345, order);
    if (bload_oracle_plan(lengths, N, T, order, block_of, offset_of, block_first, &B, &frames) != 0) return 2;
    if (frames != total || B < 1 || block_first[B] != N) return 3;
    so[N] = total;
    if (bload_oracle_plan_check(so, lengths, order, block_of, offset_of, block_first, N, B, T, total) != -1) return 10;
    offset_of[order[40]] += 1;
    if (bload_oracle_plan_check(so, lengths, order, block_of, offset_of, block_first, N, B, T, total) != 40) return 11;
    offset_of[order[40]] -= 1;

    size_t slots = (size_t)B * T;
    uint8_t* packed = malloc(slots * D * 4);
    int32_t* seq_id = malloc(slots * 4);
    int32_t* frame_idx = malloc(slots * 4);
    uint8_t* reset = malloc(slots);
    uint8_t* valid = malloc(slots);
    bload_oracle_pack_blocks((const uint8_t*)src, so, lengths, block_of, offset_of, N, T, D * 4, 0, B,
                             packed, seq_id, frame_idx, reset, valid);
    int64_t n_valid = 0, n_reset = 0;
    for (size_t s = 0; s < slots; ++s) { n_valid += valid[s]; n_reset += reset[s]; }
    if (n_valid != total || n_reset != N) return 4;

    int64_t* sums = malloc((size_t)N * D * sizeof(int64_t));
    int64_t* sums2 = calloc((size_t)N * D, sizeof(int64_t));
    if (bload_oracle_segment_reduce(src, so, lengths, N, D, 3, 0, sums) != 0) return 5;
    if (bload_oracle_segment_reduce_packed(packed, seq_id, reset, valid, B, T, D, 3, 0, N, sums2) != N) return 6;
    if (memcmp(sums, sums2, (size_t)N * D * sizeof(int64_t)) != 0) return 7;

    float* means = malloc((size_t)N * D * sizeof(float));
    float* fsrc = malloc((size_t)total * D * sizeof(float));
    for (int64_t e = 0; e < total * D; ++e) fsrc[e] = (float)src[e] * 0.25f;
    if (bload_oracle_segment_reduce(fsrc, so, lengths, N, D, 2, 1, means) != 0) return 8;

    int32_t* order_l = malloc(N * sizeof(int32_t));
    int32_t* block_l = malloc(N * sizeof(int32_t));
    int32_t* first_l = malloc((size_t)(B + 2) * sizeof(int32_t));
    int64_t seen = 0;
    for (int r = 0; r < 3; ++r) seen += bload_oracle_plan_shard(order, block_of, block_first, N, B, r, 3, order_l, block_l, first_l);
    if (seen != N) return 9;

    free(lengths); free(so); free(src); free(order); free(block_of); free(offset_of); free(block_first);
    free(packed); free(seq_id); free(frame_idx); free(reset); free(valid); free(sums); free(sums2);
    free(means); free(fsrc); free(order_l); free(block_l); free(first_l);
    puts("oracle sanitize run ok");
    return 0;
}
