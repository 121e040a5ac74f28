/*
 * bload_yardsticks.h -- streaming kernels without any of the packer's logic.
 *
 * The packer's kernels are bound by HBM traffic, and how fast HBM goes depends on the access
 * pattern: one stream or five, short workgroups in address order or waves that each walk a long
 * row of their own.  These kernels move the same bytes in the same patterns and nothing else, so
 * that a benchmark can put what a pattern alone reaches on this GPU beside what the library's
 * kernel reaches with it.  They are measuring sticks, not part of the method: libbload.so does not
 * contain them (they live in libbload_yardsticks.so) and nothing in the packer calls them.
 *
 * Conventions as in bload.h: d_* are device pointers owned by the caller, `hip_stream` is a
 * hipStream_t passed as void*; every call enqueues one kernel and returns without waiting.
 * Return value: 0 = enqueued, 1 = refused (null pointer, size not as required), 6 = the launch
 * failed.  Base pointers must be 16-byte aligned.
 */
#ifndef BLOAD_YARDSTICKS_H
#define BLOAD_YARDSTICKS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* d_dst[0 .. bytes) = d_src[0 .. bytes): workgroups of 256 threads in address order, one 16-byte
 * streaming load and one 16-byte streaming store per thread (the shape of the packer's 4 KiB
 * tiles).  `bytes` a multiple of 16. */
int bload_ys_copy(const void* d_src, void* d_dst, size_t bytes, void* hip_stream);

/* Reads d_src[0 .. bytes) the same way and writes nothing (d_sink: 4 bytes that are written only
 * if the data hold an improbable value, so that the loads cannot be dropped). */
int bload_ys_read(const void* d_src, size_t bytes, void* d_sink, void* hip_stream);

/* The traffic of packing 4-byte frames (tokens) in tiles of 1024 slots: per slot 4 bytes read
 * and 4 + 4 + 4 + 1 + 1 bytes written to five separate arrays (payload, two int32 planes, two byte
 * planes), four slots per thread.  As in the packer, workgroup b takes the tile that gives each
 * of the 8 XCDs a contiguous eighth of the tiles.  `padding_percent` of every 100 blocks of four
 * tiles are written with constants without reading (a block's padding); the source of each
 * block of four tiles lies at a hashed 16 KiB-aligned place of d_src when `scattered` is
 * non-zero (sequences come from all over the source), else at the tile's own place.
 * n_slots a multiple of 4096; d_src, d_payload, d_plane_a, d_plane_b hold 4 * n_slots bytes,
 * d_flags_a and d_flags_b hold n_slots bytes.
 * Bytes moved = n_slots * (14 + 4 * (1 - padding share)). */
int bload_ys_token_pack(const void* d_src, void* d_payload, void* d_plane_a, void* d_plane_b,
                        void* d_flags_a, void* d_flags_b, int64_t n_slots, int padding_percent,
                        int scattered, void* hip_stream);

/* Waves that each walk rows of their own from end to end: n_rows rows of row_bytes bytes, laid
 * out one after the other; a wave takes `rows_per_wave` (1, 2 or 4) rows side by side, 64 /
 * rows_per_wave lanes each, of which the first `active_lanes` read 16 bytes per access, so that
 * one access covers active_lanes * 16 contiguous bytes of a row; eight accesses are in flight,
 * then their data (if d_dst is not null) are written to the same place of d_dst.  This is the
 * shape of the reduction and the scan over blocks of frames narrower than a wave (d_dst null: the
 * reduction).  row_bytes a multiple of 8 * 16 * active_lanes.  d_sink as in bload_ys_read. */
int bload_ys_rows(const void* d_src, void* d_dst, int64_t n_rows, int64_t row_bytes, int rows_per_wave,
                  int active_lanes, void* d_sink, void* hip_stream);

#ifdef __cplusplus
}
#endif

#endif /* BLOAD_YARDSTICKS_H */
