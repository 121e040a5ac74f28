"""Pins for the oracle's gather / zero-pad and per-slot start table (Methods
section: blocks padded with 0's; the table of where each new video starts)."""
import numpy as np
import pytest

import oracle
from paper_2310_10879_amd import workloads


def run_pack(L, T, F, seed, src=None):
    L = np.asarray(L, dtype=np.int32)
    so = workloads.src_offsets(L)
    if src is None:
        src = workloads.tagged_source(L, F)
    o = oracle.order(len(L), seed)
    pl = oracle.plan(L, T, o)
    return src, so, pl, oracle.pack(src, so, L, pl, F)


def check_pack_properties(L, T, F, src, so, pl, out):
    packed, seq_id, frame_idx, reset, valid = out
    L = np.asarray(L, dtype=np.int64)
    B = pl.num_blocks
    assert packed.shape == (B, T, F) and seq_id.shape == (B, T)
    assert set(np.unique(valid)) <= {0, 1} and set(np.unique(reset)) <= {0, 1}
    v = valid.astype(bool)
    assert v.sum() == L.sum()                                  # every frame once ...
    assert reset.sum() == len(L)                               # one start per sequence
    assert np.array_equal(reset.astype(bool), v & (frame_idx == 0))
    # valid slots are a prefix of each block
    fill = v.sum(axis=1)
    assert np.array_equal(v, np.arange(T)[None, :] < fill[:, None])
    # padding: zero payload, -1 ids, no flags
    assert not packed[~v].any()
    assert np.all(seq_id[~v] == -1) and np.all(frame_idx[~v] == -1)
    assert not reset[~v].any()
    # ... and it is the right frame, in order
    sid, fid = seq_id[v].astype(np.int64), frame_idx[v].astype(np.int64)
    assert np.array_equal(np.bincount(sid, minlength=len(L)), L)
    assert np.all(fid < L[sid]) and np.all(fid >= 0)
    src_b = np.ascontiguousarray(src).view(np.uint8).reshape(-1, F)
    assert np.array_equal(packed[v], src_b[so[sid] + fid])
    # consecutive valid slots of one block: same sequence -> frame index + 1,
    # otherwise a new sequence starting at frame 0 after the previous one ended
    flat_s, flat_f = seq_id.reshape(-1), frame_idx.reshape(-1)
    both = (v.reshape(-1)[1:] & v.reshape(-1)[:-1]) & (np.arange(1, B * T) % T != 0)
    same = flat_s[1:] == flat_s[:-1]
    assert np.all(flat_f[1:][both & same] == flat_f[:-1][both & same] + 1)
    ends = both & ~same
    assert np.all(flat_f[1:][ends] == 0)
    assert np.all(flat_f[:-1][ends] == L[flat_s[:-1][ends]] - 1)
    # the slot of every sequence's first frame is what the plan's table says
    b_idx, t_idx = np.nonzero(reset)
    assert np.array_equal(pl.block_of_seq[seq_id[b_idx, t_idx]], b_idx)
    assert np.array_equal(pl.offset_of_seq[seq_id[b_idx, t_idx]], t_idx)


@pytest.mark.parametrize("F", [1, 3, 4, 8, 16, 48, 320])
@pytest.mark.parametrize("n,T,kind", [(1, 4, "uniform"), (9, 5, "uniform"), (64, 32, "uniform"),
                                      (300, 17, "short"), (100, 64, "long"), (200, 33, "mixed")])
def test_every_frame_once_in_order(F, n, T, kind):
    rng = np.random.default_rng(n + T + F)
    L = workloads.random_lengths(rng, n, T, kind)
    src, so, pl, out = run_pack(L, T, F, seed=3)
    check_pack_properties(L, T, F, src, so, pl, out)


def test_tagged_payload_decodes_to_metadata():
    # frames carry (sequence, frame) in their first 8 bytes: decode every valid slot
    rng = np.random.default_rng(11)
    L = workloads.random_lengths(rng, 150, 40, "mixed")
    src, so, pl, (packed, seq_id, frame_idx, reset, valid) = run_pack(L, 40, 12, seed=5)
    v = valid.astype(bool)
    dec = packed[v][:, :8].copy().view("<i4")
    assert np.array_equal(dec[:, 0], seq_id[v])
    assert np.array_equal(dec[:, 1], frame_idx[v])


def test_single_full_sequence_is_a_copy():
    T, F = 23, 10
    L = np.array([T], dtype=np.int32)
    src, so, pl, (packed, seq_id, frame_idx, reset, valid) = run_pack(L, T, F, seed=0)
    assert np.array_equal(packed.reshape(-1), src.reshape(-1))
    assert np.all(seq_id == 0) and np.array_equal(frame_idx[0], np.arange(T))
    assert reset[0, 0] == 1 and reset.sum() == 1 and valid.all()


def test_empty_input():
    L = np.zeros(0, dtype=np.int32)
    src, so, pl, (packed, *_rest) = run_pack(L, 8, 4, seed=0)
    assert packed.shape == (0, 8, 4)


def test_slabs_agree_with_whole():
    rng = np.random.default_rng(21)
    L = workloads.random_lengths(rng, 120, 30, "uniform")
    src, so, pl, whole = run_pack(L, 30, 6, seed=9)
    for lo, hi in [(0, 1), (3, 11), (pl.num_blocks - 2, pl.num_blocks)]:
        part = oracle.pack_blocks(src, so, L, pl, 6, lo, hi)
        for a, b in zip(part, whole):
            assert np.array_equal(a, b[lo:hi])


def test_workload_1_shape():
    w = workloads.WORKLOADS[1]
    L = workloads.lengths(1)
    assert L.min() >= 2 and L.max() <= 32 and len(L) == 64
    src = workloads.source(1, 0, int(L.sum()))
    so = workloads.src_offsets(L)
    pl = oracle.plan(L, w.t_blk, oracle.order(w.n_seq, 0))
    out = oracle.pack(src, so, L, pl, w.frame_bytes)
    check_pack_properties(L, w.t_blk, w.frame_bytes, src, so, pl, out)
