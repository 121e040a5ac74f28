"""Pins for the oracle's per-sequence reduction (the consumer of the start
table of the Methods section, as a sum / mean over each sequence's frames)."""
import numpy as np
import pytest

import oracle
from paper_2310_10879_amd import workloads


def test_half_decoding_matches_numpy_for_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))


def ragged(L, D, fn, dtype):
    """source[sum(L), D] with element (i, t, d) = fn(i, t, d)."""
    L = np.asarray(L, dtype=np.int64)
    so = workloads.src_offsets(L.astype(np.int32))
    i = np.repeat(np.arange(len(L)), L)
    t = np.arange(L.sum()) - np.repeat(so[:-1], L)
    d = np.arange(D)
    return fn(i[:, None], t[:, None], d[None, :]).astype(dtype), so


L_CASES = [np.array([1]), np.array([5, 1, 1, 9, 2]), np.arange(1, 60)]


@pytest.mark.parametrize("L", L_CASES)
@pytest.mark.parametrize("dtype,np_dtype", [("u8", np.uint8), ("f16", np.float16),
                                            ("f32", np.float32)])
def test_closed_forms_float_paths(L, dtype, np_dtype):
    D = 5
    Lf = L.astype(np.float64)[:, None]
    # constant payload: mean is the constant, sum is c * L
    src, so = ragged(L, D, lambda i, t, d: 3 + 0 * i + 0 * t + d, np_dtype)
    assert np.array_equal(oracle.segment_reduce(src, so, L, D, dtype, "mean"),
                          np.broadcast_to(3.0 + np.arange(D), (len(L), D)).astype(np.float32))
    assert np.array_equal(oracle.segment_reduce(src, so, L, D, dtype, "sum"),
                          (Lf * (3.0 + np.arange(D))).astype(np.float32))
    # payload = frame index: sum is L(L-1)/2, mean is (L-1)/2
    src, so = ragged(L, D, lambda i, t, d: t + 0 * d, np_dtype)
    assert np.array_equal(oracle.segment_reduce(src, so, L, D, dtype, "sum"),
                          np.broadcast_to(Lf * (Lf - 1) / 2, (len(L), D)).astype(np.float32))
    assert np.array_equal(oracle.segment_reduce(src, so, L, D, dtype, "mean"),
                          np.broadcast_to((Lf - 1) / 2, (len(L), D)).astype(np.float32))
    # payload = sequence index: the mean gives the index back; a frame taken
    # from a neighbour would change it
    src, so = ragged(L, D, lambda i, t, d: i + 0 * t + 0 * d, np_dtype)
    assert np.array_equal(oracle.segment_reduce(src, so, L, D, dtype, "mean"),
                          np.broadcast_to(np.arange(len(L))[:, None], (len(L), D)).astype(np.float32))
    # feature index must not be mixed with time: payload = d * (t + 1)
    src, so = ragged(L, D, lambda i, t, d: d * (t + 1), np_dtype)
    assert np.array_equal(oracle.segment_reduce(src, so, L, D, dtype, "sum"),
                          (np.arange(D)[None, :] * (Lf * (Lf + 1) / 2)).astype(np.float32))


@pytest.mark.parametrize("L", L_CASES)
def test_closed_forms_int_path(L):
    D = 3
    big = 2_000_000_000                       # sums overflow int32, not int64
    src, so = ragged(L, D, lambda i, t, d: big - d + 0 * i + 0 * t, np.int32)
    got = oracle.segment_reduce(src, so, L, D, "i32", "sum")
    assert got.dtype == np.int64
    assert np.array_equal(got, L.astype(np.int64)[:, None] * (big - np.arange(D))[None, :])
    src, so = ragged(L, D, lambda i, t, d: -t * (d + 1), np.int32)
    Li = L.astype(np.int64)[:, None]
    assert np.array_equal(oracle.segment_reduce(src, so, L, D, "i32", "sum"),
                          -(Li * (Li - 1) // 2) * (np.arange(D) + 1)[None, :])
    with pytest.raises(ValueError):
        oracle.segment_reduce(src, so, L, D, "i32", "mean")


@pytest.mark.parametrize("dtype,np_dtype", [("u8", np.uint8), ("f16", np.float16),
                                            ("f32", np.float32)])
def test_against_numpy_reduceat_in_float64(dtype, np_dtype):
    rng = np.random.default_rng(3)
    L = workloads.random_lengths(rng, 200, 300, "mixed")
    so = workloads.src_offsets(L)
    D = 7
    x = (rng.standard_normal((int(L.sum()), D)) * 2 - 4)
    src = (np.abs(x) * 20).astype(np.uint8) if dtype == "u8" else x.astype(np_dtype)
    ref_sum = np.add.reduceat(src.astype(np.float64), so[:-1], axis=0)
    got_sum = oracle.segment_reduce(src, so, L, D, dtype, "sum")
    got_mean = oracle.segment_reduce(src, so, L, D, dtype, "mean")
    # numpy adds pairwise, the oracle serially: both in float64, so they agree
    # far below float32 resolution; the result is float32
    assert got_sum.dtype == np.float32
    np.testing.assert_allclose(got_sum, ref_sum, rtol=2e-7, atol=0)
    np.testing.assert_allclose(got_mean, ref_sum / L[:, None], rtol=2e-7, atol=0)


def test_workload_reductions_have_the_expected_statistics():
    # workload 4 payload is N(-4, 2): per-sequence means sit near -4
    w = workloads.WORKLOADS[4]
    L = workloads.lengths(4)[:50]
    so = workloads.src_offsets(L)
    src = workloads.source(4, 0, int(so[-1]))
    m = oracle.segment_reduce(src, so, L, w.frame_elems, "f32", "mean")
    assert m.shape == (50, 80)
    assert abs(float(m.mean()) + 4.0) < 0.01
    assert float(np.abs(m + 4.0).max()) < 2.0 * 6 / np.sqrt(L.min())


# ---- the reduction read from the packed blocks and their flags

@pytest.mark.parametrize("dtype,np_dtype,op", [("u8", np.uint8, "mean"), ("f16", np.float16, "sum"),
                                               ("f32", np.float32, "mean"), ("i32", np.int32, "sum")])
def test_packed_reading_equals_the_ragged_definition(dtype, np_dtype, op):
    # on what a correct pack writes, walking the blocks with resets at the start flags must
    # give exactly the per-sequence reduction of the ragged source (both add in time order)
    rng = np.random.default_rng(17)
    n, T, D = 150, 40, 3
    L = workloads.random_lengths(rng, n, T, "mixed")
    so = workloads.src_offsets(L)
    src = (rng.standard_normal((int(so[-1]), D)) * 50).astype(np_dtype)
    pl = oracle.plan(L, T, oracle.order(n, 2))
    packed, seq_id, frame_idx, reset, valid = oracle.pack(src, so, L, pl, D * src.dtype.itemsize)
    want = oracle.segment_reduce(src, so, L, D, dtype, op)
    got, nseg = oracle.segment_reduce_packed(packed, seq_id, reset, valid, D, dtype, op, n)
    assert nseg == n
    assert np.array_equal(got, want)
    # garbage in the padding payload changes nothing
    packed = packed.copy()
    packed[valid == 0] = 0x5A
    got2, _ = oracle.segment_reduce_packed(packed, seq_id, reset, valid, D, dtype, op, n)
    assert np.array_equal(got2, want)


def test_packed_reading_hand_worked_flags():
    # one block of 10 slots, payload = slot number + 1, flags chosen by hand:
    # slot     0  1  2  3  4  5  6  7  8  9
    # valid    1  1  0  1  1  1  0  0  1  1
    # reset    0  0  0  0  1  0  0  0  0  1
    # segments [0,1] (block start)  [3] (after padding)  [4,5] (flag)  [8] (after padding)  [9] (flag)
    valid = np.array([[1, 1, 0, 1, 1, 1, 0, 0, 1, 1]], dtype=np.uint8)
    reset = np.array([[0, 0, 0, 0, 1, 0, 0, 0, 0, 1]], dtype=np.uint8)
    seq_id = np.array([[0, 0, -1, 1, 2, 2, -1, -1, 3, 4]], dtype=np.int32)
    packed = (np.arange(10, dtype=np.int32) + 1).reshape(1, 10, 1)
    got, nseg = oracle.segment_reduce_packed(packed, seq_id, reset, valid, 1, "i32", "sum", 6)
    assert nseg == 5
    assert got[:, 0].tolist() == [1 + 2, 4, 5 + 6, 9, 10, 0]
    gotf, _ = oracle.segment_reduce_packed(packed.astype(np.float32), seq_id, reset, valid, 1, "f32",
                                           "mean", 6)
    assert gotf[:, 0].tolist() == [1.5, 4.0, 5.5, 9.0, 10.0, 0.0]
    # two blocks never share a segment: the same flags twice, second block without any start flag
    valid2 = np.ones((2, 4), dtype=np.uint8)
    reset2 = np.zeros((2, 4), dtype=np.uint8)
    seq2 = np.array([[0, 0, 0, 0], [1, 1, 1, 1]], dtype=np.int32)
    pk2 = np.arange(8, dtype=np.int32).reshape(2, 4, 1)
    got2, nseg2 = oracle.segment_reduce_packed(pk2, seq2, reset2, valid2, 1, "i32", "sum", 2)
    assert nseg2 == 2 and got2[:, 0].tolist() == [0 + 1 + 2 + 3, 4 + 5 + 6 + 7]
