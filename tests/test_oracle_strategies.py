"""Pins for the counts of the comparison strategies (Problem Statement; Table 1, rows
"padding amount" and "# frames deleted"): padding to the longest sequence, and cutting
every sequence into pieces of a fixed length."""
import numpy as np
import pytest

import oracle
from conftest import golden_rows
from paper_2310_10879_amd import workloads


def test_table1_sampling_column_is_whole_pieces_of_the_average_length():
    (n, total, deleted, padding, t_chunk, pieces), = golden_rows("table1_sampling.txt")
    assert t_chunk == total // n                      # "the length of the average entry"
    assert padding == 0
    assert total - deleted == t_chunk * pieces        # the paper's own numbers: whole pieces only


def test_paper_aggregates_are_reproduced_by_a_length_set_with_them():
    """A length multiset with the paper's N, frame total, shortest and longest video, cut into
    pieces of 22: kept + deleted = total, and the kept frames are whole pieces."""
    (n, total, deleted, _, t_chunk, pieces), = golden_rows("table1_sampling.txt")
    rng = np.random.default_rng(7)
    L = np.full(n, 3, dtype=np.int64)
    L[0] = 94
    spare = total - int(L.sum())
    while spare:                                       # spread the rest without passing 94
        i = rng.integers(1, n)
        add = min(spare, int(rng.integers(1, 40)), 94 - int(L[i]))
        L[i] += add
        spare -= add
    assert L.sum() == total and L.min() == 3 and L.max() == 94
    samples, gone = oracle.chunk_sampling(L, t_chunk)
    assert samples * t_chunk + gone == total
    assert samples == int((L // t_chunk).sum()) and gone == int((L % t_chunk).sum())
    pad_longest, _ = oracle.padding(L.astype(np.int32), 94, 0, 94)
    assert pad_longest == 534831                       # the table's "0 padding" column


def test_closed_forms():
    assert oracle.chunk_sampling(np.array([], np.int32), 5) == (0, 0)
    assert oracle.chunk_sampling(np.array([5, 10, 15], np.int32), 5) == (6, 0)
    assert oracle.chunk_sampling(np.array([4, 4, 4], np.int32), 5) == (0, 12)     # all too short
    assert oracle.chunk_sampling(np.array([7, 1, 12], np.int32), 1) == (20, 0)    # pieces of one frame
    assert oracle.chunk_sampling(np.array([3, 94, 22, 23, 21, 44], np.int32), 22) == (1 + 4 + 1 + 2, 3 + 6 + 1 + 21)


@pytest.mark.parametrize("wid", [1, 2, 3, 4])
def test_identities_on_the_workloads(wid):
    w = workloads.WORKLOADS[wid]
    L = workloads.lengths(wid)
    total = int(L.astype(np.int64).sum())
    for t_chunk in (1, 7, int(L.mean()), w.t_blk, w.t_blk + 1):
        samples, gone = oracle.chunk_sampling(L, t_chunk)
        assert samples * t_chunk + gone == total
        assert 0 <= gone <= len(L) * (t_chunk - 1)
        if t_chunk > L.max():
            assert samples == 0 and gone == total
