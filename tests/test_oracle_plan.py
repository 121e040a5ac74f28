"""Pins for the oracle's block assignment (Methods section: blocks of T_max
frames made of whole sequences, closed as near T_max as the order allows) and
for the padding counts (Problem Statement, Table 1)."""
import itertools

import numpy as np
import pytest

import oracle
from conftest import golden_rows
from paper_2310_10879_amd import workloads


def optimal_bins(L, T):
    """Fewest bins of capacity T that hold all items: exact DP over subsets
    (state = set of packed items -> (bins used, room left in the last bin),
    lexicographically best).  Brute force, N <= 12."""
    n = len(L)
    best = [(n + 1, 0)] * (1 << n)
    best[0] = (0, 0)                     # no bin open yet
    for mask in range(1 << n):
        bins, room = best[mask]
        if bins > n:
            continue
        for i in range(n):
            if mask & (1 << i):
                continue
            if L[i] <= room:
                cand = (bins, room - L[i])
            else:
                cand = (bins + 1, T - L[i])
            nxt = mask | (1 << i)
            # fewer bins is better; with equal bins, more room left is better
            if cand[0] < best[nxt][0] or (cand[0] == best[nxt][0] and cand[1] > best[nxt][1]):
                best[nxt] = cand
    return best[(1 << n) - 1][0]


def check_plan_invariants(L, T, order, pl):
    """Everything that characterises next-fit over `order`, without re-running it."""
    n = len(L)
    L = np.asarray(L, dtype=np.int64)
    B = pl.num_blocks
    if n == 0:
        assert B == 0 and pl.total_frames == 0
        return
    assert pl.total_frames == int(L.sum())
    bf = pl.block_first.astype(np.int64)
    assert bf.shape == (B + 1,)
    assert bf[0] == 0 and bf[B] == n
    assert np.all(np.diff(bf) >= 1)                       # no empty block
    Ls = L[order]                                         # lengths in shuffled order
    fills = np.add.reduceat(Ls, bf[:-1])
    assert fills.sum() == L.sum()                         # (i)
    assert np.all(fills > 0) and np.all(fills <= T)       # (ii)
    assert B * T - L.sum() == np.sum(T - fills)           # (iii) padding
    if B > 1:                                             # (iv) the next one did not fit
        assert np.all(fills[:-1] + Ls[bf[1:-1]] > T)
        # consequence: adjacent fills exceed T, so B <= 2*ceil(sum/T) - 1
        assert np.all(fills[:-1] + fills[1:] > T)
    assert B <= 2 * -(-int(L.sum()) // T) - 1 or B == 1
    # block / offset of every sequence agree with the contiguous runs
    blk_of_pos = np.repeat(np.arange(B), np.diff(bf))
    assert np.array_equal(pl.block_of_seq[order], blk_of_pos)
    starts = np.cumsum(Ls) - Ls
    off_of_pos = starts - np.repeat(starts[bf[:-1]], np.diff(bf))
    assert np.array_equal(pl.offset_of_seq[order], off_of_pos)
    # (vii) reading the blocks in order gives back the shuffled order
    rebuilt = []
    for b in range(min(B, 50)):
        members = np.nonzero(pl.block_of_seq == b)[0]
        members = members[np.argsort(pl.offset_of_seq[members], kind="stable")]
        rebuilt.extend(members.tolist())
    assert rebuilt == list(order[:len(rebuilt)])


@pytest.mark.parametrize("kind", ["uniform", "short", "long", "mixed"])
@pytest.mark.parametrize("n,T", [(1, 1), (1, 5), (2, 3), (7, 4), (64, 32), (257, 16),
                                 (1000, 600), (5000, 7), (4096, 4096)])
def test_invariants_random(kind, n, T):
    rng = np.random.default_rng(n * 1000 + T)
    L = workloads.random_lengths(rng, n, T, kind)
    for seed in (0, 1, 99):
        o = oracle.order(n, seed)
        pl = oracle.plan(L, T, o)
        check_plan_invariants(L, T, o, pl)


def test_empty():
    pl = oracle.plan(np.zeros(0, np.int32), 8, np.zeros(0, np.int32))
    assert pl.num_blocks == 0 and pl.total_frames == 0


def test_closed_forms():
    n, T = 37, 12
    ident = np.arange(n, dtype=np.int32)
    # every sequence fills a block
    pl = oracle.plan(np.full(n, T), T, ident)
    assert pl.num_blocks == n and np.all(pl.offset_of_seq == 0)
    assert np.array_equal(pl.block_of_seq, ident)
    assert oracle.padding(np.full(n, T), T, pl.num_blocks, T) == (0, 0)
    # unit sequences: T per block
    pl = oracle.plan(np.ones(n), T, ident)
    assert pl.num_blocks == -(-n // T)
    assert np.array_equal(pl.block_of_seq, ident // T)
    assert np.array_equal(pl.offset_of_seq, ident % T)
    # just over half: nothing shares a block
    pl = oracle.plan(np.full(n, T // 2 + 1), T, ident)
    assert pl.num_blocks == n
    # exactly half: two per block, an exactly full block closes on the next item
    pl = oracle.plan(np.full(n, T // 2), T, ident)
    assert pl.num_blocks == -(-n // 2)
    assert np.array_equal(pl.offset_of_seq, (ident % 2) * (T // 2))
    # one sequence
    pl = oracle.plan(np.array([5]), T, np.array([0]))
    assert (pl.num_blocks, int(pl.block_of_seq[0]), int(pl.offset_of_seq[0])) == (1, 0, 0)
    assert list(pl.block_first) == [0, 1]


def test_hand_worked_example():
    # T = 10, visiting order 2,0,3,1 with lengths L0=4, L1=7, L2=6, L3=3:
    # 6 | +4 = 10 full | 3 opens block 1 | +7 = 10 full  ->  2 blocks, no padding
    L = np.array([4, 7, 6, 3], dtype=np.int32)
    o = np.array([2, 0, 3, 1], dtype=np.int32)
    pl = oracle.plan(L, 10, o)
    assert pl.num_blocks == 2
    assert list(pl.block_of_seq) == [0, 1, 0, 1]
    assert list(pl.offset_of_seq) == [6, 3, 0, 0]
    assert list(pl.block_first) == [0, 2, 4]
    # same lengths, identity order: 4 | 7 does not fit -> block 1 | 6 -> block 2, +3 = 9
    pl = oracle.plan(L, 10, np.arange(4, dtype=np.int32))
    assert pl.num_blocks == 3
    assert list(pl.block_of_seq) == [0, 1, 2, 2]
    assert list(pl.offset_of_seq) == [0, 0, 0, 6]
    assert list(pl.block_first) == [0, 1, 2, 4]
    assert oracle.padding(L, 7, 3, 10) == (4 * 7 - 20, 30 - 20)


def test_rejects_bad_lengths():
    ident = np.arange(3, dtype=np.int32)
    for bad in ([1, 0, 2], [1, 9, 2], [-3, 1, 1]):
        with pytest.raises(ValueError):
            oracle.plan(np.array(bad, dtype=np.int32), 8, ident)


def test_within_twice_the_optimum_bruteforce():
    rng = np.random.default_rng(2024)
    for trial in range(60):
        n = int(rng.integers(1, 11))
        T = int(rng.integers(1, 13))
        L = rng.integers(1, T, size=n, endpoint=True).astype(np.int32)
        opt = optimal_bins([int(x) for x in L], T)
        assert opt >= -(-int(L.sum()) // T)
        for seed in range(4):
            o = oracle.order(n, seed)
            pl = oracle.plan(L, T, o)
            assert opt <= pl.num_blocks <= max(1, 2 * opt - 1)


def test_bruteforce_optimum_agrees_with_exhaustive_orders():
    # the DP itself, checked on tiny inputs against trying every order with next-fit
    rng = np.random.default_rng(5)
    for _ in range(20):
        n = int(rng.integers(1, 7))
        T = int(rng.integers(2, 9))
        L = rng.integers(1, T, size=n, endpoint=True).astype(np.int32)
        best = min(oracle.plan(L, T, np.array(p, dtype=np.int32)).num_blocks
                   for p in itertools.permutations(range(n)))
        assert best == optimal_bins([int(x) for x in L], T)


def test_paper_pad_to_longest_count():
    # Table 1, "0 padding" column: N * T_max - sum(L) for the training split.
    (n, total, lo, tmax, expect), = golden_rows("table1_padding.txt")
    # any lengths with that N, sum, minimum and maximum give the same count
    rng = np.random.default_rng(1)
    L = np.full(n, lo, dtype=np.int64)
    L[0] = tmax
    rest = total - int(L.sum())
    while rest > 0:
        i = int(rng.integers(1, n))
        add = min(rest, tmax - int(L[i]), int(rng.integers(1, 40)))
        L[i] += add
        rest -= add
    assert L.sum() == total and L.min() == lo and L.max() == tmax
    pad_longest, _ = oracle.padding(L.astype(np.int32), tmax, 0, tmax)
    assert pad_longest == expect


def test_padding_below_pad_to_longest_on_the_workloads():
    # the paper's claim in kind (abstract: padding cut by more than 100x on its
    # dataset): block padding is well below pad-to-longest padding on every
    # workload, the more so the further the typical length is from T_max
    floor = {1: 3, 2: 20, 3: 1000, 4: 2}
    for wid in (1, 2, 3, 4):
        w = workloads.WORKLOADS[wid]
        L = workloads.lengths(wid)
        o = oracle.order(w.n_seq, 0)
        pl = oracle.plan(L, w.t_blk, o)
        check_plan_invariants(L, w.t_blk, o, pl)
        pad_longest, pad_blocks = oracle.padding(L, w.t_blk, pl.num_blocks, w.t_blk)
        assert pad_blocks == pl.num_blocks * w.t_blk - pl.total_frames
        assert pad_blocks * floor[wid] < pad_longest
