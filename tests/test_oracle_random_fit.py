"""Pins for the oracle's random-fit plan: the sampler named in the caption of the paper's
pseudocode figure (a random entry of the length dictionary among those no longer than
the frames remaining in the open block)."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2310_10879_amd import workloads

M64 = (1 << 64) - 1


def check_random_fit_invariants(L, T, pl):
    """What any run of the sampler must satisfy, whatever it drew."""
    L = np.asarray(L, dtype=np.int64)
    n = len(L)
    B = pl.num_blocks
    if n == 0:
        assert B == 0 and pl.total_frames == 0
        return
    assert pl.total_frames == int(L.sum())
    assert np.array_equal(np.sort(pl.order), np.arange(n))            # every sequence once
    bf = pl.block_first.astype(np.int64)
    assert bf.shape == (B + 1,) and bf[0] == 0 and bf[B] == n
    assert np.all(np.diff(bf) >= 1)
    Lp = L[pl.order]                                                  # lengths as placed
    fills = np.add.reduceat(Lp, bf[:-1])
    assert np.all(fills <= T)
    # block and offset of every sequence: the block of its position, the fill before it
    block_of_pos = np.repeat(np.arange(B), np.diff(bf))
    before = np.cumsum(Lp) - Lp
    offset_of_pos = before - before[bf[:-1]][block_of_pos]
    assert np.array_equal(pl.block_of_seq[pl.order], block_of_pos)
    assert np.array_equal(pl.offset_of_seq[pl.order], offset_of_pos)
    # a block closes only when nothing that remains fits: every sequence placed later is
    # longer than the room the block was left with
    shortest_later = np.minimum.accumulate(Lp[::-1])[::-1]            # min over positions >= p
    for b in range(B - 1):
        assert shortest_later[bf[b + 1]] > T - fills[b]
    assert B >= -(-int(L.sum()) // T)


@pytest.mark.parametrize("kind", ["uniform", "short", "long", "mixed"])
@pytest.mark.parametrize("n,t_blk", [(1, 5), (2, 2), (37, 16), (500, 64), (3000, 600)])
def test_invariants(kind, n, t_blk):
    rng = np.random.default_rng(n * 131 + t_blk)
    L = workloads.random_lengths(rng, n, t_blk, kind)
    for seed in workloads.SHUFFLE_SEEDS:
        check_random_fit_invariants(L, t_blk, oracle.plan_random_fit(L, t_blk, seed))


def test_empty_and_bad_lengths():
    pl = oracle.plan_random_fit(np.zeros(0, np.int32), 8, 3)
    assert pl.num_blocks == 0 and pl.total_frames == 0
    for bad in ([0, 3], [9, 1], [-1]):
        with pytest.raises(ValueError):
            oracle.plan_random_fit(np.array(bad, np.int32), 8, 0)


def test_closed_forms():
    # equal lengths l: floor(T/l) per block
    for n, l, T in [(100, 7, 30), (64, 5, 5), (10, 1, 4), (1000, 3, 10)]:
        pl = oracle.plan_random_fit(np.full(n, l, np.int32), T, 5)
        per = T // l
        assert pl.num_blocks == -(-n // per)
        assert np.array_equal(np.diff(pl.block_first)[:-1], np.full(pl.num_blocks - 1, per))
    # pairs that only fit with their complement: lengths a and T-a with 2a > T ... every
    # block of a perfect pairing is full when the long ones cannot share a block
    T = 100
    L = np.array([70] * 20 + [30] * 20, np.int32)
    pl = oracle.plan_random_fit(L, T, 11)
    check_random_fit_invariants(L, T, pl)
    # 30s may also group by three, so the count is not fixed; but each 70 sits with at most one 30
    blocks_of_70 = pl.block_of_seq[:20]
    assert len(set(blocks_of_70.tolist())) == 20
    # all of length T: one per block, in the order they were drawn
    pl = oracle.plan_random_fit(np.full(9, 12, np.int32), 12, 3)
    assert pl.num_blocks == 9 and np.array_equal(pl.offset_of_seq, np.zeros(9))


def splitmix64(seed, k):
    z = (seed + (k + 1) * 0x9E3779B97F4A7C15) & M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def test_first_draws_by_hand():
    """The first placements, re-derived with Python integers from the stated reading:
    draw number 6+p of the seed's stream scaled to the count of fitting sequences, counted
    through the lengths in ascending order, the class giving up its last entry in seeded
    order."""
    L = np.array([5, 3, 3, 8, 1, 3, 5, 2, 8, 1], np.int32)
    T = 9
    for seed in (0, 1, 12345, 0x9E3779B97F4A7C15):
        pl = oracle.plan_random_fit(L, T, seed)
        seeded = oracle.order(len(L), seed).tolist()
        remaining = list(seeded)
        room, p = T, 0
        expect = []
        while remaining and p < 4:
            fits = sorted((int(L[i]), seeded.index(i), i) for i in remaining if L[i] <= room)
            if not fits:
                room = T
                continue
            k = (splitmix64(seed, 6 + p) * len(fits)) >> 64
            length = fits[k][0]
            pick = max((pos, i) for (l, pos, i) in fits if l == length)[1]
            expect.append(pick)
            remaining.remove(pick)
            room -= length
            p += 1
        assert pl.order[:len(expect)].tolist() == expect, seed


def outcome_distribution(lengths, T):
    """Exact law of the sequence of (length placed, block) under 'each remaining sequence
    that fits is equally likely', by walking the whole tree of choices."""
    dist = {}

    def walk(counts, room, trace, prob):
        if sum(counts.values()) == 0:
            dist[trace] = dist.get(trace, 0) + prob
            return
        fit = {l: c for l, c in counts.items() if c and l <= room}
        m = sum(fit.values())
        if m == 0:
            walk(counts, T, trace + ("|",), prob)
            return
        for l, c in fit.items():
            nxt = dict(counts)
            nxt[l] -= 1
            walk(nxt, room - l, trace + (l,), prob * Fraction(c, m))

    counts = {}
    for l in lengths:
        counts[l] = counts.get(l, 0) + 1
    walk(counts, T, (), Fraction(1))
    return dist


def test_law_of_the_blocks_on_a_small_case():
    """Frequencies over many seeds against the exact law of the sampler."""
    L = np.array([3, 2, 2, 1, 4, 1], np.int32)
    T = 5
    law = outcome_distribution(L.tolist(), T)
    assert sum(law.values()) == 1
    runs = 6000
    seen = {}
    for seed in range(runs):
        pl = oracle.plan_random_fit(L, T, seed * 0x2545F4914F6CDD1D + 17)
        trace = []
        for b in range(pl.num_blocks):
            if b:
                trace.append("|")
            trace += L[pl.order[pl.block_first[b]:pl.block_first[b + 1]]].tolist()
        seen[tuple(trace)] = seen.get(tuple(trace), 0) + 1
    assert set(seen) <= set(law)                         # nothing the law forbids
    chi2 = 0.0
    for trace, p in law.items():
        e = float(p) * runs
        chi2 += (seen.get(trace, 0) - e) ** 2 / e
    dof = len(law) - 1
    # chi-square: mean dof, variance 2*dof; five standard deviations of slack
    assert chi2 < dof + 5 * (2 * dof) ** 0.5, (chi2, dof)


def test_each_sequence_is_equally_likely_to_come_first():
    L = np.array([4, 4, 4, 2, 2, 7, 1, 1, 1, 1], np.int32)
    runs = 8000
    first = np.zeros(len(L))
    for seed in range(runs):
        first[oracle.plan_random_fit(L, 8, seed * 0x9E3779B97F4A7C15 + 3).order[0]] += 1
    e = runs / len(L)
    chi2 = float(((first - e) ** 2 / e).sum())
    dof = len(L) - 1
    assert chi2 < dof + 5 * (2 * dof) ** 0.5, (first, chi2)


@pytest.mark.parametrize("wid,n", [(2, 1000), (3, 10000), (4, 20000), (5, 60000)])
def test_pads_no_more_than_next_fit_on_the_workloads(wid, n):
    """Drawing only among what fits fills blocks at least as well as closing at the first
    misfit, on the length mixes of the workloads."""
    w = workloads.WORKLOADS[wid]
    L = workloads.lengths(wid, n)
    rf = oracle.plan_random_fit(L, w.t_blk, 0)
    nf = oracle.plan(L, w.t_blk, oracle.order(n, 0))
    check_random_fit_invariants(L, w.t_blk, rf)
    assert rf.num_blocks <= nf.num_blocks
    assert rf.num_blocks >= -(-int(L.astype(np.int64).sum()) // w.t_blk)


def test_seed_changes_the_plan_and_repeats_for_equal_seeds():
    L = workloads.random_lengths(np.random.default_rng(5), 400, 50, "mixed")
    a = oracle.plan_random_fit(L, 50, 1)
    b = oracle.plan_random_fit(L, 50, 1)
    c = oracle.plan_random_fit(L, 50, 2)
    assert np.array_equal(a.order, b.order) and np.array_equal(a.block_first, b.block_first)
    assert not np.array_equal(a.order, c.order)
