"""Pins for the oracle's seeded order (the random choice of sequences of the Methods
section).  None of them re-types the oracle's formula: they use published known
answers, algebraic inverses, and the properties a shuffle must have."""
import numpy as np
import pytest

import oracle
from conftest import golden_rows


def test_splitmix64_known_answers():
    for seed, k, expect in golden_rows("splitmix64_kat.txt"):
        assert oracle.splitmix64(seed, k) == expect


def test_fmix32_is_undone_by_modular_inverses():
    # the finaliser is xorshift / odd multiply / xorshift / odd multiply /
    # xorshift; undo it with the multiplicative inverses mod 2^32 (computed
    # here by pow) and the xorshift inverses.  A wrong constant, shift or
    # step order does not survive this round trip.
    inv1 = pow(0x85EBCA6B, -1, 2**32)
    inv2 = pow(0xC2B2AE35, -1, 2**32)

    def unshift(h, s):
        out = h
        sh = s
        while sh < 32:
            out = h ^ (out >> s)
            sh += s
        return out & 0xFFFFFFFF

    rng = np.random.default_rng(7)
    xs = [0, 1, 0xFFFFFFFF, 0x80000000] + [int(v) for v in rng.integers(0, 2**32, 500)]
    for x in xs:
        h = oracle.fmix32(x)
        h = unshift(h, 16)
        h = (h * inv2) & 0xFFFFFFFF
        h = unshift(h, 13)
        h = (h * inv1) & 0xFFFFFFFF
        h = unshift(h, 16)
        assert h == x
    assert oracle.fmix32(0) == 0
    # avalanche: flipping one input bit flips about half of the output bits
    flips = []
    for x in xs[4:204]:
        for bit in (0, 7, 19, 31):
            flips.append(bin(oracle.fmix32(x) ^ oracle.fmix32(x ^ (1 << bit))).count("1"))
    assert 14.0 < np.mean(flips) < 18.0


@pytest.mark.parametrize("n", [0, 1, 2, 3, 4, 5, 15, 16, 17, 63, 64, 65, 255, 256, 257,
                               1000, 1023, 1024, 1025, 4097, 65536, 65537, 100003])
@pytest.mark.parametrize("seed", [0, 1, 0x9E3779B97F4A7C15, 2**64 - 1])
def test_order_is_a_bijection(n, seed):
    o = oracle.order(n, seed)
    assert o.shape == (n,)
    assert np.array_equal(np.sort(o), np.arange(n, dtype=np.int32))


def test_order_million_is_a_bijection():
    o = oracle.order(1_000_000, 0)
    seen = np.zeros(1_000_000, dtype=bool)
    seen[o] = True
    assert seen.all()


def test_order_is_deterministic_and_seed_dependent():
    a = oracle.order(1000, 42)
    b = oracle.order(1000, 42)
    c = oracle.order(1000, 43)
    assert np.array_equal(a, b)
    assert not np.array_equal(a, c)
    assert not np.array_equal(a, np.arange(1000))
    # two seeds agree on about 1/n of the positions, like independent shuffles
    assert np.mean(a == c) < 0.02


def test_order_spreads_elements_uniformly_over_seeds():
    # where sequence 0 lands, and which sequence comes first, over many seeds:
    # chi-square against the uniform law (df = n-1 = 36; 99.99% quantile ~ 76)
    n, trials = 37, 7400
    land = np.zeros(n)
    first = np.zeros(n)
    for seed in range(trials):
        o = oracle.order(n, seed)
        land[int(np.nonzero(o == 0)[0][0])] += 1
        first[o[0]] += 1
    e = trials / n
    assert np.sum((land - e) ** 2 / e) < 76.0
    assert np.sum((first - e) ** 2 / e) < 76.0


def test_order_mixes_neighbours():
    # in a shuffle the successor of i follows i immediately about once in n
    # positions, and displacement |order[p] - p| averages n/3
    n = 5000
    o = oracle.order(n, 12345).astype(np.int64)
    adj = np.mean(np.diff(o) == 1)
    assert adj < 0.005
    disp = np.mean(np.abs(o - np.arange(n)))
    assert 0.30 * n < disp < 0.37 * n
