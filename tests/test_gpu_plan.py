"""bload_plan on the GPU against the oracle: bit-exact order, blocks, offsets."""
import numpy as np
import pytest
import torch

import oracle
from paper_2310_10879_amd import workloads
from gpu_util import assert_plan_equal, binding, gpu_plan, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kind", ["uniform", "short", "long", "mixed"])
@pytest.mark.parametrize("n,T", [(1, 1), (1, 9), (2, 2), (3, 5), (64, 32), (255, 7), (257, 600),
                                 (1000, 600), (2047, 33), (2048, 1), (2049, 4096), (5000, 3),
                                 (70001, 100),
                                 # around the tiles of the scans (2048) and of the jumping (8192)
                                 (4096, 17), (4097, 900), (8191, 2), (8192, 50), (8193, 7),
                                 (16384, 64), (16385, 300), (24577, 5)])
def test_plan_matches_oracle(kind, n, T):
    rng = np.random.default_rng(n * 7 + T)
    L = workloads.random_lengths(rng, n, T, kind)
    for seed in workloads.SHUFFLE_SEEDS:
        print(f"plan n={n} T={T} kind={kind} seed={seed}", flush=True)
        ref = oracle.plan(L, T, oracle.order(n, seed))
        assert_plan_equal(gpu_plan(L, T, seed), ref, n)


@pytest.mark.parametrize("case", range(16))
def test_plan_random_sizes_of_several_jump_tiles(case):
    # 2 .. 37 tiles of 8192 positions: every tile finds where the orbit of position 0 enters it
    rng = np.random.default_rng(9000 + case)
    n = int(rng.integers(8193, 300000))
    T = int(rng.choice([1, 3, 64, 600, 4096, 100000]))
    kind = str(rng.choice(["uniform", "short", "long", "mixed"]))
    L = workloads.random_lengths(rng, n, T, kind)
    seed = int(rng.integers(0, 2 ** 63))
    print(f"plan n={n} T={T} kind={kind} seed={seed}", flush=True)
    assert_plan_equal(gpu_plan(L, T, seed), oracle.plan(L, T, oracle.order(n, seed)), n)


@pytest.mark.parametrize("wid", [1, 2, 3, 4, 5])
def test_plan_workloads_full_size(wid):
    w = workloads.WORKLOADS[wid]
    L = workloads.lengths(wid)
    for seed in workloads.SHUFFLE_SEEDS:
        print(f"plan workload {wid} seed={seed}", flush=True)
        ref = oracle.plan(L, w.t_blk, oracle.order(w.n_seq, seed))
        assert_plan_equal(gpu_plan(L, w.t_blk, seed), ref, w.n_seq)


@pytest.mark.parametrize("n", [4100, 8192, 20000])        # one jump tile, a full one, three
def test_plan_closed_forms(n):
    # every position a block head; one block head in 12; every position; every second one
    T = 12
    for L in (np.full(n, T), np.ones(n), np.full(n, T // 2 + 1), np.full(n, T // 2)):
        L = L.astype(np.int32)
        ref = oracle.plan(L, T, oracle.order(n, 5))
        assert_plan_equal(gpu_plan(L, T, 5), ref, n)


def test_plan_empty_and_errors():
    bl = binding()
    pl = gpu_plan(np.zeros(0, np.int32), 8, 0)
    assert pl.num_blocks == 0 and pl.total_frames == 0
    for bad in ([3, 0, 2], [3, 9, 2], [-1, 1, 1]):
        with pytest.raises(bl.BloadError) as e:
            gpu_plan(np.array(bad, dtype=np.int32), 8, 0)
        assert e.value.status == bl.ELENGTH
    with pytest.raises(bl.BloadError) as e:
        gpu_plan(np.array([1, 2], dtype=np.int32), 0, 0)
    assert e.value.status == bl.EINVAL
    # workspace too small
    L = to_dev(np.array([1, 2, 3], dtype=np.int32))
    with pytest.raises(bl.BloadError) as e:
        bl.bload_plan(L, 8, 0, workspace=torch.empty(16, dtype=torch.uint8, device=L.device))
    assert e.value.status == bl.EWORKSPACE
    # the library still works after the refused calls
    ref = oracle.plan(np.array([1, 2, 3], dtype=np.int32), 8, oracle.order(3, 0))
    assert_plan_equal(bl.bload_plan(L, 8, 0), ref, 3)


def test_plan_is_deterministic():
    L = workloads.lengths(3)
    a = gpu_plan(L, 3000, 11)
    b = gpu_plan(L, 3000, 11)
    assert torch.equal(a.order, b.order) and torch.equal(a.offset_of_seq, b.offset_of_seq)
    assert torch.equal(a.block_of_seq, b.block_of_seq)
