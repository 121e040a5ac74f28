"""bload_strategy_counts on the GPU against the oracle's counts (exact integers)."""
import numpy as np
import pytest

import oracle
from paper_2310_10879_amd import workloads
from gpu_util import binding, gpu_plan, to_dev

pytestmark = pytest.mark.gpu


def expected(L, t_chunk, t_max, num_blocks, t_blk):
    samples, gone = oracle.chunk_sampling(L, t_chunk)
    longest = int(L.max()) if len(L) else 0
    pad_longest, pad_blocks = oracle.padding(L, t_max if t_max > 0 else longest, num_blocks, t_blk)
    return {"total_frames": int(L.astype(np.int64).sum()), "longest": longest,
            "pad_to_longest": pad_longest, "pad_blocks": pad_blocks if num_blocks else 0,
            "chunk_samples": samples, "chunk_deleted": gone}


@pytest.mark.parametrize("wid", [1, 2, 3, 4, 5])
def test_counts_on_the_workloads(wid):
    bl = binding()
    w = workloads.WORKLOADS[wid]
    L = workloads.lengths(wid)
    d_L = to_dev(L)
    pl = gpu_plan(L, w.t_blk, 0)
    for t_chunk in (1, max(1, int(L.mean())), w.t_blk):
        for t_max in (0, w.t_blk):
            print(f"counts workload {wid} t_chunk={t_chunk} t_max={t_max}", flush=True)
            got = bl.bload_strategy_counts(d_L, t_chunk, t_max, pl.num_blocks, w.t_blk)
            assert got == expected(L, t_chunk, t_max, pl.num_blocks, w.t_blk)


@pytest.mark.parametrize("n", [1, 63, 64, 65, 255, 257, 100003])
def test_counts_ragged_sizes(n):
    bl = binding()
    rng = np.random.default_rng(n)
    L = rng.integers(0, 500, size=n, dtype=np.int32)
    for t_chunk in (1, 3, 499, 1000):
        assert bl.bload_strategy_counts(to_dev(L), t_chunk) == expected(L, t_chunk, 0, 0, 0)


def test_counts_empty_and_errors():
    bl = binding()
    got = bl.bload_strategy_counts(to_dev(np.zeros(0, np.int32)), 5)
    assert set(got.values()) == {0}
    with pytest.raises(bl.BloadError) as e:
        bl.bload_strategy_counts(to_dev(np.array([1, 2], np.int32)), 0)
    assert e.value.status == bl.EINVAL
    # the paper's own aggregate: any set of 7464 lengths with 166785 frames padded to 94
    L = np.full(7464, 22, dtype=np.int32)
    L[:2577] += 1
    assert int(L.sum()) == 166785
    assert bl.bload_strategy_counts(to_dev(L), 22, 94)["pad_to_longest"] == 534831
