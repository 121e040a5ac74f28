"""bload_plan_random_fit on the GPU against the oracle: bit-exact order, blocks, offsets,
and the plan carried through bload_pack and bload_segment_reduce."""
import numpy as np
import pytest
import torch

import oracle
from paper_2310_10879_amd import workloads
from gpu_util import assert_packed_equal, assert_plan_equal, binding, gpu_pack_guarded, to_dev

pytestmark = pytest.mark.gpu


def gpu_random_fit(L, t_blk, seed):
    return binding().bload_plan_random_fit(to_dev(np.asarray(L, dtype=np.int32)), t_blk, seed)


@pytest.mark.parametrize("kind", ["uniform", "short", "long", "mixed"])
@pytest.mark.parametrize("n,T", [(1, 1), (1, 9), (2, 2), (3, 5), (64, 32), (255, 7), (257, 600),
                                 (1000, 600), (2049, 4096), (5000, 3), (300, 64), (300, 65),
                                 (3000, 4097), (900, 8191), (4000, 8192), (70001, 100)])
def test_random_fit_matches_oracle(kind, n, T):
    rng = np.random.default_rng(n * 11 + T)
    L = workloads.random_lengths(rng, n, T, kind)
    for seed in workloads.SHUFFLE_SEEDS:
        print(f"random fit n={n} T={T} kind={kind} seed={seed}", flush=True)
        assert_plan_equal(gpu_random_fit(L, T, seed), oracle.plan_random_fit(L, T, seed), n)


@pytest.mark.parametrize("wid", [1, 2, 3, 4, 5])
def test_random_fit_workloads_full_size(wid):
    w = workloads.WORKLOADS[wid]
    L = workloads.lengths(wid)
    seeds = workloads.SHUFFLE_SEEDS if wid < 5 else (0,)     # the oracle scans all lengths per draw
    for seed in seeds:
        print(f"random fit workload {wid} seed={seed}", flush=True)
        ref = oracle.plan_random_fit(L, w.t_blk, seed)
        assert_plan_equal(gpu_random_fit(L, w.t_blk, seed), ref, w.n_seq)


def test_random_fit_closed_forms():
    n, T = 4100, 12
    for L in (np.full(n, T), np.ones(n), np.full(n, T // 2 + 1), np.full(n, T // 2)):
        assert_plan_equal(gpu_random_fit(L, T, 5), oracle.plan_random_fit(L, T, 5), n)
    # one length per group of 64, and only the longest length
    T = 8192
    L = np.concatenate([np.arange(64, T + 1, 64), np.full(50, T), np.full(7, 1)]).astype(np.int32)
    assert_plan_equal(gpu_random_fit(L, T, 9), oracle.plan_random_fit(L, T, 9), len(L))


def test_random_fit_empty_and_errors():
    bl = binding()
    pl = gpu_random_fit(np.zeros(0, np.int32), 8, 0)
    assert pl.num_blocks == 0 and pl.total_frames == 0
    for bad in ([3, 0, 2], [3, 9, 2], [-1, 1, 1]):
        with pytest.raises(bl.BloadError) as e:
            gpu_random_fit(np.array(bad, dtype=np.int32), 8, 0)
        assert e.value.status == bl.ELENGTH
    with pytest.raises(bl.BloadError) as e:
        gpu_random_fit(np.array([1, 2], dtype=np.int32), 8193, 0)
    assert e.value.status == bl.EOVERFLOW
    L = to_dev(np.array([1, 2, 3], dtype=np.int32))
    with pytest.raises(bl.BloadError) as e:
        bl.bload_plan_random_fit(L, 8, 0, workspace=torch.empty(16, dtype=torch.uint8, device=L.device))
    assert e.value.status == bl.EWORKSPACE
    # the library still works after the refused calls
    ref = oracle.plan_random_fit(np.array([1, 2, 3], dtype=np.int32), 8, 0)
    assert_plan_equal(bl.bload_plan_random_fit(L, 8, 0), ref, 3)


def test_random_fit_is_deterministic_and_reuses_its_workspace():
    bl = binding()
    L = workloads.lengths(3)
    d_L = to_dev(L)
    ws = torch.empty(bl.bload_plan_random_fit_workspace_bytes(len(L)), dtype=torch.uint8, device=d_L.device)
    a = bl.bload_plan_random_fit(d_L, 3000, 11, workspace=ws)
    other = bl.bload_plan_random_fit(d_L, 3000, 12, workspace=ws)
    b = bl.bload_plan_random_fit(d_L, 3000, 11, workspace=ws)
    assert torch.equal(a.order, b.order) and torch.equal(a.offset_of_seq, b.offset_of_seq)
    assert torch.equal(a.block_of_seq, b.block_of_seq) and a.num_blocks == b.num_blocks
    assert not torch.equal(a.order, other.order)


@pytest.mark.parametrize("n,T,F,kind", [(300, 33, 4, "mixed"), (5000, 100, 16, "short"),
                                        (400, 64, 520, "long"), (600, 600, 4096, "uniform")])
def test_random_fit_plan_packs_and_reduces(n, T, F, kind):
    bl = binding()
    rng = np.random.default_rng(n + T + F)
    L = workloads.random_lengths(rng, n, T, kind)
    so = workloads.src_offsets(L)
    D = F // 4
    src = rng.integers(-1000, 1000, size=(int(so[-1]), D), dtype=np.int32)
    ref_plan = oracle.plan_random_fit(L, T, 3)
    ref = oracle.pack(src, so, L, ref_plan, F)
    plan_dev = gpu_random_fit(L, T, 3)
    assert_plan_equal(plan_dev, ref_plan, n)
    out = gpu_pack_guarded(src, so, L, plan_dev, F)
    assert_packed_equal(out, ref)
    red = bl.bload_segment_reduce(out.packed, out.seq_id, out.reset, out.valid, plan_dev.num_blocks,
                                  T, D, "i32", "sum", n)
    assert np.array_equal(red.cpu().numpy(), oracle.segment_reduce(src, so, L, D, "i32", "sum"))
