"""bload_pack on the GPU against the oracle: bit-exact packed tensor and start table."""
import numpy as np
import pytest
import torch

import oracle
from paper_2310_10879_amd import workloads
from gpu_util import (assert_packed_equal, binding, gpu_pack_guarded, gpu_plan, to_dev,
                      upload_plan)

pytestmark = pytest.mark.gpu

FRAME_BYTES = [1, 2, 3, 4, 6, 8, 12, 16, 20, 48, 64, 100, 255, 256, 257, 320, 1000, 3072, 4100]


def run_case(n, T, F, kind, seed, plan_from="oracle"):
    rng = np.random.default_rng(n * 31 + T * 7 + F)
    L = workloads.random_lengths(rng, n, T, kind)
    so = workloads.src_offsets(L)
    src = workloads.tagged_source(L, F)
    ref_plan = oracle.plan(L, T, oracle.order(n, seed))
    ref = oracle.pack(src, so, L, ref_plan, F)
    plan_dev = upload_plan(ref_plan, n) if plan_from == "oracle" else gpu_plan(L, T, seed)
    out = gpu_pack_guarded(src, so, L, plan_dev, F)
    assert_packed_equal(out, ref, f"n={n} T={T} F={F} {kind}: ")


@pytest.mark.parametrize("F", FRAME_BYTES)
def test_pack_frame_sizes_with_oracle_plan(F):
    # several tiles of both kernels, ragged tails, blocks not a multiple of anything
    for n, T, kind in [(1, 1, "uniform"), (5, 7, "uniform"), (300, 33, "mixed"),
                       (700, 130, "short"), (90, 1500, "uniform")]:
        if n * T * F > 200_000_000:
            continue
        print(f"pack F={F} n={n} T={T} {kind}", flush=True)
        run_case(n, T, F, kind, seed=1)


@pytest.mark.parametrize("F", [4, 16, 320, 4096])
def test_pack_with_device_plan(F):
    for n, T, kind in [(64, 32, "uniform"), (3000, 100, "mixed"), (2500, 4096, "short")]:
        if n * T * F > 400_000_000:
            continue
        print(f"plan+pack F={F} n={n} T={T} {kind}", flush=True)
        run_case(n, T, F, kind, seed=0, plan_from="gpu")


@pytest.mark.parametrize("F", [64, 65, 100, 256, 320, 333, 500, 511])
def test_pack_middle_frames_take_either_tile_shape(F):
    """Frames of 64..511 bytes go through the 4 KiB tiles when sequences are long and through the
    1024-slot tiles when they are short: both, and the mixes in between, against the oracle."""
    for n, T, lo, hi in [(40, 2000, 1000, 2000),      # every run far longer than a tile
                         (3000, 64, 1, 3),            # dozens of runs in every 4 KiB
                         (600, 300, 40, 120),         # a few tiles per run
                         (400, 700, 1, 700)]:         # everything at once
        rng = np.random.default_rng(F * 13 + n)
        L = rng.integers(lo, hi + 1, size=n).astype(np.int32)
        so = workloads.src_offsets(L)
        src = workloads.tagged_source(L, F)
        ref_plan = oracle.plan(L, T, oracle.order(n, 5))
        ref = oracle.pack(src, so, L, ref_plan, F)
        print(f"pack F={F} n={n} T={T} L in [{lo}, {hi}]", flush=True)
        out = gpu_pack_guarded(src, so, L, upload_plan(ref_plan, n), F)
        assert_packed_equal(out, ref, f"F={F} n={n} T={T}: ")


def test_pack_degenerate_blocks():
    # every block full, every block one frame, blocks of unit sequences
    for n, T, L in [(50, 8, np.full(50, 8)), (50, 8, np.ones(50)), (50, 8, np.full(50, 5)),
                    (3000, 4096, np.ones(3000)), (3, 5000, np.full(3, 5000))]:
        for F in (4, 12, 512):
            L = L.astype(np.int32)
            so = workloads.src_offsets(L)
            src = workloads.tagged_source(L, F)
            ref_plan = oracle.plan(L, T, oracle.order(n, 2))
            ref = oracle.pack(src, so, L, ref_plan, F)
            print(f"pack degenerate n={n} T={T} F={F} L0={L[0]}", flush=True)
            out = gpu_pack_guarded(src, so, L, upload_plan(ref_plan, n), F)
            assert_packed_equal(out, ref)


def test_pack_unaligned_source_base():
    # the ragged source may start at any byte address
    bl = binding()
    n, T = 200, 50
    rng = np.random.default_rng(4)
    L = workloads.random_lengths(rng, n, T, "uniform")
    so = workloads.src_offsets(L)
    for F, shift in [(300, 1), (300, 4), (6, 2), (7, 3), (1024, 8)]:
        src = workloads.tagged_source(L, F)
        ref_plan = oracle.plan(L, T, oracle.order(n, 3))
        ref = oracle.pack(src, so, L, ref_plan, F)
        plan_dev = upload_plan(ref_plan, n)
        big = torch.zeros(src.size + 64, dtype=torch.uint8, device="cuda:0")
        view = big[shift:shift + src.size]
        view.copy_(to_dev(src.reshape(-1)))
        print(f"pack unaligned F={F} shift={shift}", flush=True)
        out = bl.bload_pack(view, to_dev(so), to_dev(L), plan_dev, F)
        torch.cuda.synchronize()
        assert_packed_equal(out, ref)


def test_pack_empty_and_errors():
    bl = binding()
    L = np.array([2, 3], dtype=np.int32)
    so = workloads.src_offsets(L)
    src = workloads.tagged_source(L, 8)
    plan_dev = gpu_plan(L, 4, 0)
    good = bl.bload_pack(to_dev(src.reshape(-1)), to_dev(so), to_dev(L), plan_dev, 8)
    # misaligned packed buffer
    raw = torch.empty(plan_dev.num_blocks * 4 * 8 + 16, dtype=torch.uint8, device="cuda:0")
    out = bl.alloc_packed(plan_dev.num_blocks, 4, 8, raw.device)
    out.packed = raw[1:1 + plan_dev.num_blocks * 4 * 8].view(plan_dev.num_blocks, 4, 8)
    with pytest.raises(bl.BloadError) as e:
        bl.bload_pack(to_dev(src.reshape(-1)), to_dev(so), to_dev(L), plan_dev, 8, out)
    assert e.value.status == bl.EALIGN
    assert good.valid.sum().item() == 5


@pytest.mark.parametrize("wid", [1, 2, 3])
def test_pack_workloads_full_size(wid):
    # workloads 1-3 whole, every byte compared (seed 0 = the configuration the benchmark times)
    w = workloads.WORKLOADS[wid]
    L = workloads.lengths(wid)
    so = workloads.src_offsets(L)
    src = workloads.source(wid, 0, int(so[-1]))
    for seed in (workloads.SHUFFLE_SEEDS if wid == 1 else (0,)):
        print(f"pack workload {wid} seed={seed}", flush=True)
        ref_plan = oracle.plan(L, w.t_blk, oracle.order(w.n_seq, seed))
        plan_dev = gpu_plan(L, w.t_blk, seed)
        bl = binding()
        out = bl.bload_pack(to_dev(src.view(np.uint8).reshape(-1)), to_dev(so), to_dev(L),
                            plan_dev, w.frame_bytes)
        torch.cuda.synchronize()
        # compare in slabs of blocks to bound host memory
        step = max(1, (256 << 20) // (w.t_blk * w.frame_bytes))
        for lo in range(0, ref_plan.num_blocks, step):
            hi = min(lo + step, ref_plan.num_blocks)
            ref = oracle.pack_blocks(src, so, L, ref_plan, w.frame_bytes, lo, hi)
            got = bl.Packed(out.packed[lo:hi], out.seq_id[lo:hi], out.frame_idx[lo:hi],
                            out.reset[lo:hi], out.valid[lo:hi])
            assert_packed_equal(got, ref, f"workload {wid} blocks {lo}:{hi} ")


@pytest.mark.parametrize("n,T,F,kind", [(3000, 1000, 68, "long"),      # frames no vector load fits, long runs
                                        (2000, 3000, 320, "uniform"),  # the shape of the largest workload
                                        (70000, 64, 516, "mixed")])    # many short runs per tile, blocks of 64
def test_pack_large_tensors_of_wide_frames(n, T, F, kind, progress):
    """From 2^21 slots on, 4 KiB tiles copy the payload and a pass of its own writes the start
    table: every block against the oracle, slab by slab."""
    from gpu_util import assert_packed_equal_whole
    bl = binding()
    rng = np.random.default_rng(n + T + F)
    L = workloads.random_lengths(rng, n, T, kind)
    so = workloads.src_offsets(L)
    src = rng.integers(0, 256, size=int(so[-1]) * F, dtype=np.uint8)
    ref_plan = oracle.plan(L, T, oracle.order(n, 2))
    assert ref_plan.num_blocks * T >= 1 << 21
    assert bl.bload_pack_tile_bytes(n, ref_plan.num_blocks, T, F, True) == 4096
    plan_dev = upload_plan(ref_plan, n)
    out = bl.bload_pack(to_dev(src), to_dev(so), to_dev(L), plan_dev, F)
    torch.cuda.synchronize()
    assert_packed_equal_whole(out, src, so, L, ref_plan, F, max(1, (64 << 20) // (T * F)),
                              f"n={n} T={T} F={F} {kind}: ", say=progress)


@pytest.mark.parametrize("n,T,F,kind", [(400000, 256, 4, "mixed"),     # tokens: payload and table share a quad per lane
                                        (3000, 4096, 4, "long"),       # tokens: most tiles inside one run or inside padding
                                        (5000, 3000, 4, "mixed"),      # tokens: blocks that are no whole number of tiles
                                        (2052, 1025, 4, "long"),       # tokens: an odd number of tiles, the last one short
                                        (300000, 100, 6, "uniform"),   # 2-byte elements
                                        (500000, 33, 12, "uniform"),   # 4-byte elements, blocks not a multiple of anything
                                        (100000, 300, 48, "mixed"),    # 16-byte vectors
                                        (2500000, 7, 1, "short")])     # bytes, blocks far shorter than a tile
def test_pack_large_tensors_of_small_frames(n, T, F, kind, progress):
    """Large tensors in slot tiles (from 2^21 slots on, 4-byte frames are written in two passes,
    payload and start table): every block against the oracle, slab by slab."""
    from gpu_util import assert_packed_equal_whole
    bl = binding()
    rng = np.random.default_rng(n + T + F)
    L = workloads.random_lengths(rng, n, T, kind)
    so = workloads.src_offsets(L)
    src = rng.integers(0, 256, size=int(so[-1]) * F, dtype=np.uint8)
    ref_plan = oracle.plan(L, T, oracle.order(n, 3))
    assert ref_plan.num_blocks * T >= 1 << 21
    assert bl.bload_pack_tile_bytes(n, ref_plan.num_blocks, T, F, True) == 0
    plan_dev = upload_plan(ref_plan, n)
    out = bl.bload_pack(to_dev(src), to_dev(so), to_dev(L), plan_dev, F)
    torch.cuda.synchronize()
    assert_packed_equal_whole(out, src, so, L, ref_plan, F, max(1, (64 << 20) // (T * F)),
                              f"n={n} T={T} F={F} {kind}: ", say=progress)
