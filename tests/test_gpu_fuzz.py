"""Seeded random configurations through the whole path (plan, pack, reduce, scan) against the
oracle: frame sizes, block lengths, length mixes and seeds that no hand-picked case lists, small
enough for the oracle to finish each in a moment."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2310_10879_amd import workloads
from gpu_util import assert_packed_equal, assert_plan_equal, binding, gpu_pack_guarded, to_dev

pytestmark = pytest.mark.gpu
EPS = 2.0 ** -24


def draw_case(rng):
    F = int(rng.choice([1, 2, 3, 4, 5, 8, 12, 16, 24, 32, 48, 60, 64, 65, 72, 96, 100, 128, 160, 200, 256,
                        300, 320, 333, 384, 500, 512, 513, 600, 768, 1000, 1024, 2048, 3000, 4096, 4100, 5000]))
    T = int(rng.choice([1, 2, 7, 16, 33, 64, 100, 255, 256, 300, 600, 1000, 2048, 3000]))
    shape = rng.choice(["tiny", "short", "uniform", "long", "mixed", "heavy"])
    budget = 24_000_000 // F                                   # packed slots the case may take
    n = int(np.clip(rng.integers(1, 4000), 1, max(1, budget // max(1, T // 2))))
    if shape == "tiny":
        L = rng.integers(1, min(T, 3) + 1, size=n)
    elif shape == "short":
        L = rng.integers(1, max(1, T // 8) + 1, size=n)
    elif shape == "uniform":
        L = rng.integers(1, T + 1, size=n)
    elif shape == "long":
        L = rng.integers(max(1, T // 2), T + 1, size=n)
    elif shape == "mixed":
        L = np.where(rng.random(n) < 0.5, rng.integers(1, max(1, T // 16) + 1, size=n), rng.integers(1, T + 1, size=n))
    else:                                                      # mostly ones, a few as long as a block
        L = np.where(rng.random(n) < 0.9, 1, T)
    return F, T, L.astype(np.int32), shape


@pytest.mark.parametrize("chunk", range(20))
def test_random_configurations(chunk):
    bl = binding()
    rng = np.random.default_rng(1000 + chunk)
    for case in range(16):
        F, T, L, shape = draw_case(rng)
        n = len(L)
        seed = int(rng.integers(0, 2 ** 63))
        planner = "random-fit" if (rng.random() < 0.3 and T <= 8192) else "next-fit"
        print(f"fuzz {chunk}.{case}: F={F} T={T} n={n} {shape} {planner} seed={seed}", flush=True)
        so = workloads.src_offsets(L)
        src = workloads.tagged_source(L, F)
        if planner == "random-fit":
            ref_plan = oracle.plan_random_fit(L, T, seed)
            plan_dev = bl.bload_plan_random_fit(to_dev(L), T, seed)
        else:
            ref_plan = oracle.plan(L, T, oracle.order(n, seed))
            plan_dev = bl.bload_plan(to_dev(L), T, seed)
        assert_plan_equal(plan_dev, ref_plan, n)
        ref = oracle.pack(src, so, L, ref_plan, F)
        out = gpu_pack_guarded(src, so, L, plan_dev, F)
        assert_packed_equal(out, ref, f"F={F} T={T} n={n} {shape}: ")
        B = ref_plan.num_blocks

        # the consumers read the bytes as u8 features (and as f32 where a frame is whole floats)
        red = bl.bload_segment_reduce(out.packed, out.seq_id, out.reset, out.valid, B, T, F, "u8", "sum", n)
        assert np.array_equal(red.cpu().numpy(), oracle.segment_reduce(src.reshape(-1, F), so, L, F, "u8", "sum"))
        h = bl.bload_segment_scan(out.packed, out.reset, out.valid, B, T, F, "u8", 0.5)
        ref_h, scale = oracle.segment_scan_packed(ref[0], ref[3], ref[4], F, "u8", 0.5)
        k = np.arange(1, T + 1, dtype=np.float64)[None, :, None]
        err = np.abs(h.cpu().numpy().astype(np.float64) - ref_h)
        assert np.all(err <= (3 * k + 4) * EPS * scale), f"scan F={F} T={T}: max err {err.max()}"
        torch.cuda.synchronize()


@pytest.mark.skipif("BLOAD_FUZZ_MORE" not in os.environ,
                    reason="set BLOAD_FUZZ_MORE=first:last to run the same checks on chunks of other seeds")
def test_more_random_configurations(progress):
    """The checks above on any further range of seeds, e.g. BLOAD_FUZZ_MORE=5000:5250 (4000
    configurations, about 7 minutes; a line per chunk goes past pytest's capture)."""
    first, last = (int(v) for v in os.environ["BLOAD_FUZZ_MORE"].split(":"))
    for chunk in range(first, last):
        test_random_configurations(chunk)
        progress(f"fuzz chunk {chunk} of {first}:{last} equal to the oracle")
