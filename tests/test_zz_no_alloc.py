"""bload_pack_noalloc (the entry point for callers that cannot allocate: its scratch is a
fixed array inside the library) against bload_pack on the same inputs: all five outputs
byte for byte, on two calls in a row, the second with a smaller input (stale scratch from the
first call must not show), then the first again."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2310_10879_amd import workloads
from gpu_util import binding, gpu_plan, to_dev


def pack_both_ways(bl, n, T, F, kind, seed):
    rng = np.random.default_rng(seed)
    L = workloads.random_lengths(rng, n, T, kind)
    so = workloads.src_offsets(L)
    g = torch.Generator(device="cuda:0").manual_seed(seed)
    src = torch.randint(0, 256, (int(so[-1]) * F,), dtype=torch.uint8, device="cuda:0", generator=g)
    d_L, d_so = to_dev(L), to_dev(so)
    plan = gpu_plan(L, T, seed)
    want = bl.bload_pack(src, d_so, d_L, plan, F)
    got = bl.alloc_packed(plan.num_blocks, T, F, src.device)
    for t in (got.packed, got.seq_id, got.frame_idx, got.reset, got.valid):
        t.fill_(0x5A if t.dtype == torch.uint8 else 0x5A5A5A5A)      # garbage the call must overwrite
    count = lambda: torch.cuda.memory_stats()["allocation.all.allocated"]   # allocations made so far
    before = count()
    bl.bload_pack_noalloc(src, d_so, d_L, plan, F, got)
    assert count() == before                                           # nothing came from torch either
    torch.cuda.synchronize()
    for name in ("packed", "seq_id", "frame_idx", "reset", "valid"):
        assert torch.equal(getattr(got, name), getattr(want, name)), f"{name} differs (n={n} T={T} F={F})"
    return plan


@pytest.mark.gpu
def test_noalloc_pack_equals_pack_on_consecutive_calls():
    bl = binding()
    big = pack_both_ways(bl, 4000, 600, 4096, "uniform", 1)        # 4 KiB tiles: ~6 GB, ~1.6 M of them
    assert bl.bload_pack_tile_bytes(4000, big.num_blocks, 600, 4096) == 4096
    assert big.num_blocks * 600 > bl.PACK_NOALLOC_MAX_TILES // 2
    pack_both_ways(bl, 700, 300, 4096, "mixed", 2)                 # smaller, same tile shape
    wide = pack_both_ways(bl, 3000, 1000, 68, "long", 5)           # 4 KiB tiles and the start table in a pass of its own
    assert bl.bload_pack_tile_bytes(3000, wide.num_blocks, 1000, 68) == 4096 and wide.num_blocks * 1000 >= 1 << 21
    pack_both_ways(bl, 200000, 64, 4, "short", 3)                  # 1024-slot tiles, many runs
    pack_both_ways(bl, 300, 33, 12, "mixed", 4)                    # smaller again
    pack_both_ways(bl, 4000, 600, 4096, "uniform", 1)              # and the first once more


def test_noalloc_pack_refuses_what_its_array_cannot_hold():
    # host-side checks: answered before any GPU call
    bl = binding()
    lib = ctypes.CDLL(bl.LIB_PATH)
    f = lib.bload_pack_noalloc
    f.restype = ctypes.c_int
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    f.argtypes = [vp] * 7 + [i64, i64, i32, i64] + [vp] * 5 + [vp]
    p = 0x2000
    ok = [p] * 7
    outs = [p] * 5
    assert f(*ok, (1 << 18) + 1, 10, 8, 16, *outs, None) == bl.EOVERFLOW          # too many sequences
    assert f(*ok, 1000, 1000, 3000, 4096, *outs, None) == bl.EOVERFLOW            # 12 GB: too many 4 KiB tiles
    assert f(*ok, 1000, 10, 0, 16, *outs, None) == bl.EINVAL
    assert f(None, *ok[1:], 1000, 10, 8, 16, *outs, None) == bl.EINVAL
    assert f(*ok, 1000, 10, 8, 16, p + 4, *outs[1:], None) == bl.EALIGN
    assert f(*ok, 0, 0, 8, 16, *outs, None) == bl.OK
