"""bload_plan_shard on the GPU: a worker's share of the plan equals the oracle's, and packing /
reducing it gives that worker's rows of the whole packed tensor and of the whole reduction."""
import numpy as np
import pytest
import torch

import oracle
from paper_2310_10879_amd import workloads
from gpu_util import assert_packed_equal, binding, gpu_plan, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("world", [1, 2, 3, 8])
@pytest.mark.parametrize("n,T,F,kind", [(1, 4, 8, "uniform"), (300, 33, 4, "mixed"),
                                        (5000, 100, 16, "short"), (400, 64, 520, "long"),
                                        (1000, 600, 4096, "uniform")])
def test_shard_plan_pack_reduce(world, n, T, F, kind):
    bl = binding()
    if n * T * F > 300_000_000:
        n = 300_000_000 // (T * F)
    rng = np.random.default_rng(n + T + F + world)
    L = workloads.random_lengths(rng, n, T, kind)
    so = workloads.src_offsets(L)
    D = F // 4
    src = rng.integers(-1000, 1000, size=(int(so[-1]), D), dtype=np.int32)
    seed = 7
    ref_plan = oracle.plan(L, T, oracle.order(n, seed))
    whole = oracle.pack(src, so, L, ref_plan, F)
    ref_red = oracle.segment_reduce(src, so, L, D, "i32", "sum")
    plan_dev = gpu_plan(L, T, seed)
    d_src, d_so, d_L = to_dev(src.view(np.uint8).reshape(-1)), to_dev(so), to_dev(L)
    B = ref_plan.num_blocks
    for rank in range(world):
        print(f"shard n={n} T={T} F={F} {kind} rank {rank}/{world}", flush=True)
        ref_sh = oracle.plan_shard(ref_plan, rank, world)
        sh = bl.bload_plan_shard(plan_dev, rank, world)
        assert sh.num_blocks == ref_sh.num_blocks and sh.n_local == ref_sh.n_local
        assert np.array_equal(sh.order.cpu().numpy(), ref_sh.order)
        assert np.array_equal(sh.block_of_seq.cpu().numpy(), ref_sh.block_of_seq)
        assert np.array_equal(sh.block_first.cpu().numpy(), ref_sh.block_first)
        out = bl.bload_pack(d_src, d_so, d_L, sh, F)
        torch.cuda.synchronize()
        rows = [j * world + rank for j in range(sh.num_blocks)]
        want = []
        for k, ref in enumerate(whole):
            pad = {0: 0, 1: -1, 2: -1, 3: 0, 4: 0}[k]
            want.append(np.stack([ref[b] if b < B else np.full_like(ref[0], pad) for b in rows]))
        assert_packed_equal(out, want, f"rank {rank}/{world}: ")
        red = bl.bload_segment_reduce(out.packed, out.seq_id, out.reset, out.valid, sh.num_blocks,
                                      T, D, "i32", "sum", n)
        mine = ref_sh.block_of_seq >= 0
        got = red.cpu().numpy()
        assert np.array_equal(got[mine], ref_red[mine])
        assert not got[~mine].any()                   # other workers' rows are left untouched (zeros)


def test_shard_errors():
    bl = binding()
    plan_dev = gpu_plan(np.array([2, 3, 1], dtype=np.int32), 4, 0)
    for rank, world in [(2, 2), (-1, 2), (0, 0)]:
        with pytest.raises(bl.BloadError) as e:
            bl.bload_plan_shard(plan_dev, rank, world)
        assert e.value.status == bl.EINVAL
