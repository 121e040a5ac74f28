"""bload_pack, bload_segment_reduce and bload_segment_scan neither synchronise nor allocate nor clear
memory through the runtime, so a caller may record them into a HIP graph: captured once, replayed
with changing source contents, every replay compared with the eager result."""
import numpy as np
import pytest
import torch

from paper_2310_10879_amd import workloads
from gpu_util import binding, gpu_plan, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("F,dtype", [(4096, "u8"), (320, "f32"), (16, "f32")])
def test_captured_pack_reduce_scan_replays_like_eager(F, dtype):
    bl = binding()
    n, T = 700, 300
    rng = np.random.default_rng(F)
    L = workloads.random_lengths(rng, n, T, "mixed")
    so = workloads.src_offsets(L)
    total = int(so[-1])
    D = F if dtype == "u8" else F // 4
    plan = gpu_plan(L, T, 3)
    B = plan.num_blocks
    d_so, d_L = to_dev(so), to_dev(L)

    def draw():
        if dtype == "u8":
            return torch.from_numpy(rng.integers(0, 256, size=total * F, dtype=np.uint8)).cuda()
        return torch.from_numpy(rng.standard_normal(total * D).astype(np.float32)).cuda()

    src = draw()
    packed = bl.alloc_packed(B, T, F, src.device)
    pack_ws = torch.empty(max(32, bl.bload_pack_workspace_bytes(n, B, T, F)), dtype=torch.uint8, device="cuda")
    red_ws = torch.empty(max(16, bl.bload_segment_reduce_workspace_bytes(B, T, D, dtype)), dtype=torch.uint8,
                         device="cuda")
    scan_ws = torch.empty(max(16, bl.bload_segment_scan_workspace_bytes(B, T, D, dtype)), dtype=torch.uint8,
                          device="cuda")
    red = torch.zeros((n, D), dtype=torch.float32, device="cuda")
    h = torch.empty((B, T, D), dtype=torch.float32, device="cuda")

    def run():
        bl.bload_pack(src, d_so, d_L, plan, F, out=packed, workspace=pack_ws)
        bl.bload_segment_reduce(packed.packed, packed.seq_id, packed.reset, packed.valid, B, T, D, dtype,
                                "mean", n, out=red, workspace=red_ws)
        bl.bload_segment_scan(packed.packed, packed.reset, packed.valid, B, T, D, dtype, 0.75, out=h,
                              workspace=scan_ws)

    run()                                   # warm up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for replay in range(3):
        print(f"graph F={F} {dtype} replay {replay}", flush=True)
        src.copy_(draw())                   # same buffers, new contents
        run()                               # eager
        torch.cuda.synchronize()
        want = [t.clone() for t in (packed.packed, packed.seq_id, packed.frame_idx, packed.reset, packed.valid,
                                    red, h)]
        for t in (packed.packed, packed.seq_id, packed.frame_idx, red, h):
            t.fill_(77)                     # what the replay must overwrite
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (packed.packed, packed.seq_id, packed.frame_idx, packed.reset, packed.valid, red, h)
        for k, (g, w) in enumerate(zip(got, want)):
            assert torch.equal(g, w), f"replay {replay}: output {k} differs from the eager run"
