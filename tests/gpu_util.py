"""Helpers shared by the GPU parity tests: upload seeded inputs, run the HIP
library through its binding, bring results back as numpy."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

import oracle
from paper_2310_10879_amd import workloads


def binding():
    from paper_2310_10879_amd import bload       # raises if libbload.so is missing
    return bload


def dev():
    return torch.device("cuda:0")


def to_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev())


def gpu_plan(L: np.ndarray, t_blk: int, seed: int):
    bl = binding()
    return bl.bload_plan(to_dev(L.astype(np.int32)), t_blk, seed)


def assert_plan_equal(pl_gpu, pl_ref: oracle.Plan, n: int):
    assert pl_gpu.num_blocks == pl_ref.num_blocks
    assert pl_gpu.total_frames == pl_ref.total_frames
    assert np.array_equal(pl_gpu.order.cpu().numpy(), pl_ref.order)
    assert np.array_equal(pl_gpu.block_of_seq.cpu().numpy(), pl_ref.block_of_seq)
    assert np.array_equal(pl_gpu.offset_of_seq.cpu().numpy(), pl_ref.offset_of_seq)
    if n:
        assert np.array_equal(pl_gpu.block_first.cpu().numpy()[:pl_ref.num_blocks + 1],
                              pl_ref.block_first)


def upload_plan(pl_ref: oracle.Plan, n: int):
    """An oracle plan as the binding's device-side Plan (to test the packer alone)."""
    bl = binding()
    bf = np.zeros(n + 1, dtype=np.int32)
    bf[:pl_ref.num_blocks + 1] = pl_ref.block_first
    return bl.Plan(to_dev(pl_ref.order), to_dev(pl_ref.block_of_seq), to_dev(pl_ref.offset_of_seq),
                   to_dev(bf), pl_ref.num_blocks, pl_ref.total_frames, pl_ref.t_blk)


class Guarded:
    """A device buffer with canary bytes before and after the part handed to the library."""
    PAD = 256

    def __init__(self, nbytes: int, fill: int = 0xCD):
        self.nbytes = nbytes
        self.raw = torch.full((nbytes + 2 * self.PAD,), fill, dtype=torch.uint8, device=dev())
        self.fill = fill

    def view(self, dtype, shape):
        return self.raw[self.PAD:self.PAD + self.nbytes].view(dtype).view(shape)

    def intact(self) -> bool:
        a = self.raw[:self.PAD]
        b = self.raw[self.PAD + self.nbytes:]
        return bool((a == self.fill).all().item() and (b == self.fill).all().item())


def gpu_pack_guarded(src: np.ndarray, so: np.ndarray, L: np.ndarray, plan_dev, frame_bytes: int):
    """Run bload_pack into canary-guarded, garbage-prefilled outputs."""
    bl = binding()
    B, T = plan_dev.num_blocks, plan_dev.t_blk
    slots = B * T
    g = [Guarded(slots * frame_bytes), Guarded(slots * 4), Guarded(slots * 4), Guarded(slots),
         Guarded(slots)]
    out = bl.Packed(g[0].view(torch.uint8, (B, T, frame_bytes)), g[1].view(torch.int32, (B, T)),
                    g[2].view(torch.int32, (B, T)), g[3].view(torch.uint8, (B, T)),
                    g[4].view(torch.uint8, (B, T)))
    src_b = np.ascontiguousarray(src).view(np.uint8).reshape(-1)
    bl.bload_pack(to_dev(src_b), to_dev(so), to_dev(L.astype(np.int32)), plan_dev, frame_bytes, out)
    torch.cuda.synchronize()
    assert all(x.intact() for x in g), "bload_pack wrote outside its output buffers"
    return out


def assert_packed_equal(out, ref, what=""):
    names = ["packed", "seq_id", "frame_idx", "reset", "valid"]
    got = [out.packed, out.seq_id, out.frame_idx, out.reset, out.valid]
    for name, g, r in zip(names, got, ref):
        gn = g.cpu().numpy()
        if not np.array_equal(gn, r):
            bad = np.argwhere(gn != r)
            raise AssertionError(f"{what}{name}: {len(bad)} mismatches, first at {bad[0].tolist()} "
                                 f"got {gn[tuple(bad[0])]} want {r[tuple(bad[0])]}")


def assert_packed_equal_whole(out, src, so, L, ref_plan, frame_bytes, slab_blocks, what="", workers=8,
                              say=print):
    """Compare ALL blocks of a packed tensor (payload and the four planes of the start table)
    with the oracle, slab by slab: the oracle packs blocks [lo, hi) on the host (several slabs
    at a time on separate threads, each a call of its own), the slab is uploaded and compared
    on the device.  Bounded host memory: `workers` slabs."""
    B = ref_plan.num_blocks
    slabs = [(lo, min(B, lo + slab_blocks)) for lo in range(0, B, slab_blocks)]

    def make(rng):
        return rng, oracle.pack_blocks(src, so, L, ref_plan, frame_bytes, rng[0], rng[1])

    done = 0
    with ThreadPoolExecutor(max_workers=workers) as ex:
        # a bounded window of slabs in flight
        for start in range(0, len(slabs), workers):
            for (lo, hi), ref in ex.map(make, slabs[start:start + workers]):
                got = (out.packed[lo:hi], out.seq_id[lo:hi], out.frame_idx[lo:hi], out.reset[lo:hi],
                       out.valid[lo:hi])
                same = all(torch.equal(g, torch.from_numpy(r).to(g.device)) for g, r in zip(got, ref))
                if not same:
                    binding_out = binding().Packed(*got)
                    assert_packed_equal(binding_out, ref, f"{what}blocks {lo}:{hi}: ")
                    raise AssertionError(f"{what}blocks {lo}:{hi} differ")
                done += hi - lo
            say(f"{what}{done} of {B} blocks equal to the oracle's")
    assert done == B
