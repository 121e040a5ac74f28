"""The two largest workloads at full size, in the launch shapes the benchmark uses:
plan, packed tensor, start table and every per-sequence reduction compared whole with the
oracle (the packed tensor slab by slab), plus properties that hold at any size."""
import numpy as np
import pytest
import torch

import oracle
from paper_2310_10879_amd import workloads
from gpu_util import assert_packed_equal_whole, assert_plan_equal, binding, gpu_plan, to_dev

pytestmark = pytest.mark.gpu


def check_reduction(got, src, so, L, D, dtype, op, say=print):
    """Every row of the reduction against the oracle's (float64 accumulation over the ragged
    source): |gpu - oracle| <= 1e-5 * max(|oracle|, A), A = mean |x| of the sequence (sum |x|
    for sums).  A >= |oracle| always, so rows inside 1e-5 * |oracle| pass without A."""
    ref = oracle.segment_reduce(src, so, L, D, dtype, op)
    if dtype == "i32":
        assert np.array_equal(got, ref)
        return
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    assert np.all(np.isfinite(got))
    rows = np.nonzero((err > 1e-5 * np.abs(ref.astype(np.float64))).any(axis=1))[0]
    say(f"reduction: {len(L) - len(rows)} rows inside 1e-5 * |oracle|, {len(rows)} need the "
        f"sequence's own scale; largest error {err.max():.3g}")
    for i in rows:
        seg = np.abs(src[so[i]:so[i] + L[i]].astype(np.float64)).sum(axis=0)
        scale = seg / L[i] if op == "mean" else seg
        bound = 1e-5 * np.maximum(np.abs(ref[i].astype(np.float64)), scale)
        assert np.all(err[i] <= bound), f"sequence {i}: max err {err[i].max()} bound {bound[np.argmax(err[i])]}"


@pytest.mark.parametrize("wid", [4, 5])
def test_workload_full_size(wid, progress):
    bl = binding()
    w = workloads.WORKLOADS[wid]
    L = workloads.lengths(wid)
    so = workloads.src_offsets(L)
    progress(f"workload {wid}: drawing {int(so[-1]) * w.frame_bytes / 1e9:.1f} GB of source")
    src = workloads.source(wid, 0, int(so[-1]), threads=16)
    N, T, F, D = w.n_seq, w.t_blk, w.frame_bytes, w.frame_elems
    seed = 0
    ref_plan = oracle.plan(L, T, oracle.order(N, seed))
    progress(f"workload {wid}: plan")
    d_L = to_dev(L)
    plan_dev = gpu_plan(L, T, seed)
    assert_plan_equal(plan_dev, ref_plan, N)
    B = ref_plan.num_blocks

    progress(f"workload {wid}: upload + pack ({B} blocks)")
    d_src = torch.from_numpy(src.view(np.uint8).reshape(-1)).to("cuda:0")
    out = bl.bload_pack(d_src, to_dev(so), d_L, plan_dev, F)
    torch.cuda.synchronize()

    progress(f"workload {wid}: every block against the oracle")
    assert_packed_equal_whole(out, src, so, L, ref_plan, F, 256 if wid == 4 else 4096,
                              f"workload {wid}: ", say=progress)

    progress(f"workload {wid}: whole-tensor properties")
    valid = out.valid.view(-1).bool()
    assert int(valid.sum().item()) == int(so[-1])                     # every frame has a slot
    assert int(out.reset.sum(dtype=torch.int64).item()) == N          # one start per sequence
    assert bool(((out.frame_idx.view(-1) == 0) == out.reset.view(-1).bool()).all().item())
    sid = out.seq_id.view(-1)
    assert bool((sid[~valid] == -1).all().item()) and bool((out.frame_idx.view(-1)[~valid] == -1).all().item())
    counts = torch.bincount(sid[valid].long(), minlength=N)
    assert torch.equal(counts.cpu(), torch.from_numpy(L.astype(np.int64)))   # each sequence L_i times
    # valid slots are a prefix of every block, and inside a sequence the frame index counts up
    fill = out.valid.sum(dim=1, dtype=torch.int64)
    assert bool((out.valid == (torch.arange(T, device="cuda:0")[None, :] < fill[:, None])).all().item())
    fi = out.frame_idx.view(-1)
    same = (sid[1:] == sid[:-1]) & valid[1:] & valid[:-1]
    assert bool((fi[1:][same] == fi[:-1][same] + 1).all().item())
    # the slot of a frame is the plan's: block * T + offset + frame index
    pos = torch.nonzero(valid).view(-1)
    want = (plan_dev.block_of_seq.long()[sid[pos].long()] * T
            + plan_dev.offset_of_seq.long()[sid[pos].long()] + fi[pos].long())
    assert torch.equal(pos, want)
    del pos, want, same, counts
    # padding payload is zero, in slabs to bound temporaries
    words = out.packed.view(-1).view(torch.int32).view(B * T, F // 4)
    step = max(1, (1 << 30) // F)
    for lo in range(0, B * T, step):
        hi = min(B * T, lo + step)
        nz = (words[lo:hi] != 0).any(dim=1)
        assert not bool((nz & ~valid[lo:hi]).any().item()), f"non-zero padding in slots {lo}:{hi}"

    progress(f"workload {wid}: reduce")
    red = bl.bload_segment_reduce(out.packed, out.seq_id, out.reset, out.valid, B, T, D, w.dtype,
                                  w.op, N)
    torch.cuda.synchronize()
    check_reduction(red.cpu().numpy(), src, so, L, D, w.dtype, w.op, say=progress)
