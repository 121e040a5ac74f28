"""bload_segment_scan on the GPU against the oracle's recurrence, element by element.

Bound used throughout (float32 arithmetic in time order, states handed across chunks of time as
decay^chunk * state + the chunk's own part, against the oracle's double): at the k-th slot of a
block (k counted from 1, an upper bound of the frame's place in its sequence)
|gpu - oracle| <= (3k + 4) * 2^-24 * S, S = the same recurrence on |x| with |decay|.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2310_10879_amd import workloads
from gpu_util import binding, gpu_plan, to_dev
from test_gpu_reduce import draw_source, random_flags

pytestmark = pytest.mark.gpu
EPS = 2.0 ** -24


def assert_scan_close(got, ref, scale, what):
    B, T, D = ref.shape
    k = np.arange(1, T + 1, dtype=np.float64)[None, :, None]
    bound = (3 * k + 4) * EPS * scale.astype(np.float64)
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    bad = err > bound
    if bad.any():
        at = tuple(np.argwhere(bad)[0])
        raise AssertionError(f"{what}: {int(bad.sum())} outside the bound, first at {at}: got {got[at]} "
                             f"want {ref[at]} bound {bound[at]}")


def gpu_scan(packed_np, reset, valid, D, dtype, decay):
    bl = binding()
    B, T = valid.shape
    out = torch.full((B, T, D), float("nan"), dtype=torch.float32, device="cuda")
    bl.bload_segment_scan(to_dev(packed_np.view(np.uint8).reshape(-1)), to_dev(reset), to_dev(valid), B, T, D,
                          dtype, decay, out=out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("dtype", ["u8", "f16", "f32"])
@pytest.mark.parametrize("B,T,D", [(1, 1, 1), (3, 10, 1), (700, 33, 1), (40, 5000, 1), (9, 4096, 2),
                                   (70, 130, 3), (300, 130, 16), (50, 700, 80), (60, 300, 100),
                                   (20, 3000, 256), (64, 32, 3072), (5, 257, 1040),
                                   # fewer than 8 slots in all, exactly 8, blocks shorter than 8 slots
                                   (2, 3, 5), (1, 7, 4), (1, 8, 4), (3, 5, 8), (11, 7, 16)])
def test_scan_follows_the_flags(B, T, D, dtype):
    rng = np.random.default_rng(B + T + D)
    for (p_valid, p_reset), decay in zip([(0.85, 0.02), (0.5, 0.3), (1.0, 0.0)], [0.9, -0.5, 1.0]):
        print(f"scan B={B} T={T} D={D} {dtype} valid {p_valid} reset {p_reset} decay {decay}", flush=True)
        valid, reset, _, _ = random_flags(rng, B, T, p_valid, p_reset)
        src = draw_source(rng, B * T, D, dtype)            # payload in every slot, padding included
        ref, scale = oracle.segment_scan_packed(src, reset, valid, D, dtype, decay)
        got = gpu_scan(src, reset, valid, D, dtype, decay)
        assert not got[valid == 0].any()                   # padding yields exact zeros
        assert_scan_close(got, ref, scale, f"{dtype} B={B} T={T} D={D}")


@pytest.mark.parametrize("wid", [1, 2, 3])
def test_scan_of_packed_workloads(wid):
    """Plan, pack and scan on the GPU; the oracle's recurrence on the ragged source, carried to the
    slots through the oracle's own pack tables, is the reference (sampled blocks at full size)."""
    bl = binding()
    w = workloads.WORKLOADS[wid]
    L = workloads.lengths(wid)
    so = workloads.src_offsets(L)
    src = workloads.source(wid, 0, int(so[-1]))
    D, T, F = w.frame_elems, w.t_blk, w.frame_bytes
    plan_dev = gpu_plan(L, T, 0)
    d_src = to_dev(src.view(np.uint8).reshape(-1))
    out = bl.bload_pack(d_src, to_dev(so), to_dev(L), plan_dev, F)
    decay = 0.97
    h = bl.bload_segment_scan(out.packed, out.reset, out.valid, plan_dev.num_blocks, T, D, w.dtype, decay)
    torch.cuda.synchronize()
    ref_plan = oracle.plan(L, T, oracle.order(w.n_seq, 0))
    rng = np.random.default_rng(wid)
    blocks = sorted(set([0, ref_plan.num_blocks - 1] +
                        rng.integers(0, ref_plan.num_blocks, size=6).tolist()))
    for b in blocks:
        print(f"scan workload {wid} block {b}", flush=True)
        packed, seq_id, frame_idx, reset, valid = oracle.pack_blocks(src, so, L, ref_plan, F, b, b + 1)
        seqs = ref_plan.order[ref_plan.block_first[b]:ref_plan.block_first[b + 1]]
        ref = np.zeros((1, T, D), np.float32)
        scale = np.zeros((1, T, D), np.float32)
        for i in seqs:                                      # the ragged definition, sequence by sequence
            hi, si = oracle.segment_scan(src[so[i]:so[i + 1]], np.array([0, L[i]]), L[i:i + 1], D, w.dtype, decay)
            o = ref_plan.offset_of_seq[i]
            ref[0, o:o + L[i]] = hi
            scale[0, o:o + L[i]] = si
        got = h[b:b + 1].cpu().numpy()
        assert not got[valid == 0].any()
        assert_scan_close(got, ref, scale, f"workload {wid} block {b}")


def test_scan_closed_forms_and_determinism():
    bl = binding()
    B, T, D = 7, 200, 64
    valid = np.ones((B, T), np.uint8)
    reset = np.zeros((B, T), np.uint8)
    reset[:, ::20] = 1
    x = np.full((B, T, D), 3.0, np.float32)
    t_in_seg = (np.arange(T) % 20)[None, :, None]
    for decay, want in ((0.0, x), (1.0, 3.0 * (t_in_seg + 1) + 0 * x), (0.5, 6.0 * (1 - 0.5 ** (t_in_seg + 1)) + 0 * x)):
        got = gpu_scan(x, reset, valid, D, "f32", decay)
        assert np.array_equal(got, want.astype(np.float32))       # all exact in float32
    rng = np.random.default_rng(1)
    x = rng.normal(size=(B, T, D)).astype(np.float32)
    a = gpu_scan(x, reset, valid, D, "f32", 0.8)
    b = gpu_scan(x, reset, valid, D, "f32", 0.8)
    assert np.array_equal(a, b)
    # a non-finite state does not leak across a start
    x[:, 19] = np.inf
    got = gpu_scan(x, reset, valid, D, "f32", 0.8)
    assert np.isfinite(got[:, 20:]).all() and np.isinf(got[:, 19]).all()


def test_scan_errors():
    bl = binding()
    z = torch.zeros(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(bl.BloadError) as e:
        bl.bload_segment_scan(z, z, z, 1, 4, 4, "i32", 0.5)
    assert e.value.status == bl.EINVAL
    with pytest.raises(bl.BloadError) as e:
        bl.bload_segment_scan(z[1:], z, z, 1, 4, 4, "f32", 0.5)
    assert e.value.status == bl.EALIGN
    assert bl.bload_segment_scan(z, z, z, 0, 4, 4, "f32", 0.5).numel() == 0
