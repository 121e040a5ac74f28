"""bload_segment_reduce on the GPU against the oracle's per-sequence sums / means
(computed in float64 from the ragged source, never from the packed tensor)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2310_10879_amd import workloads
from gpu_util import binding, gpu_plan, to_dev

pytestmark = pytest.mark.gpu

NP_OF = {"u8": np.uint8, "f16": np.float16, "f32": np.float32, "i32": np.int32}
REL_TOL = 1e-5          # the bar for float32 reductions


def draw_source(rng, total, D, dtype):
    if dtype == "u8":
        return rng.integers(0, 256, size=(total, D), dtype=np.uint8)
    if dtype == "f16":
        return rng.standard_normal((total, D), dtype=np.float32).astype(np.float16)
    if dtype == "f32":
        return (rng.standard_normal((total, D), dtype=np.float32) * 2 - 4).astype(np.float32)
    return rng.integers(-2_000_000_000, 2_000_000_000, size=(total, D), dtype=np.int32)


def check_reduction(got, src, so, L, D, dtype, op):
    """|gpu - oracle| <= 1e-5 * max(|oracle|, A), A = mean|x| (mean) or sum|x| (sum) of the
    segment: the relative bar, with the scale of the summands as floor because a
    mean near zero has no relative accuracy in any finite-precision sum."""
    ref = oracle.segment_reduce(src, so, L, D, dtype, op)
    if dtype == "i32":
        assert got.dtype == np.int64
        assert np.array_equal(got, ref)
        return
    assert got.dtype == np.float32
    scale = np.add.reduceat(np.abs(src.astype(np.float64)), so[:-1], axis=0)
    if op == "mean":
        scale = scale / L[:, None]
    bound = REL_TOL * np.maximum(np.abs(ref.astype(np.float64)), scale)
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    assert np.all(err <= bound), (f"worst at {worst}: got {got[worst]} want {ref[worst]} "
                                  f"err {err[worst]} bound {bound[worst]}")
    if dtype == "u8":
        if op == "sum":         # integer sums below 2^24 are exact in float32
            assert np.array_equal(got, ref)
        else:                   # one rounding of an exact quotient on either side
            assert np.all(err <= np.spacing(np.abs(ref)))


def reduce_case(n, T, D, dtype, op, kind, seed=0, poison=False):
    bl = binding()
    rng = np.random.default_rng(n * 13 + T * 5 + D)
    L = workloads.random_lengths(rng, n, T, kind)
    so = workloads.src_offsets(L)
    src = draw_source(rng, int(so[-1]), D, dtype)
    F = D * src.dtype.itemsize
    pl = oracle.plan(L, T, oracle.order(n, seed))
    packed, seq_id, frame_idx, reset, valid = oracle.pack(src, so, L, pl, F)
    if poison:      # garbage in the padding payload must not reach any sum
        packed = packed.copy()
        packed[valid == 0] = 0x7B
    out = bl.bload_segment_reduce(to_dev(packed), to_dev(seq_id), to_dev(reset), to_dev(valid),
                                  pl.num_blocks, T, D, dtype, op, n)
    torch.cuda.synchronize()
    check_reduction(out.cpu().numpy(), src, so, L, D, dtype, op)
    return out


CASES = [  # n, T, D: wide rows of every width, several time chunks, narrow tiles across blocks
    (1, 1, 1), (5, 7, 1), (300, 33, 1), (40, 5000, 1), (2000, 100, 1), (90, 4096, 1),
    (300, 33, 3), (60, 600, 5), (64, 32, 16), (64, 32, 17), (200, 130, 64), (100, 300, 80),
    (150, 64, 100), (80, 200, 192), (30, 3000, 256), (25, 700, 300), (12, 3000, 2048),
    (64, 32, 3072),
]


@pytest.mark.parametrize("dtype,op", [("u8", "mean"), ("u8", "sum"), ("f16", "mean"),
                                      ("f32", "mean"), ("f32", "sum"), ("i32", "sum")])
@pytest.mark.parametrize("n,T,D", CASES)
def test_reduce_matches_oracle(n, T, D, dtype, op):
    if n * T * D > 60_000_000:
        n = max(1, 60_000_000 // (T * D))
    for kind in ("uniform", "mixed"):
        print(f"reduce n={n} T={T} D={D} {dtype} {op} {kind}", flush=True)
        reduce_case(n, T, D, dtype, op, kind)


@pytest.mark.parametrize("n,T,D,dtype", [(200, 130, 64, "f32"), (300, 33, 1, "i32"),
                                         (30, 3000, 256, "u8"), (40, 5000, 2, "f16")])
def test_reduce_ignores_padding_payload(n, T, D, dtype):
    reduce_case(n, T, D, dtype, "sum", "uniform", poison=True)


def test_reduce_long_and_short_segments():
    for kind in ("short", "long"):
        reduce_case(3000, 4096, 1, "i32", "sum", kind)
        reduce_case(400, 512, 128, "f32", "mean", kind)


def test_reduce_closed_forms():
    # payload = sequence index: every mean gives the index back, so a frame taken
    # across a boundary (or a chunk stitched to the wrong sequence) shows
    bl = binding()
    for n, T, D, dtype in [(500, 700, 1, "f32"), (40, 3000, 256, "f32"), (700, 100, 2, "i32")]:
        rng = np.random.default_rng(n)
        L = workloads.random_lengths(rng, n, T, "mixed")
        so = workloads.src_offsets(L)
        src = np.repeat(np.arange(n), L)[:, None].repeat(D, axis=1).astype(NP_OF[dtype])
        pl = oracle.plan(L, T, oracle.order(n, 7))
        packed, seq_id, _, reset, valid = oracle.pack(src, so, L, pl, D * 4)
        op = "sum" if dtype == "i32" else "mean"
        out = bl.bload_segment_reduce(to_dev(packed), to_dev(seq_id), to_dev(reset),
                                      to_dev(valid), pl.num_blocks, T, D, dtype, op, n)
        got = out.cpu().numpy()
        want = np.arange(n)[:, None] * (L[:, None] if dtype == "i32" else 1)
        assert np.array_equal(got, np.broadcast_to(want, (n, D)).astype(got.dtype))


def test_reduce_is_deterministic_and_reports_errors():
    bl = binding()
    a = reduce_case(25, 700, 300, "f32", "mean", "uniform")
    b = reduce_case(25, 700, 300, "f32", "mean", "uniform")
    assert torch.equal(a, b)
    x = torch.zeros(16, dtype=torch.uint8, device="cuda:0")
    i = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    with pytest.raises(bl.BloadError) as e:       # int32 mean is not defined
        bl.bload_segment_reduce(x, i, x[:4], x[:4], 1, 4, 1, "i32", "mean", 1)
    assert e.value.status == bl.EINVAL


@pytest.mark.parametrize("wid", [1, 2, 3, 5])
def test_reduce_workloads_full_size(wid):
    # plan + pack + reduce on the device at full size; the oracle sums the ragged source
    bl = binding()
    w = workloads.WORKLOADS[wid]
    L = workloads.lengths(wid)
    so = workloads.src_offsets(L)
    src = workloads.source(wid, 0, int(so[-1]))
    print(f"reduce workload {wid}", flush=True)
    plan_dev = gpu_plan(L, w.t_blk, 0)
    out = bl.bload_pack(to_dev(src.view(np.uint8).reshape(-1)), to_dev(so), to_dev(L), plan_dev,
                        w.frame_bytes)
    red = bl.bload_segment_reduce(out.packed, out.seq_id, out.reset, out.valid,
                                  plan_dev.num_blocks, w.t_blk, w.frame_elems, w.dtype, w.op,
                                  w.n_seq)
    torch.cuda.synchronize()
    check_reduction(red.cpu().numpy(), src, so, L, w.frame_elems, w.dtype, w.op)


# ---- float32 sums that are accurate by construction, not by the luck of random rounding

U = 2.0 ** -24          # unit roundoff of float32


def same_sign_source(rng, total, D):
    """Positive float32 values over six decades, every 97th frame a huge one in front of
    thousands of small ones: a single float32 accumulator per feature loses the small terms
    (error ~ n/2 units in the last place of the sum), which is what must not happen."""
    x = np.exp(rng.uniform(np.log(1e-3), np.log(1e3), size=(total, D))).astype(np.float32)
    x[::97] *= np.float32(4096.0)
    return x


def assert_sum_accuracy(got, src, so, L, D, op, ulps):
    """Against the float64 oracle: inside the 1e-5 bar, and inside `ulps` units of float32
    roundoff of sum |x| (what the summation scheme guarantees at any length)."""
    ref = oracle.segment_reduce(src, so, L, D, "f32", op).astype(np.float64)
    scale = np.add.reduceat(np.abs(src.astype(np.float64)), so[:-1], axis=0)
    if op == "mean":
        scale = scale / L[:, None]
    err = np.abs(got.astype(np.float64) - ref)
    assert np.all(err <= REL_TOL * np.maximum(np.abs(ref), scale)), f"max relative error {np.max(err / scale)}"
    assert np.all(err <= ulps * U * scale), f"{np.max(err / (U * scale)):.1f} units of roundoff, allowed {ulps}"


@pytest.mark.parametrize("n,T,D,ulps", [(48, 3000, 80, 12),      # lanes across features, many chunks + stitch
                                        (300, 3000, 80, 12),     # fewer chunks per block
                                        (6, 3000, 2048, 12),     # a wave per row
                                        (40, 30000, 1, 48),      # lanes across time, 8 tiles per sequence
                                        (64, 3000, 3, 48)])
@pytest.mark.parametrize("op", ["sum", "mean"])
def test_reduce_float32_sums_hold_at_any_length(n, T, D, ulps, op):
    bl = binding()
    rng = np.random.default_rng(T + D)
    L = np.full(n, T, dtype=np.int32)                 # every sequence fills a block
    so = workloads.src_offsets(L)
    src = same_sign_source(rng, int(so[-1]), D)
    pl = oracle.plan(L, T, oracle.order(n, 3))
    packed, seq_id, _, reset, valid = oracle.pack(src, so, L, pl, D * 4)
    out = bl.bload_segment_reduce(to_dev(packed), to_dev(seq_id), to_dev(reset), to_dev(valid),
                                  pl.num_blocks, T, D, "f32", op, n)
    assert_sum_accuracy(out.cpu().numpy(), src, so, L, D, op, ulps)


def test_reduce_float32_one_chunk_per_block_of_3000_frames():
    """8192 blocks of one 3000-frame sequence of 80 float32 features: enough blocks that every
    block is one chunk, so a sequence is summed by one row of lanes from end to end (the launch
    shape of the largest workload).  The payload is drawn on the device; the oracle sums sampled
    sequences copied back from it."""
    bl = binding()
    B, T, D = 8192, 3000, 80
    assert bl.bload_segment_reduce_workspace_bytes(B, T, D, "f32") == 0       # no chunk borders
    g = torch.Generator(device="cuda:0").manual_seed(5)
    x = torch.empty((B, T, D), dtype=torch.float32, device="cuda:0")
    x.uniform_(float(np.log(1e-3)), float(np.log(1e3)), generator=g).exp_()
    x[:, ::97] *= 4096.0
    seq_id = torch.arange(B, dtype=torch.int32, device="cuda:0")[:, None].expand(B, T).contiguous()
    valid = torch.ones((B, T), dtype=torch.uint8, device="cuda:0")
    reset = torch.zeros((B, T), dtype=torch.uint8, device="cuda:0")
    reset[:, 0] = 1
    out = bl.bload_segment_reduce(x, seq_id, reset, valid, B, T, D, "f32", "mean", B)
    pick = np.unique(np.concatenate([[0, B - 1], np.random.default_rng(1).integers(0, B, size=62)]))
    src = x[torch.from_numpy(pick).to("cuda:0")].cpu().numpy().reshape(-1, D)
    L = np.full(len(pick), T, dtype=np.int32)
    assert_sum_accuracy(out[torch.from_numpy(pick).to("cuda:0")].cpu().numpy(), src,
                        workloads.src_offsets(L), L, D, "mean", 12)


# ---- arbitrary flags: the consumer's rule, not only what a correct pack writes

def random_flags(rng, B, T, p_valid, p_reset):
    """valid / reset planes with runs of padding anywhere, start flags anywhere, and a seq_id
    plane that gives every segment of the consumer's rule its own row."""
    valid = (rng.random((B, T)) < p_valid).astype(np.uint8)
    # make padding come in runs so that long segments exist too
    keep = rng.random((B, T)) < 0.9
    for t in range(1, T):
        valid[:, t] = np.where(keep[:, t], valid[:, t - 1], valid[:, t])
    reset = ((rng.random((B, T)) < p_reset) & (valid == 1)).astype(np.uint8)
    prev_valid = np.concatenate([np.zeros((B, 1), np.uint8), valid[:, :-1]], axis=1)
    starts = (valid == 1) & ((reset == 1) | (prev_valid == 0))
    starts[:, 0] = valid[:, 0] == 1
    ids = np.cumsum(starts.reshape(-1)).reshape(B, T) - 1
    seq_id = np.where(valid == 1, ids, -1).astype(np.int32)
    return valid, reset, seq_id, int(starts.sum())


@pytest.mark.parametrize("dtype,op", [("f32", "mean"), ("i32", "sum"), ("u8", "sum"), ("f16", "mean")])
@pytest.mark.parametrize("B,T,D", [(3, 10, 1), (700, 33, 1), (40, 5000, 1), (9, 4096, 2),
                                   (300, 130, 16), (50, 700, 80), (20, 3000, 256), (64, 32, 3072)])
def test_reduce_follows_the_flags(B, T, D, dtype, op):
    bl = binding()
    rng = np.random.default_rng(B + T + D)
    for p_valid, p_reset in [(0.85, 0.02), (0.5, 0.3), (1.0, 0.0)]:
        valid, reset, seq_id, n_seg = random_flags(rng, B, T, p_valid, p_reset)
        src = draw_source(rng, B * T, D, dtype)          # payload in every slot, padding included
        packed = src.reshape(B, T, D)
        want, counted = oracle.segment_reduce_packed(packed, seq_id, reset, valid, D, dtype, op, n_seg)
        assert counted == n_seg
        print(f"flags B={B} T={T} D={D} {dtype} {op} valid~{p_valid} reset~{p_reset} segments={n_seg}",
              flush=True)
        if n_seg == 0:
            continue
        got = bl.bload_segment_reduce(to_dev(packed), to_dev(seq_id), to_dev(reset), to_dev(valid),
                                      B, T, D, dtype, op, n_seg).cpu().numpy()
        if dtype == "i32":
            assert np.array_equal(got, want)
            continue
        absval = np.abs(packed.astype(np.float64)).astype(np.float32)
        scale, _ = oracle.segment_reduce_packed(absval, seq_id, reset, valid, D, "f32", op, n_seg)
        bound = REL_TOL * np.maximum(np.abs(want.astype(np.float64)), scale.astype(np.float64)) + 1e-30
        err = np.abs(got.astype(np.float64) - want.astype(np.float64))
        assert np.all(err <= bound), f"max err {err.max()} at {np.unravel_index(np.argmax(err - bound), err.shape)}"
