"""The yardstick kernels move what their header says they move (small sizes, compared with
numpy): a benchmark figure of a kernel that skipped part of its traffic would be worthless."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_copy_and_read():
    from paper_2310_10879_amd import yardsticks as ys
    rng = np.random.default_rng(0)
    src = torch.from_numpy(rng.integers(0, 256, size=16 * 70001, dtype=np.uint8)).cuda()
    dst = torch.zeros_like(src)
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    ys.bload_ys_copy(src, dst)
    ys.bload_ys_read(src, sink)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    assert int(sink[0]) == 0


@pytest.mark.parametrize("pad,scattered", [(0, False), (35, True), (100, False)])
def test_token_pack_writes_every_stream(pad, scattered):
    from paper_2310_10879_amd import yardsticks as ys
    n_slots = 4096 * 301
    rng = np.random.default_rng(1)
    h_src = rng.integers(0, 2 ** 32, size=n_slots, dtype=np.uint32)
    src = torch.from_numpy(h_src.view(np.int32)).cuda()
    outs = [torch.full((n_slots,), 7, dtype=torch.int32, device="cuda") for _ in range(3)]
    flags = [torch.full((n_slots // 4,), 7, dtype=torch.int32, device="cuda") for _ in range(2)]
    ys.bload_ys_token_pack(src, outs[0], outs[1], outs[2], flags[0], flags[1], n_slots, pad, scattered)
    torch.cuda.synchronize()
    n_blocks = n_slots // 4096
    want = np.full(n_slots, 0xFFFFFFFF, dtype=np.uint32)
    for b in range(n_blocks):
        if b % 100 >= pad:
            fb = ((b * 0x9E3779B97F4A7C15) % (1 << 64) >> 20) % n_blocks if scattered else b
            want[b * 4096:(b + 1) * 4096] = h_src[fb * 4096:(fb + 1) * 4096]
    for o in outs:
        assert np.array_equal(o.cpu().numpy().view(np.uint32), want)
    quads = want.reshape(-1, 4)
    assert np.array_equal(flags[0].cpu().numpy().view(np.uint32), quads[:, 0])
    assert np.array_equal(flags[1].cpu().numpy().view(np.uint32), quads[:, 1])


@pytest.mark.parametrize("rows_per_wave,active", [(2, 20), (1, 60), (4, 15), (1, 64)])
def test_rows_copy_every_active_byte(rows_per_wave, active):
    from paper_2310_10879_amd import yardsticks as ys
    n_rows, row_bytes = 37, 8 * 16 * active * 5
    rng = np.random.default_rng(2)
    src = torch.from_numpy(rng.integers(0, 256, size=n_rows * row_bytes, dtype=np.uint8)).cuda()
    dst = torch.zeros_like(src)
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    ys.bload_ys_rows(src, dst, n_rows, row_bytes, rows_per_wave, active, sink)
    ys.bload_ys_rows(src, None, n_rows, row_bytes, rows_per_wave, active, sink)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
