"""Thin binding of ``libbload_yardsticks.so`` (``include/bload_yardsticks.h``): streaming kernels
without any of the packer's logic, and ``measure()``, which times them on buffers of the sizes of
the large workloads so that ``bench.py`` can print what each access pattern alone reaches on the
GPU it runs on.  Nothing here is on the packer's path."""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbload_yardsticks.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2310_10879_amd.build`")
_lib = ctypes.CDLL(LIB_PATH)
_vp, _i64, _sz, _int = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t, ctypes.c_int
_lib.bload_ys_copy.argtypes = [_vp, _vp, _sz, _vp]
_lib.bload_ys_read.argtypes = [_vp, _sz, _vp, _vp]
_lib.bload_ys_token_pack.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i64, _int, _int, _vp]
_lib.bload_ys_rows.argtypes = [_vp, _vp, _i64, _i64, _int, _int, _vp, _vp]
for _f in (_lib.bload_ys_copy, _lib.bload_ys_read, _lib.bload_ys_token_pack, _lib.bload_ys_rows):
    _f.restype = ctypes.c_int


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(status: int) -> None:
    if status != 0:
        raise RuntimeError(f"yardstick refused or failed to launch (status {status})")


def bload_ys_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    _check(_lib.bload_ys_copy(src.data_ptr(), dst.data_ptr(), src.numel() * src.element_size(), _stream()))


def bload_ys_read(src: torch.Tensor, sink: torch.Tensor) -> None:
    _check(_lib.bload_ys_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(), _stream()))


def bload_ys_token_pack(src, payload, plane_a, plane_b, flags_a, flags_b, n_slots: int, padding_percent: int,
                        scattered: bool) -> None:
    _check(_lib.bload_ys_token_pack(src.data_ptr(), payload.data_ptr(), plane_a.data_ptr(), plane_b.data_ptr(),
                                    flags_a.data_ptr(), flags_b.data_ptr(), n_slots, padding_percent,
                                    1 if scattered else 0, _stream()))


def bload_ys_rows(src, dst, n_rows: int, row_bytes: int, rows_per_wave: int, active_lanes: int, sink) -> None:
    _check(_lib.bload_ys_rows(src.data_ptr(), None if dst is None else dst.data_ptr(), n_rows, row_bytes,
                              rows_per_wave, active_lanes, sink.data_ptr(), _stream()))


def _time(fn, reps: int = 5) -> float:
    for _ in range(2):
        fn()
    torch.cuda.synchronize()
    ms = []
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        torch.cuda.synchronize()
        ms.append(a.elapsed_time(b))
    return float(np.mean(ms))


def measure(device: torch.device) -> dict:
    """GB/s (bytes the pattern moves / mean time of 5 launches) of every yardstick: 4 GiB buffers
    for the copy, the read and the token traffic (2^30 slots), 34560 rows of 3000 x 320 bytes for
    the rows (the shape of the largest workload's blocks)."""
    out = {}
    gib = 1 << 30
    sink = torch.zeros(4, dtype=torch.int32, device=device)
    a = torch.empty(4 * gib, dtype=torch.uint8, device=device)
    b = torch.empty(4 * gib, dtype=torch.uint8, device=device)
    a.fill_(1)
    out["copy_tiles_GBps"] = 2 * a.numel() / _time(lambda: bload_ys_copy(a, b)) * 1e-6
    out["read_tiles_GBps"] = a.numel() / _time(lambda: bload_ys_read(a, sink)) * 1e-6
    n_slots = gib                                     # 4 GiB of tokens
    c = torch.empty(4 * gib, dtype=torch.uint8, device=device)
    d = torch.empty(4 * gib, dtype=torch.uint8, device=device)
    fa = torch.empty(gib, dtype=torch.uint8, device=device)
    fb = torch.empty(gib, dtype=torch.uint8, device=device)
    for name, pad, scattered in (("token_pack_plain_GBps", 0, False), ("token_pack_padded_scattered_GBps", 35, True)):
        moved = n_slots * (14 + 4 * (100 - pad) / 100)
        out[name] = moved / _time(lambda: bload_ys_token_pack(a, b, c, d, fa, fb, n_slots, pad, scattered)) * 1e-6
    del c, d, fa, fb
    n_rows, row_bytes = 34560, 3000 * 320
    src = torch.empty(n_rows * row_bytes, dtype=torch.uint8, device=device)
    dst = torch.empty(n_rows * row_bytes, dtype=torch.uint8, device=device)
    src.fill_(1)
    size = n_rows * row_bytes
    out["rows_read_GBps"] = size / _time(lambda: bload_ys_rows(src, None, n_rows, row_bytes, 2, 20, sink)) * 1e-6
    out["rows_read_write_GBps"] = 2 * size / _time(lambda: bload_ys_rows(src, dst, n_rows, row_bytes, 2, 20, sink)) * 1e-6
    out["what"] = ("kernels of libbload_yardsticks.so (include/bload_yardsticks.h) on 4 GiB buffers: copy and read in "
                   "4 KiB tiles; the traffic of packing 2^30 tokens (one read, five written streams) without and with "
                   "35 % padding blocks and hashed source blocks; waves walking 34560 rows of 3000 x 320 bytes, two "
                   "rows per wave, 20 of 32 lanes (read only, and read + write)")
    return out
