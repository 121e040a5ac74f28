"""Seeded synthetic inputs for the BLoad block packer.

This module only *draws inputs*: sequence lengths and frame payloads with the
shapes and value distributions of the workloads the packer is measured on.
It holds none of the method's arithmetic (no shuffle, no block assignment, no
packing, no reduction), so both the CPU oracle's tests and the HIP path's tests
can feed from it without sharing anything that is under test.

The paper (Experiments section) measures on a video dataset with a wide length
spread (3 to 94 frames, 7464 videos); that dataset is not available, so the
five workloads below stand in for it: a wide spread of lengths with the block
length equal to (or above) the longest sequence.

Everything is a pure function of (workload id, index range): lengths come from
``PCG64(1000 + wid)``; the ragged source ``[sum(L), frame_elems]`` is produced in
fixed chunks of frames, chunk ``c`` from ``PCG64([2000 + wid, c])``, so any
range of frames can be regenerated without holding the whole source.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    wid: int
    name: str
    n_seq: int
    t_blk: int
    frame_shape: Tuple[int, ...]
    dtype: str          # "u8" | "f16" | "f32" | "i32"  (element type of a frame)
    op: str             # "mean" | "sum"  (per-sequence reduction of the workload)

    @property
    def np_dtype(self):
        return {"u8": np.uint8, "f16": np.float16, "f32": np.float32, "i32": np.int32}[self.dtype]

    @property
    def frame_elems(self) -> int:
        return int(np.prod(self.frame_shape))

    @property
    def frame_bytes(self) -> int:
        return self.frame_elems * np.dtype(self.np_dtype).itemsize


WORKLOADS = {
    1: Workload(1, "toy-video u8 3x32x32", 64, 32, (3, 32, 32), "u8", "mean"),
    2: Workload(2, "video u8 3x112x112", 1000, 600, (3, 112, 112), "u8", "mean"),
    3: Workload(3, "features f16 2048", 10000, 3000, (2048,), "f16", "mean"),
    4: Workload(4, "log-mel f32 80", 50000, 3000, (80,), "f32", "mean"),
    5: Workload(5, "tokens i32", 1000000, 4096, (1,), "i32", "sum"),
}

SHUFFLE_SEEDS = (0, 1, 0x9E3779B97F4A7C15)


def lengths(wid: int, n_seq: int | None = None) -> np.ndarray:
    """Sequence lengths (int32[N]) of workload ``wid``.

    ``n_seq`` overrides N (the draw is a prefix-stable stream only for the
    integer-uniform workloads; the others simply draw ``n_seq`` values).
    """
    w = WORKLOADS[wid]
    n = w.n_seq if n_seq is None else int(n_seq)
    rng = np.random.Generator(np.random.PCG64(1000 + wid))
    if wid == 1:
        L = rng.integers(2, 32, size=n, endpoint=True)
    elif wid == 2:
        # "lognormal (mean 60, sigma 1.0)": the mean is that of the underlying
        # normal on the log scale, ln 60, i.e. the median length is 60.
        L = np.clip(np.rint(rng.lognormal(mean=np.log(60.0), sigma=1.0, size=n)), 1, 600)
    elif wid == 3:
        # Pareto(alpha=1.5) with minimum 8: numpy's pareto() is the Lomax form,
        # so the classical Pareto variate is 8 * (1 + lomax).
        L = np.clip(np.floor(8.0 * (1.0 + rng.pareto(1.5, size=n))), 8, 3000)
    elif wid == 4:
        L = rng.integers(100, 3000, size=n, endpoint=True)
    elif wid == 5:
        # "clipped" read literally: draws above 4096 become 4096.
        L = np.clip(rng.zipf(1.2, size=n), 1, 4096)
    else:
        raise KeyError(wid)
    return np.ascontiguousarray(L, dtype=np.int32)


def src_offsets(L: np.ndarray) -> np.ndarray:
    """Exclusive running frame count, int64[N+1]: where each sequence starts in
    the ragged source (a layout fact of the input, not a step of the method)."""
    off = np.zeros(L.shape[0] + 1, dtype=np.int64)
    np.cumsum(L, dtype=np.int64, out=off[1:])
    return off


def _chunk_frames(w: Workload) -> int:
    # about 32 MiB of payload per chunk, at least one frame
    return max(1, (32 << 20) // w.frame_bytes)


def _draw_chunk(w: Workload, c: int, n_frames: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64([2000 + w.wid, c]))
    shape = (n_frames, w.frame_elems)
    if w.dtype == "u8":
        return rng.integers(0, 256, size=shape, dtype=np.uint8)
    if w.dtype == "f16":
        return rng.standard_normal(size=shape, dtype=np.float32).astype(np.float16)
    if w.dtype == "f32":
        x = rng.standard_normal(size=shape, dtype=np.float32)
        x *= np.float32(2.0)
        x += np.float32(-4.0)
        return x
    if w.dtype == "i32":
        return rng.integers(0, 32000, size=shape, dtype=np.int32)
    raise KeyError(w.dtype)


def source(wid: int, frame_lo: int, frame_hi: int, threads: int = 8) -> np.ndarray:
    """Frames ``[frame_lo, frame_hi)`` of the ragged source of workload ``wid``
    as an array ``[frame_hi - frame_lo, frame_elems]`` of the frame dtype."""
    w = WORKLOADS[wid]
    ch = _chunk_frames(w)
    out = np.empty((frame_hi - frame_lo, w.frame_elems), dtype=w.np_dtype)
    if frame_hi <= frame_lo:
        return out
    c_lo, c_hi = frame_lo // ch, (frame_hi - 1) // ch

    def fill(c: int) -> None:
        # a chunk is always drawn whole so that its content does not depend on
        # the range asked for
        data = _draw_chunk(w, c, ch)
        a, b = max(frame_lo, c * ch), min(frame_hi, (c + 1) * ch)
        out[a - frame_lo:b - frame_lo] = data[a - c * ch:b - c * ch]

    chunks = list(range(c_lo, c_hi + 1))
    if threads > 1 and len(chunks) > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, chunks))
    else:
        for c in chunks:
            fill(c)
    return out


def tagged_source(L: np.ndarray, frame_bytes: int) -> np.ndarray:
    """A byte payload ``[sum(L), frame_bytes]`` whose frames say who they are:
    byte k of frame t of sequence i is a fixed hash of (i, t, k), and when the
    frame is at least 8 bytes wide its first 8 bytes are (i, t) as two little
    endian int32.  Used to check "every frame exactly once, in order"."""
    total = int(np.sum(L, dtype=np.int64))
    seq = np.repeat(np.arange(L.shape[0], dtype=np.int64), L)
    start = np.repeat(src_offsets(L)[:-1], L)
    t = np.arange(total, dtype=np.int64) - start
    k = np.arange(frame_bytes, dtype=np.int64)[None, :]
    h = (seq[:, None] * 2654435761 + t[:, None] * 40503 + k * 97 + 13) & 0xFFFFFFFF
    out = ((h >> 11) & 0xFF).astype(np.uint8)
    if frame_bytes >= 8:
        out[:, 0:4] = seq.astype("<i4").view(np.uint8).reshape(-1, 4)
        out[:, 4:8] = t.astype("<i4").view(np.uint8).reshape(-1, 4)
    return out


def random_lengths(rng: np.random.Generator, n: int, t_blk: int, kind: str = "uniform") -> np.ndarray:
    """Lengths in [1, t_blk] for property tests: 'uniform', 'short' (mostly
    tiny), 'long' (mostly near t_blk) or 'mixed'."""
    if n == 0:
        return np.zeros(0, dtype=np.int32)
    if kind == "uniform":
        L = rng.integers(1, t_blk, size=n, endpoint=True)
    elif kind == "short":
        L = np.minimum(1 + rng.geometric(0.5, size=n) - 1, t_blk)
    elif kind == "long":
        L = t_blk - np.minimum(rng.geometric(0.3, size=n) - 1, t_blk - 1)
    elif kind == "mixed":
        a = rng.integers(1, t_blk, size=n, endpoint=True)
        b = np.minimum(rng.geometric(0.5, size=n), t_blk)
        c = np.full(n, t_blk)
        pick = rng.integers(0, 3, size=n)
        L = np.where(pick == 0, a, np.where(pick == 1, b, c))
    else:
        raise KeyError(kind)
    return np.ascontiguousarray(L, dtype=np.int32)
