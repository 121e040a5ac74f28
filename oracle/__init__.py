"""numpy front end of the CPU oracle (``bload_oracle.c``) -- TEST INFRASTRUCTURE.

Only ``tests/``, the smoke check and the benchmark's CPU-baseline leg may use
this package; the HIP library and its binding never do.  The C file is
compiled with gcc on first use if the shared object is missing or older than
the source.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bload_oracle.c")
_LIB = os.path.join(_HERE, "libbload_oracle.so")

DTYPE_CODE = {"u8": 0, "f16": 1, "f32": 2, "i32": 3}
OP_CODE = {"sum": 0, "mean": 1}
_NP_OF = {"u8": np.uint8, "f16": np.float16, "f32": np.float32, "i32": np.int32}


def build(force: bool = False) -> str:
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(["gcc", "-O2", "-Wall", "-Wextra", "-shared", "-fPIC",
                               "-o", _LIB, _SRC])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.bload_oracle_splitmix64.restype = ctypes.c_uint64
        lib.bload_oracle_splitmix64.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
        lib.bload_oracle_fmix32.restype = ctypes.c_uint32
        lib.bload_oracle_fmix32.argtypes = [ctypes.c_uint32]
        lib.bload_oracle_half_to_double.restype = ctypes.c_double
        lib.bload_oracle_half_to_double.argtypes = [ctypes.c_uint16]
        lib.bload_oracle_order.restype = None
        lib.bload_oracle_order.argtypes = [ctypes.c_int64, ctypes.c_uint64, ctypes.c_void_p]
        lib.bload_oracle_plan.restype = ctypes.c_int
        lib.bload_oracle_plan.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.bload_oracle_pack_blocks.restype = None
        lib.bload_oracle_pack_blocks.argtypes = [ctypes.c_void_p] * 5 + [
            ctypes.c_int64, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64
        ] + [ctypes.c_void_p] * 5
        lib.bload_oracle_segment_reduce.restype = ctypes.c_int
        lib.bload_oracle_segment_reduce.argtypes = [ctypes.c_void_p, ctypes.c_void_p,
                                                    ctypes.c_void_p, ctypes.c_int64,
                                                    ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                                    ctypes.c_void_p]
        lib.bload_oracle_plan_shard.restype = ctypes.c_int64
        lib.bload_oracle_plan_shard.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int64, ctypes.c_int64,
                                                                       ctypes.c_int32, ctypes.c_int32] + \
            [ctypes.c_void_p] * 3
        lib.bload_oracle_segment_reduce_packed.restype = ctypes.c_int64
        lib.bload_oracle_segment_reduce_packed.argtypes = [ctypes.c_void_p] * 4 + [
            ctypes.c_int64, ctypes.c_int32, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int64,
            ctypes.c_void_p]
        lib.bload_oracle_plan_random_fit.restype = ctypes.c_int
        lib.bload_oracle_plan_random_fit.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32,
                                                     ctypes.c_uint64] + [ctypes.c_void_p] * 7
        lib.bload_oracle_padding.restype = None
        lib.bload_oracle_padding.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                             ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
                                             ctypes.c_void_p]
        lib.bload_oracle_segment_scan.restype = ctypes.c_int
        lib.bload_oracle_segment_scan.argtypes = [ctypes.c_void_p] * 3 + [
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_double, ctypes.c_void_p,
            ctypes.c_void_p]
        lib.bload_oracle_segment_scan_packed.restype = ctypes.c_int
        lib.bload_oracle_segment_scan_packed.argtypes = [ctypes.c_void_p] * 3 + [
            ctypes.c_int64, ctypes.c_int32, ctypes.c_int64, ctypes.c_int, ctypes.c_double,
            ctypes.c_void_p, ctypes.c_void_p]
        lib.bload_oracle_chunk_sampling.restype = None
        lib.bload_oracle_chunk_sampling.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                                    ctypes.c_void_p, ctypes.c_void_p]
        lib.bload_oracle_plan_check.restype = ctypes.c_int64
        lib.bload_oracle_plan_check.argtypes = [ctypes.c_void_p] * 6 + [ctypes.c_int64, ctypes.c_int64,
                                                                       ctypes.c_int32, ctypes.c_int64]
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _c(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def splitmix64(seed: int, k: int) -> int:
    return int(_load().bload_oracle_splitmix64(seed & (2**64 - 1), k))


def fmix32(h: int) -> int:
    return int(_load().bload_oracle_fmix32(h & 0xFFFFFFFF))


def half_to_double(bits: int) -> float:
    return float(_load().bload_oracle_half_to_double(bits))


def order(n: int, seed: int) -> np.ndarray:
    out = np.full(max(n, 0), -7, dtype=np.int32)
    _load().bload_oracle_order(n, seed & (2**64 - 1), _p(out))
    return out


class Plan:
    """Result of the next-fit plan."""

    def __init__(self, order, block_of_seq, offset_of_seq, block_first, num_blocks,
                 total_frames, t_blk):
        self.order = order
        self.block_of_seq = block_of_seq
        self.offset_of_seq = offset_of_seq
        self.block_first = block_first            # int32[num_blocks + 1]
        self.num_blocks = num_blocks
        self.total_frames = total_frames
        self.t_blk = t_blk


def plan(lengths, t_blk: int, order_) -> Plan:
    """Next-fit over ``order_``; raises ValueError on a length outside [1, t_blk]."""
    L = _c(lengths, np.int32)
    o = _c(order_, np.int32)
    n = L.shape[0]
    assert o.shape[0] == n
    block_of = np.full(n, -7, dtype=np.int32)
    offset_of = np.full(n, -7, dtype=np.int32)
    block_first = np.full(n + 1, -7, dtype=np.int32)
    nb = np.zeros(1, dtype=np.int64)
    tot = np.zeros(1, dtype=np.int64)
    rc = _load().bload_oracle_plan(_p(L), n, t_blk, _p(o), _p(block_of), _p(offset_of),
                                   _p(block_first), _p(nb), _p(tot))
    if rc != 0:
        raise ValueError("length outside [1, t_blk]")
    b = int(nb[0])
    return Plan(o, block_of, offset_of, block_first[:b + 1].copy() if n else block_first[:0],
                b, int(tot[0]), t_blk)


def plan_random_fit(lengths, t_blk: int, seed: int) -> Plan:
    """The paper's sampler: each block draws uniformly among the remaining sequences that
    still fit until none does.  Raises ValueError on a length outside [1, t_blk]."""
    L = _c(lengths, np.int32)
    n = L.shape[0]
    seeded = order(n, seed)
    o = np.full(n, -7, dtype=np.int32)
    block_of = np.full(n, -7, dtype=np.int32)
    offset_of = np.full(n, -7, dtype=np.int32)
    block_first = np.full(n + 1, -7, dtype=np.int32)
    nb = np.zeros(1, dtype=np.int64)
    tot = np.zeros(1, dtype=np.int64)
    rc = _load().bload_oracle_plan_random_fit(_p(L), n, t_blk, seed & (2**64 - 1), _p(seeded), _p(o),
                                              _p(block_of), _p(offset_of), _p(block_first), _p(nb),
                                              _p(tot))
    if rc != 0:
        raise ValueError("length outside [1, t_blk]")
    b = int(nb[0])
    return Plan(o, block_of, offset_of, block_first[:b + 1].copy() if n else block_first[:0],
                b, int(tot[0]), t_blk)


def plan_shard(pl: Plan, rank: int, world: int) -> Plan:
    """Worker ``rank``'s share of the plan (blocks b = rank mod world, plus a padding block
    when the worker would fall short): a Plan whose tables are local to the worker.
    ``order`` keeps length N with -1 behind the worker's own sequences."""
    n = pl.order.shape[0]
    nb_local = -(-pl.num_blocks // world)
    order_local = np.full(n, -7, dtype=np.int32)
    block_of_local = np.full(n, -7, dtype=np.int32)
    block_first_local = np.full(nb_local + 1, -7, dtype=np.int32)
    bf = np.zeros(pl.num_blocks + 1, dtype=np.int32)
    bf[:] = pl.block_first
    n_local = _load().bload_oracle_plan_shard(_p(pl.order), _p(pl.block_of_seq), _p(bf), n,
                                              pl.num_blocks, rank, world, _p(order_local),
                                              _p(block_of_local), _p(block_first_local))
    out = Plan(order_local, block_of_local, pl.offset_of_seq, block_first_local, nb_local,
               pl.total_frames, pl.t_blk)
    out.n_local = int(n_local)
    return out


def alloc_pack_outputs(nb: int, t_blk: int, frame_bytes: int):
    """Output arrays for ``pack_blocks``, prefilled with garbage so that a slot the
    oracle fails to write shows up."""
    return (np.full((nb, t_blk, frame_bytes), 0xA5, dtype=np.uint8),
            np.full((nb, t_blk), -9, dtype=np.int32), np.full((nb, t_blk), -9, dtype=np.int32),
            np.full((nb, t_blk), 9, dtype=np.uint8), np.full((nb, t_blk), 9, dtype=np.uint8))


def pack_blocks(src, src_offsets, lengths, pl: Plan, frame_bytes: int, block_lo: int,
                block_hi: int, out=None):
    """Blocks [block_lo, block_hi) -> (packed u8[nb, T, frame_bytes], seq_id i32[nb, T],
    frame_idx i32[nb, T], reset u8[nb, T], valid u8[nb, T]); ``out`` may bring
    preallocated arrays of those shapes."""
    src = np.ascontiguousarray(src)
    src_b = src.view(np.uint8).reshape(-1)
    so = _c(src_offsets, np.int64)
    L = _c(lengths, np.int32)
    n = L.shape[0]
    assert src_b.shape[0] == int(so[-1]) * frame_bytes if n else True
    nb = block_hi - block_lo
    T = pl.t_blk
    packed, seq_id, frame_idx, reset, valid = (alloc_pack_outputs(nb, T, frame_bytes)
                                               if out is None else out)
    assert packed.shape == (nb, T, frame_bytes) and packed.dtype == np.uint8
    _load().bload_oracle_pack_blocks(_p(src_b), _p(so), _p(L), _p(pl.block_of_seq),
                                     _p(pl.offset_of_seq), n, T, frame_bytes, block_lo,
                                     block_hi, _p(packed), _p(seq_id), _p(frame_idx),
                                     _p(reset), _p(valid))
    return packed, seq_id, frame_idx, reset, valid


def pack(src, src_offsets, lengths, pl: Plan, frame_bytes: int, out=None):
    return pack_blocks(src, src_offsets, lengths, pl, frame_bytes, 0, pl.num_blocks, out)


def segment_reduce(src, src_offsets, lengths, feat_dim: int, dtype: str, op: str) -> np.ndarray:
    """Per-sequence sum / mean over time of the ragged source ``[sum(L), feat_dim]``."""
    src = np.ascontiguousarray(src, dtype=_NP_OF[dtype])
    so = _c(src_offsets, np.int64)
    L = _c(lengths, np.int32)
    n = L.shape[0]
    out = np.zeros((n, feat_dim), dtype=np.int64 if dtype == "i32" else np.float32)
    rc = _load().bload_oracle_segment_reduce(_p(src), _p(so), _p(L), n, feat_dim,
                                             DTYPE_CODE[dtype], OP_CODE[op], _p(out))
    if rc != 0:
        raise ValueError("unsupported dtype/op combination")
    return out


def segment_reduce_packed(packed, seq_id, reset, valid, feat_dim: int, dtype: str, op: str,
                          n_seq: int):
    """Per-sequence sum / mean read from the packed blocks and their flags (any flags).
    Returns (out[n_seq, feat_dim], number of segments); rows no segment names stay 0."""
    B, T = seq_id.shape
    pk = np.ascontiguousarray(packed).view(_NP_OF[dtype]).reshape(B, T, feat_dim)
    sid, rs, vl = _c(seq_id, np.int32), _c(reset, np.uint8), _c(valid, np.uint8)
    out = np.zeros((n_seq, feat_dim), dtype=np.int64 if dtype == "i32" else np.float32)
    n = _load().bload_oracle_segment_reduce_packed(_p(pk), _p(sid), _p(rs), _p(vl), B, T, feat_dim,
                                                   DTYPE_CODE[dtype], OP_CODE[op], n_seq, _p(out))
    if n < 0:
        raise ValueError("unsupported dtype/op combination")
    return out, int(n)


def padding(lengths, t_max: int, num_blocks: int, t_blk: int):
    """(pad_longest, pad_blocks) in frames."""
    L = _c(lengths, np.int32)
    a = np.zeros(1, dtype=np.int64)
    b = np.zeros(1, dtype=np.int64)
    _load().bload_oracle_padding(_p(L), L.shape[0], t_max, num_blocks, t_blk, _p(a), _p(b))
    return int(a[0]), int(b[0])


def chunk_sampling(lengths, t_chunk: int):
    """(samples, frames deleted) when every sequence is cut into pieces of t_chunk frames."""
    L = _c(lengths, np.int32)
    a = np.zeros(1, dtype=np.int64)
    b = np.zeros(1, dtype=np.int64)
    _load().bload_oracle_chunk_sampling(_p(L), L.shape[0], t_chunk, _p(a), _p(b))
    return int(a[0]), int(b[0])


def segment_scan(src, src_offsets, lengths, feat_dim: int, dtype: str, decay: float):
    """h_0 = x_0, h_t = decay * h_(t-1) + x_t inside every sequence of the ragged source.
    Returns (h, scale), float32[sum(L), feat_dim]; scale is the same recurrence on |x|, |decay|."""
    src = np.ascontiguousarray(src, dtype=_NP_OF[dtype])
    so = _c(src_offsets, np.int64)
    L = _c(lengths, np.int32)
    total = int(so[-1]) if L.shape[0] else 0
    out = np.full((total, feat_dim), np.nan, dtype=np.float32)
    scale = np.full((total, feat_dim), np.nan, dtype=np.float32)
    rc = _load().bload_oracle_segment_scan(_p(src), _p(so), _p(L), L.shape[0], feat_dim,
                                           DTYPE_CODE[dtype], float(decay), _p(out), _p(scale))
    if rc != 0:
        raise ValueError("unsupported dtype")
    return out, scale


def segment_scan_packed(packed, reset, valid, feat_dim: int, dtype: str, decay: float):
    """The recurrence read from packed blocks through their flags (any flags).
    Returns (h, scale), float32[B, T, feat_dim]; invalid slots hold 0."""
    B, T = valid.shape
    pk = np.ascontiguousarray(packed).view(_NP_OF[dtype]).reshape(B, T, feat_dim)
    rs, vl = _c(reset, np.uint8), _c(valid, np.uint8)
    out = np.full((B, T, feat_dim), np.nan, dtype=np.float32)
    scale = np.full((B, T, feat_dim), np.nan, dtype=np.float32)
    rc = _load().bload_oracle_segment_scan_packed(_p(pk), _p(rs), _p(vl), B, T, feat_dim,
                                                  DTYPE_CODE[dtype], float(decay), _p(out), _p(scale))
    if rc != 0:
        raise ValueError("unsupported dtype")
    return out, scale


def plan_check(src_offsets, lengths, order_, block_of_seq, offset_of_seq, block_first, num_blocks: int,
               t_blk: int, total_frames: int) -> int:
    """-1 if the tables describe blocks of whole sequences laid one after another, else the
    smallest block / shuffled position at which they do not.  ``block_first`` needs at least
    num_blocks + 1 entries."""
    so = _c(src_offsets, np.int64)
    L, o = _c(lengths, np.int32), _c(order_, np.int32)
    bo, oo, bf = _c(block_of_seq, np.int32), _c(offset_of_seq, np.int32), _c(block_first, np.int32)
    assert bf.shape[0] >= num_blocks + 1 and so.shape[0] == L.shape[0] + 1
    return int(_load().bload_oracle_plan_check(_p(so), _p(L), _p(o), _p(bo), _p(oo), _p(bf), L.shape[0],
                                               num_blocks, t_blk, total_frames))
