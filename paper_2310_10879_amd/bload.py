"""Python binding of the BLoad C-ABI library (``include/bload.h``).

Argument marshalling only: every function here checks dtypes / devices, takes
``data_ptr()`` of torch tensors (torch is used for device memory and streams,
nothing else) and calls the entry point of the same name in ``libbload.so``.
There is no fallback: importing this module without the built library raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbload.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2310_10879_amd.build` "
        "(there is no CPU fallback)")

_lib = ctypes.CDLL(LIB_PATH)

# status codes (mirror of bload_status)
OK, EINVAL, ELENGTH, EWORKSPACE, EALIGN, EOVERFLOW, EHIP = range(7)
DTYPES = {"u8": 0, "f16": 1, "f32": 2, "i32": 3}
OPS = {"sum": 0, "mean": 1}
TORCH_DTYPE = {"u8": torch.uint8, "f16": torch.float16, "f32": torch.float32, "i32": torch.int32}
MAX_SEQ = 1 << 27

_vp, _i64, _i32, _u64, _sz = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64,
                              ctypes.c_size_t)

_lib.bload_status_string.restype = ctypes.c_char_p
_lib.bload_status_string.argtypes = [ctypes.c_int]
_lib.bload_last_hip_error.restype = ctypes.c_int
_lib.bload_last_hip_error.argtypes = []
_lib.bload_plan_workspace_bytes.restype = _sz
_lib.bload_plan_workspace_bytes.argtypes = [_i64]
_lib.bload_plan.restype = ctypes.c_int
_lib.bload_plan.argtypes = [_vp, _i64, _i32, _u64, _vp, _vp, _vp, _vp,
                            ctypes.POINTER(_i64), ctypes.POINTER(_i64), _vp, _sz, _vp]
_lib.bload_plan_random_fit_workspace_bytes.restype = _sz
_lib.bload_plan_random_fit_workspace_bytes.argtypes = [_i64]
_lib.bload_plan_random_fit.restype = ctypes.c_int
_lib.bload_plan_random_fit.argtypes = list(_lib.bload_plan.argtypes)
_lib.bload_plan_shard.restype = ctypes.c_int
_lib.bload_plan_shard.argtypes = [_vp, _vp, _vp, _i64, _i64, _i32, _i32, _vp, _vp, _vp,
                                  ctypes.POINTER(_i64), ctypes.POINTER(_i64), _vp, _sz, _vp]
_lib.bload_pack_workspace_bytes.restype = _sz
_lib.bload_pack_workspace_bytes.argtypes = [_i64, _i64, _i32, _i64]
_lib.bload_pack_tile_bytes.restype = _i32
_lib.bload_pack_tile_bytes.argtypes = [_i64, _i64, _i32, _i64, _i32]
_lib.bload_pack.restype = ctypes.c_int
_lib.bload_pack.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _i32, _i64,
                            _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.bload_pack_noalloc.restype = ctypes.c_int
_lib.bload_pack_noalloc.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _i32, _i64,
                                    _vp, _vp, _vp, _vp, _vp, _vp]
_lib.bload_pack_check.restype = ctypes.c_int
_lib.bload_pack_check.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _i32, _i64,
                                  ctypes.POINTER(_i64), _vp, _sz, _vp]


class StrategyCounts(ctypes.Structure):
    """bload_strategy_counts_t"""
    _fields_ = [(name, ctypes.c_int64) for name in
                ("total_frames", "longest", "pad_to_longest", "pad_blocks", "chunk_samples",
                 "chunk_deleted")]

    def as_dict(self) -> dict:
        return {name: int(getattr(self, name)) for name, _ in self._fields_}


_lib.bload_strategy_counts.restype = ctypes.c_int
_lib.bload_strategy_counts.argtypes = [_vp, _i64, _i32, _i32, _i64, _i32,
                                       ctypes.POINTER(StrategyCounts), _vp, _sz, _vp]
_lib.bload_segment_scan.restype = ctypes.c_int
_lib.bload_segment_scan.argtypes = [_vp, _vp, _vp, _i64, _i32, _i64, ctypes.c_int, ctypes.c_float, _vp,
                                    _vp, _sz, _vp]
_lib.bload_segment_scan_workspace_bytes.restype = _sz
_lib.bload_segment_scan_workspace_bytes.argtypes = [_i64, _i32, _i64, ctypes.c_int]
_lib.bload_segment_reduce_workspace_bytes.restype = _sz
_lib.bload_segment_reduce_workspace_bytes.argtypes = [_i64, _i32, _i64, ctypes.c_int]
_lib.bload_segment_reduce.restype = ctypes.c_int
_lib.bload_segment_reduce.argtypes = [_vp, _vp, _vp, _vp, _i64, _i32, _i64, ctypes.c_int,
                                      ctypes.c_int, _i64, _vp, _vp, _sz, _vp]


class BloadError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        msg = _lib.bload_status_string(status).decode()
        if status == EHIP:
            msg += f" (hipError {_lib.bload_last_hip_error()})"
        super().__init__(msg)


def status_string(status: int) -> str:
    return _lib.bload_status_string(status).decode()


def _check(status: int) -> None:
    if status != OK:
        raise BloadError(status)


def _ptr(t, dtype=None) -> int:
    if t is None:
        return 0
    if not t.is_cuda:
        raise ValueError("expected a device tensor")
    if not t.is_contiguous():
        raise ValueError("expected a contiguous tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def bload_plan_workspace_bytes(n_seq: int) -> int:
    return int(_lib.bload_plan_workspace_bytes(n_seq))


def bload_pack_workspace_bytes(n_seq: int, num_blocks: int, t_blk: int, frame_bytes: int) -> int:
    return int(_lib.bload_pack_workspace_bytes(n_seq, num_blocks, t_blk, frame_bytes))


def bload_segment_reduce_workspace_bytes(num_blocks: int, t_blk: int, feat_dim: int,
                                         dtype: str) -> int:
    return int(_lib.bload_segment_reduce_workspace_bytes(num_blocks, t_blk, feat_dim,
                                                         DTYPES[dtype]))


@dataclass
class Plan:
    """Device-resident result of ``bload_plan``."""
    order: torch.Tensor            # int32[N]
    block_of_seq: torch.Tensor     # int32[N]
    offset_of_seq: torch.Tensor    # int32[N]
    block_first: torch.Tensor      # int32[N+1], entries [0..B] valid
    num_blocks: int
    total_frames: int
    t_blk: int


def bload_plan(lengths: torch.Tensor, t_blk: int, seed: int, workspace: torch.Tensor | None = None,
               out: Plan | None = None) -> Plan:
    """lengths: int32[N] on the device.  Synchronises the current stream."""
    n = lengths.shape[0]
    dev = lengths.device
    if out is None:
        out = Plan(torch.empty(n, dtype=torch.int32, device=dev),
                   torch.empty(n, dtype=torch.int32, device=dev),
                   torch.empty(n, dtype=torch.int32, device=dev),
                   torch.empty(n + 1, dtype=torch.int32, device=dev), 0, 0, t_blk)
    need = bload_plan_workspace_bytes(n)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    nb, tot = _i64(0), _i64(0)
    st = _lib.bload_plan(_ptr(lengths, torch.int32), n, t_blk, seed & (2**64 - 1),
                         _ptr(out.order, torch.int32), _ptr(out.block_of_seq, torch.int32),
                         _ptr(out.offset_of_seq, torch.int32), _ptr(out.block_first, torch.int32),
                         ctypes.byref(nb), ctypes.byref(tot), _ptr(workspace),
                         workspace.numel() * workspace.element_size(), _stream())
    _check(st)
    out.num_blocks, out.total_frames, out.t_blk = int(nb.value), int(tot.value), t_blk
    return out


def bload_plan_random_fit_workspace_bytes(n_seq: int) -> int:
    return int(_lib.bload_plan_random_fit_workspace_bytes(n_seq))


def bload_plan_random_fit(lengths: torch.Tensor, t_blk: int, seed: int,
                          workspace: torch.Tensor | None = None, out: Plan | None = None) -> Plan:
    """The plan built with the paper's sampler (uniform among the remaining sequences that
    still fit the open block).  lengths: int32[N] on the device.  Synchronises the current
    stream."""
    n = lengths.shape[0]
    dev = lengths.device
    if out is None:
        out = Plan(torch.empty(n, dtype=torch.int32, device=dev),
                   torch.empty(n, dtype=torch.int32, device=dev),
                   torch.empty(n, dtype=torch.int32, device=dev),
                   torch.empty(n + 1, dtype=torch.int32, device=dev), 0, 0, t_blk)
    if workspace is None:
        workspace = torch.empty(max(bload_plan_random_fit_workspace_bytes(n), 16), dtype=torch.uint8,
                                device=dev)
    nb, tot = _i64(0), _i64(0)
    st = _lib.bload_plan_random_fit(_ptr(lengths, torch.int32), n, t_blk, seed & (2**64 - 1),
                                    _ptr(out.order, torch.int32), _ptr(out.block_of_seq, torch.int32),
                                    _ptr(out.offset_of_seq, torch.int32),
                                    _ptr(out.block_first, torch.int32), ctypes.byref(nb),
                                    ctypes.byref(tot), _ptr(workspace),
                                    workspace.numel() * workspace.element_size(), _stream())
    _check(st)
    out.num_blocks, out.total_frames, out.t_blk = int(nb.value), int(tot.value), t_blk
    return out


def bload_plan_shard(plan: Plan, rank: int, world: int) -> Plan:
    """Worker ``rank``'s share of ``plan`` (blocks rank mod world, plus a padding block for
    the workers that would fall short) as a Plan in the worker's own block numbering.
    Synchronises the current stream."""
    n = plan.order.shape[0]
    dev = plan.order.device
    nb_local = -(-plan.num_blocks // world) if world > 0 else 0     # the library refuses world < 1
    out = Plan(torch.empty(n, dtype=torch.int32, device=dev),
               torch.empty(n, dtype=torch.int32, device=dev), plan.offset_of_seq,
               torch.empty(nb_local + 1, dtype=torch.int32, device=dev), nb_local,
               plan.total_frames, plan.t_blk)
    ws = torch.empty(16, dtype=torch.uint8, device=dev)
    nb, ns = _i64(0), _i64(0)
    st = _lib.bload_plan_shard(_ptr(plan.order, torch.int32), _ptr(plan.block_of_seq, torch.int32),
                               _ptr(plan.block_first, torch.int32), n, plan.num_blocks, rank, world,
                               _ptr(out.order, torch.int32), _ptr(out.block_of_seq, torch.int32),
                               _ptr(out.block_first, torch.int32), ctypes.byref(nb),
                               ctypes.byref(ns), _ptr(ws), 16, _stream())
    _check(st)
    assert nb.value == nb_local
    out.n_local = int(ns.value)
    return out


@dataclass
class Packed:
    """Device-resident result of ``bload_pack``."""
    packed: torch.Tensor      # uint8[B, T, frame_bytes]
    seq_id: torch.Tensor      # int32[B, T]
    frame_idx: torch.Tensor   # int32[B, T]
    reset: torch.Tensor       # uint8[B, T]
    valid: torch.Tensor       # uint8[B, T]


def alloc_packed(num_blocks: int, t_blk: int, frame_bytes: int, device) -> Packed:
    return Packed(torch.empty((num_blocks, t_blk, frame_bytes), dtype=torch.uint8, device=device),
                  torch.empty((num_blocks, t_blk), dtype=torch.int32, device=device),
                  torch.empty((num_blocks, t_blk), dtype=torch.int32, device=device),
                  torch.empty((num_blocks, t_blk), dtype=torch.uint8, device=device),
                  torch.empty((num_blocks, t_blk), dtype=torch.uint8, device=device))


def bload_pack(src: torch.Tensor, src_offsets: torch.Tensor, lengths: torch.Tensor, plan: Plan,
               frame_bytes: int, out: Packed | None = None,
               workspace: torch.Tensor | None = None) -> Packed:
    """src: the ragged source (any dtype, contiguous, ``total_frames * frame_bytes`` bytes);
    src_offsets: int64[N+1].  Asynchronous on the current stream."""
    n = lengths.shape[0]
    if src.numel() * src.element_size() != plan.total_frames * frame_bytes:
        raise ValueError("source size does not match total_frames * frame_bytes")
    if out is None:
        out = alloc_packed(plan.num_blocks, plan.t_blk, frame_bytes, lengths.device)
    if out.packed.numel() != plan.num_blocks * plan.t_blk * frame_bytes or \
            out.seq_id.numel() != plan.num_blocks * plan.t_blk:
        raise ValueError("output buffers do not match num_blocks * t_blk")
    if workspace is None:
        need = bload_pack_workspace_bytes(n, plan.num_blocks, plan.t_blk, frame_bytes)
        workspace = torch.empty(max(need, 32), dtype=torch.uint8, device=lengths.device)
    st = _lib.bload_pack(_ptr(src), _ptr(src_offsets, torch.int64), _ptr(lengths, torch.int32),
                         _ptr(plan.order, torch.int32), _ptr(plan.block_of_seq, torch.int32),
                         _ptr(plan.offset_of_seq, torch.int32), _ptr(plan.block_first, torch.int32),
                         n, plan.num_blocks, plan.t_blk, frame_bytes,
                         _ptr(out.packed, torch.uint8), _ptr(out.seq_id, torch.int32),
                         _ptr(out.frame_idx, torch.int32), _ptr(out.reset, torch.uint8),
                         _ptr(out.valid, torch.uint8), _ptr(workspace),
                         workspace.numel() * workspace.element_size(), _stream())
    _check(st)
    return out


PACK_NOALLOC_MAX_SEQ = 1 << 18
PACK_NOALLOC_MAX_TILES = 1 << 21


def bload_pack_noalloc(src: torch.Tensor, src_offsets: torch.Tensor, lengths: torch.Tensor, plan: Plan,
                       frame_bytes: int, out: Packed) -> Packed:
    """``bload_pack`` with its scratch in the library's fixed device array: nothing is allocated
    here or in the library, so ``out`` must be brought along.  Asynchronous on the current
    stream; calls on one GPU must not overlap."""
    if src.numel() * src.element_size() != plan.total_frames * frame_bytes:
        raise ValueError("source size does not match total_frames * frame_bytes")
    if out.packed.numel() != plan.num_blocks * plan.t_blk * frame_bytes or \
            out.seq_id.numel() != plan.num_blocks * plan.t_blk:
        raise ValueError("output buffers do not match num_blocks * t_blk")
    st = _lib.bload_pack_noalloc(_ptr(src), _ptr(src_offsets, torch.int64), _ptr(lengths, torch.int32),
                                 _ptr(plan.order, torch.int32), _ptr(plan.block_of_seq, torch.int32),
                                 _ptr(plan.offset_of_seq, torch.int32), _ptr(plan.block_first, torch.int32),
                                 lengths.shape[0], plan.num_blocks, plan.t_blk, frame_bytes,
                                 _ptr(out.packed, torch.uint8), _ptr(out.seq_id, torch.int32),
                                 _ptr(out.frame_idx, torch.int32), _ptr(out.reset, torch.uint8),
                                 _ptr(out.valid, torch.uint8), _stream())
    _check(st)
    return out


def bload_pack_check(src_offsets: torch.Tensor, lengths: torch.Tensor, plan: Plan,
                     total_frames: int | None = None) -> int:
    """-1 if the tables are a plan ``bload_pack`` can take, else the smallest shuffled position
    or block at which they are not.  Synchronises the current stream."""
    ws = torch.empty(16, dtype=torch.uint8, device=lengths.device)
    bad = _i64(-1)
    st = _lib.bload_pack_check(_ptr(src_offsets, torch.int64), _ptr(lengths, torch.int32),
                               _ptr(plan.order, torch.int32), _ptr(plan.block_of_seq, torch.int32),
                               _ptr(plan.offset_of_seq, torch.int32), _ptr(plan.block_first, torch.int32),
                               lengths.shape[0], plan.num_blocks, plan.t_blk,
                               plan.total_frames if total_frames is None else total_frames,
                               ctypes.byref(bad), _ptr(ws), 16, _stream())
    if st == EINVAL and bad.value >= 0:
        return int(bad.value)
    _check(st)
    return -1


def bload_segment_reduce(packed: torch.Tensor, seq_id: torch.Tensor, reset: torch.Tensor,
                         valid: torch.Tensor, num_blocks: int, t_blk: int, feat_dim: int,
                         dtype: str, op: str, n_seq: int, out: torch.Tensor | None = None,
                         workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Per-sequence sum / mean over the packed blocks -> [n_seq, feat_dim] (float32, or int64
    for ``i32``).  Rows of sequences that do not occur keep their previous content (zeros when
    this function allocates ``out``).  Asynchronous on the current stream."""
    dev = packed.device
    if out is None:
        out = torch.zeros((n_seq, feat_dim), device=dev,
                          dtype=torch.int64 if dtype == "i32" else torch.float32)
    need = bload_segment_reduce_workspace_bytes(num_blocks, t_blk, feat_dim, dtype)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    esize = torch.empty(0, dtype=TORCH_DTYPE[dtype]).element_size()
    if packed.numel() * packed.element_size() != num_blocks * t_blk * feat_dim * esize:
        raise ValueError("packed size does not match num_blocks * t_blk * feat_dim")
    st = _lib.bload_segment_reduce(_ptr(packed), _ptr(seq_id, torch.int32),
                                   _ptr(reset, torch.uint8), _ptr(valid, torch.uint8),
                                   num_blocks, t_blk, feat_dim, DTYPES[dtype], OPS[op], n_seq,
                                   _ptr(out), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream())
    _check(st)
    return out


def bload_strategy_counts(lengths: torch.Tensor, t_chunk: int, t_max: int = 0, num_blocks: int = 0,
                          t_blk: int = 0, workspace: torch.Tensor | None = None) -> dict:
    """Frames of padding / frames deleted under padding to the longest sequence, chunk sampling
    with pieces of ``t_chunk`` frames, and block packing (``num_blocks`` x ``t_blk``).
    ``t_max`` <= 0 pads to the longest sequence found.  Synchronises the current stream."""
    if workspace is None:
        workspace = torch.empty(64, dtype=torch.uint8, device=lengths.device)
    out = StrategyCounts()
    st = _lib.bload_strategy_counts(_ptr(lengths, torch.int32), lengths.shape[0], t_max, t_chunk,
                                    num_blocks, t_blk, ctypes.byref(out), _ptr(workspace),
                                    workspace.numel() * workspace.element_size(), _stream())
    _check(st)
    return out.as_dict()


def bload_segment_scan_workspace_bytes(num_blocks: int, t_blk: int, feat_dim: int, dtype: str) -> int:
    return int(_lib.bload_segment_scan_workspace_bytes(num_blocks, t_blk, feat_dim, DTYPES[dtype]))


def bload_segment_scan(packed: torch.Tensor, reset: torch.Tensor, valid: torch.Tensor, num_blocks: int,
                       t_blk: int, feat_dim: int, dtype: str, decay: float,
                       out: torch.Tensor | None = None,
                       workspace: torch.Tensor | None = None) -> torch.Tensor:
    """h = x at sequence starts, decay * h_prev + x elsewhere, 0 on padding: float32
    [num_blocks, t_blk, feat_dim].  Asynchronous on the current stream."""
    if out is None:
        out = torch.empty((num_blocks, t_blk, feat_dim), dtype=torch.float32, device=packed.device)
    if workspace is None:
        need = bload_segment_scan_workspace_bytes(num_blocks, t_blk, feat_dim, dtype) if dtype != "i32" else 0
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=packed.device)
    st = _lib.bload_segment_scan(_ptr(packed), _ptr(reset, torch.uint8), _ptr(valid, torch.uint8),
                                 num_blocks, t_blk, feat_dim, DTYPES[dtype], float(decay),
                                 _ptr(out, torch.float32), _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream())
    _check(st)
    return out


def bload_pack_tile_bytes(n_seq: int, num_blocks: int, t_blk: int, frame_bytes: int,
                          src_aligned_16: bool = True) -> int:
    """4096 if ``bload_pack`` cuts the packed tensor into 4 KiB tiles for these sizes
    (pack_wide_kernel), 0 if into tiles of 1024 slots (pack_narrow_kernel)."""
    return int(_lib.bload_pack_tile_bytes(n_seq, num_blocks, t_blk, frame_bytes, int(src_aligned_16)))
