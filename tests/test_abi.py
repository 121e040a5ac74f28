"""The C-ABI library loads and exports every entry point that include/bload.h
declares (no compute calls: this runs without a GPU), and the host-side
argument checks answer before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "bload.h")
LIB = os.path.join(ROOT, "paper_2310_10879_amd", "libbload.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bload_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2310_10879_amd import build
        build.build(verbose=False)
    return ctypes.CDLL(LIB)


def test_header_declares_the_three_entry_points():
    names = declared_functions()
    for must in ("bload_plan", "bload_pack", "bload_segment_reduce", "bload_plan_workspace_bytes",
                 "bload_pack_workspace_bytes", "bload_segment_reduce_workspace_bytes",
                 "bload_status_string"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in bload.h but not exported"


def test_status_strings(lib):
    lib.bload_status_string.restype = ctypes.c_char_p
    seen = set()
    for code in range(7):
        s = lib.bload_status_string(code).decode()
        assert s.startswith("BLOAD_")
        seen.add(s)
    assert len(seen) == 7
    assert "unknown" in lib.bload_status_string(99).decode()


def test_workspace_queries(lib):
    lib.bload_plan_workspace_bytes.restype = ctypes.c_size_t
    lib.bload_plan_workspace_bytes.argtypes = [ctypes.c_int64]
    sizes = [lib.bload_plan_workspace_bytes(n) for n in (0, 1, 1000, 10**6)]
    assert sizes == sorted(sizes) and sizes[-1] >= 21 * 10**6
    assert all(s % 16 == 0 for s in sizes)
    assert lib.bload_plan_workspace_bytes(-1) == 0
    assert lib.bload_plan_workspace_bytes((1 << 27) + 1) == 0
    f = lib.bload_segment_reduce_workspace_bytes
    f.restype = ctypes.c_size_t
    f.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int64, ctypes.c_int]
    tiles = 324084 * 2                             # blocks of 5000 token slots are cut into two tiles each:
    assert f(324084, 5000, 1, 3) == tiles * 16 + 2 * (-(-tiles * 8 // 16) * 16)   # a descriptor and two int64 partials per tile
    assert f(324084, 4096, 1, 3) == 0 and f(5, 2048, 1, 3) == 0 and f(9, 33, 1, 3) == 0   # tiles of whole blocks cut nothing
    assert f(10000, 3000, 80, 2) == 0              # one chunk per block
    chunks = 34576 * 3                             # few long rounds of whole blocks: three chunks per block
    assert f(34576, 3000, 80, 2) == chunks * 16 + 2 * chunks * 80 * 4
    assert f(180, 600, 37632, 0) == 0              # enough blocks x lane-slices: one chunk per block
    assert f(79, 3000, 2048, 1) > 0                # few blocks: cut in time, partial sums needed
    assert f(0, 600, 8, 0) == 0 and f(5, 0, 8, 0) == 0 and f(5, 8, 8, 7) == 0


def test_argument_checks_need_no_gpu(lib):
    # every call below must be refused on the host, before any HIP call
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    nb, tot = i64(7), i64(7)
    lib.bload_plan.restype = ctypes.c_int
    lib.bload_plan.argtypes = [vp, i64, i32, ctypes.c_uint64, vp, vp, vp, vp,
                               ctypes.POINTER(i64), ctypes.POINTER(i64), vp, ctypes.c_size_t, vp]
    p = 0x1000                                      # never dereferenced by a refused call
    assert lib.bload_plan(p, -1, 8, 0, p, p, p, p, nb, tot, p, 1 << 20, None) == 1
    assert lib.bload_plan(p, 4, 0, 0, p, p, p, p, nb, tot, p, 1 << 20, None) == 1
    assert lib.bload_plan(None, 4, 8, 0, p, p, p, p, nb, tot, p, 1 << 20, None) == 1
    assert lib.bload_plan(p, 4, 8, 0, p, p, p, p, nb, tot, p, 8, None) == 3
    assert lib.bload_plan(p, 4, 8, 0, p + 2, p, p, p, nb, tot, p, 1 << 20, None) == 4
    assert lib.bload_plan(p, (1 << 27) + 1, 8, 0, p, p, p, p, nb, tot, p, 1 << 20, None) == 5
    assert lib.bload_plan(p, 0, 8, 0, p, p, p, p, nb, tot, p, 0, None) == 0
    assert (nb.value, tot.value) == (0, 0)
    rf = lib.bload_plan_random_fit
    rf.restype = ctypes.c_int
    rf.argtypes = lib.bload_plan.argtypes
    nb.value = tot.value = 7
    assert rf(p, -1, 8, 0, p, p, p, p, nb, tot, p, 1 << 20, None) == 1
    assert rf(p, 4, 0, 0, p, p, p, p, nb, tot, p, 1 << 20, None) == 1
    assert rf(None, 4, 8, 0, p, p, p, p, nb, tot, p, 1 << 20, None) == 1
    assert rf(p, 4, 8, 0, p, p, p, p, nb, tot, p, 8, None) == 3
    assert rf(p, 4, 8, 0, p, p + 2, p, p, nb, tot, p, 1 << 20, None) == 4
    assert rf(p, 4, 8193, 0, p, p, p, p, nb, tot, p, 1 << 20, None) == 5       # t_blk beyond the on-chip counts
    assert rf(p, (1 << 27) + 1, 8, 0, p, p, p, p, nb, tot, p, 1 << 20, None) == 5
    assert rf(p, 0, 8, 0, p, p, p, p, nb, tot, p, 0, None) == 0
    assert (nb.value, tot.value) == (0, 0)
    w = lib.bload_plan_random_fit_workspace_bytes
    w.restype = ctypes.c_size_t
    w.argtypes = [i64]
    assert w(-1) == 0 and w((1 << 27) + 1) == 0 and w(1000) % 16 == 0
    assert 28 * 10**6 + 128 * 8192 * 4 <= w(10**6) <= 28 * 10**6 + 128 * 8192 * 4 + 70000   # + the chunks' length counts
    lib.bload_pack.restype = ctypes.c_int
    lib.bload_pack.argtypes = [vp] * 7 + [i64, i64, i32, i64] + [vp] * 6 + [ctypes.c_size_t, vp]
    p = 0x1000 * 2                                  # 32-byte aligned, never dereferenced
    ok = [p] * 7 + [4, 2, 8, 16] + [p] * 5 + [p, 1 << 20, None]
    assert lib.bload_pack(*(ok[:7] + [4, 2, 0, 16] + ok[11:])) == 1          # t_blk < 1
    assert lib.bload_pack(*(ok[:7] + [4, 2, 8, 0] + ok[11:])) == 1           # frame_bytes < 1
    assert lib.bload_pack(*([None] + ok[1:])) == 1                           # null source
    assert lib.bload_pack(*(ok[:11] + [p + 4] + ok[12:])) == 4               # packed misaligned
    assert lib.bload_pack(*(ok[:7] + [0, 0, 8, 16] + ok[11:])) == 0          # nothing to do
    assert lib.bload_pack(*(ok[:7] + [4, 2, 8, 4096] + ok[11:16] + [p, 8, None])) == 3   # workspace
    f = lib.bload_pack_workspace_bytes
    f.restype = ctypes.c_size_t
    f.argtypes = [i64, i64, i32, i64]
    need = 32 * 1000 + 4 * -(-180 * 600 * 37632 // 4096)     # a 32-byte run per sequence, an int32 per 4 KiB tile
    assert need <= f(1000, 180, 600, 37632) < need + 16 and f(1000, 180, 600, 37632) % 16 == 0
    # from 2^21 slots on, one more int32 per 1024 slots for the pass that writes the start table
    need = 32 * 50000 + 4 * -(-34576 * 3000 * 320 // 4096) + 4 * -(-34576 * 3000 // 1024)
    assert need <= f(50000, 34576, 3000, 320) < need + 32
    assert f(1000, 180, 600, 4) == 32 * 1000 + 4 * -(-180 * 600 // 1024) + 8
    assert f(1000, 0, 600, 4096) == 0 and f(0, 5, 600, 4096) == 0
    assert f(10**6, 200, 8, 64) >= 32 * 10**6 + 4 * 2          # frames that may take either tile shape
    chk = lib.bload_pack_check
    chk.restype = ctypes.c_int
    chk.argtypes = [vp] * 6 + [i64, i64, i32, i64, ctypes.POINTER(i64), vp, ctypes.c_size_t, vp]
    bad = i64(7)
    assert chk(p, p, p, p, p, p, 4, 2, 0, 9, bad, p, 16, None) == 1 and bad.value == -1     # t_blk < 1
    assert chk(p, p, p, p, p, p, 4, 5, 8, 9, bad, p, 16, None) == 1                        # more blocks than sequences
    assert chk(None, p, p, p, p, p, 4, 2, 8, 9, bad, p, 16, None) == 1
    assert chk(p, p, p, p, p, p, 4, 2, 8, 9, None, p, 8, None) == 3
    assert chk(p, p, p + 2, p, p, p, 4, 2, 8, 9, bad, p, 16, None) == 4
    assert chk(p, p, p, p, p, p, 0, 0, 8, 0, bad, p, 16, None) == 0
    tb = lib.bload_pack_tile_bytes
    tb.restype = i32
    tb.argtypes = [i64, i64, i32, i64, i32]
    assert tb(1000, 180, 600, 37632, 1) == 4096 and tb(10**6, 324084, 4096, 4, 1) == 0
    assert tb(50000, 34576, 3000, 320, 1) == 4096          # long runs of middle-sized frames
    assert tb(4000000, 100000, 64, 320, 1) == 0            # short runs of the same frames
    assert tb(10, 0, 600, 64, 1) == 0 and tb(10, 5, 600, 0, 1) == 0
    lib.bload_plan_shard.restype = ctypes.c_int
    lib.bload_plan_shard.argtypes = [vp, vp, vp, i64, i64, i32, i32, vp, vp, vp,
                                     ctypes.POINTER(i64), ctypes.POINTER(i64), vp, ctypes.c_size_t, vp]
    assert lib.bload_plan_shard(p, p, p, 4, 2, 2, 2, p, p, p, nb, tot, p, 16, None) == 1     # rank >= world
    assert lib.bload_plan_shard(p, p, p, 4, 2, 0, 0, p, p, p, nb, tot, p, 16, None) == 1     # world < 1
    assert lib.bload_plan_shard(p, p, p, 4, 2, 0, 2, p, p, p, nb, tot, p, 8, None) == 3      # workspace
    assert lib.bload_plan_shard(p, p, p, 0, 0, 0, 2, p, p, p, nb, tot, p, 16, None) == 0
    assert (nb.value, tot.value) == (0, 0)
    scan = lib.bload_segment_scan
    scan.restype = ctypes.c_int
    scan.argtypes = [vp, vp, vp, i64, i32, i64, ctypes.c_int, ctypes.c_float, vp, vp, ctypes.c_size_t, vp]
    assert scan(p, p, p, 2, 8, 4, 3, 0.5, p, p, 1 << 20, None) == 1       # int32 payload
    assert scan(p, p, p, 2, 0, 4, 2, 0.5, p, p, 1 << 20, None) == 1
    assert scan(p, p, p, 2, 8, 0, 2, 0.5, p, p, 1 << 20, None) == 1
    assert scan(p, None, p, 2, 8, 4, 2, 0.5, p, p, 1 << 20, None) == 1
    assert scan(p + 4, p, p, 2, 8, 4, 2, 0.5, p, p, 1 << 20, None) == 4
    assert scan(p, p, p, 2, 8, 4, 2, 0.5, p + 8, p, 1 << 20, None) == 4
    assert scan(p, p, p, 2, 3000, 4, 2, 0.5, p, p, 16, None) == 3         # chunks need their states
    assert scan(p, p, p, 0, 8, 4, 2, 0.5, p, p, 0, None) == 0
    sw = lib.bload_segment_scan_workspace_bytes
    sw.restype = ctypes.c_size_t
    sw.argtypes = [i64, i32, i64, ctypes.c_int]
    assert sw(2, 8, 4, 2) == 0 and sw(2, 8, 4, 3) == 0                    # one chunk: nothing handed on
    assert sw(2, 3000, 4, 2) >= 2 * 4 * 4 and sw(2, 3000, 4, 2) % 16 == 0
    sc = lib.bload_strategy_counts
    sc.restype = ctypes.c_int
    sc.argtypes = [vp, i64, i32, i32, i64, i32, vp, vp, ctypes.c_size_t, vp]
    counts = (i64 * 6)(*([7] * 6))
    assert sc(p, 4, 0, 0, 0, 0, counts, p, 64, None) == 1                  # t_chunk < 1
    assert sc(p, 4, 0, 5, 0, 0, None, p, 64, None) == 1                   # nowhere to report
    assert sc(None, 4, 0, 5, 0, 0, counts, p, 64, None) == 1
    assert sc(p, 4, 0, 5, 0, 0, counts, p, 32, None) == 3
    assert sc(p + 2, 4, 0, 5, 0, 0, counts, p, 64, None) == 4
    assert sc(p, 0, 0, 5, 0, 0, counts, p, 64, None) == 0 and list(counts) == [0] * 6
    lib.bload_segment_reduce.restype = ctypes.c_int
    lib.bload_segment_reduce.argtypes = [vp, vp, vp, vp, i64, i32, i64, ctypes.c_int, ctypes.c_int,
                                         i64, vp, vp, ctypes.c_size_t, vp]
    assert lib.bload_segment_reduce(p, p, p, p, 2, 8, 4, 3, 1, 4, p, p, 1 << 20, None) == 1  # i32 mean
    assert lib.bload_segment_reduce(p, p, p, p, 2, 8, 4, 9, 0, 4, p, p, 1 << 20, None) == 1
    assert lib.bload_segment_reduce(p, p, p, p, 2, 8, 0, 0, 0, 4, p, p, 1 << 20, None) == 1
    assert lib.bload_segment_reduce(p + 1, p, p, p, 2, 8, 4, 0, 0, 4, p, p, 1 << 20, None) == 4
    assert lib.bload_segment_reduce(p, p, p, p, 50, 5000, 1, 2, 0, 4, p, p, 8, None) == 3
    assert lib.bload_segment_reduce(p, p, p, p, 0, 8, 4, 0, 0, 4, p, p, 0, None) == 0


# ---- the yardstick library (include/bload_yardsticks.h) ----------------------------------

YS_HEADER = os.path.join(ROOT, "include", "bload_yardsticks.h")
YS_LIB = os.path.join(ROOT, "paper_2310_10879_amd", "libbload_yardsticks.so")


@pytest.fixture(scope="module")
def ys_lib():
    if not os.path.exists(YS_LIB):
        from paper_2310_10879_amd import build
        build.build(verbose=False)
    return ctypes.CDLL(YS_LIB)


def test_yardstick_library_exports_every_declared_symbol(ys_lib, lib):
    text = re.sub(r"/\*.*?\*/", "", open(YS_HEADER).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(bload_ys_[a-z_]+)\s*\(", text)))
    assert names == ["bload_ys_copy", "bload_ys_read", "bload_ys_rows", "bload_ys_token_pack"]
    for name in names:
        assert hasattr(ys_lib, name), f"{name} is declared in bload_yardsticks.h but not exported"
        assert not hasattr(lib, name), f"{name} belongs to the yardstick library, not to libbload.so"


def test_yardstick_argument_checks_need_no_gpu(ys_lib):
    vp, i64, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t
    ys_lib.bload_ys_copy.argtypes = [vp, vp, sz, vp]
    ys_lib.bload_ys_read.argtypes = [vp, sz, vp, vp]
    ys_lib.bload_ys_token_pack.argtypes = [vp, vp, vp, vp, vp, vp, i64, ctypes.c_int, ctypes.c_int, vp]
    ys_lib.bload_ys_rows.argtypes = [vp, vp, i64, i64, ctypes.c_int, ctypes.c_int, vp, vp]
    p = 0x1000                                           # never dereferenced: every call below is refused or empty
    assert ys_lib.bload_ys_copy(None, p, 16, None) == 1
    assert ys_lib.bload_ys_copy(p, p, 17, None) == 1     # not a multiple of 16
    assert ys_lib.bload_ys_copy(p + 4, p, 16, None) == 1  # base not 16-byte aligned
    assert ys_lib.bload_ys_copy(p, p, 0, None) == 0
    assert ys_lib.bload_ys_read(p, 16, None, None) == 1
    assert ys_lib.bload_ys_read(p, 0, p, None) == 0
    assert ys_lib.bload_ys_token_pack(p, p, p, p, p, p, 4097, 0, 0, None) == 1
    assert ys_lib.bload_ys_token_pack(p, p, p, p, p, p, 4096, 101, 0, None) == 1
    assert ys_lib.bload_ys_token_pack(p, p, p, None, p, p, 4096, 0, 0, None) == 1
    assert ys_lib.bload_ys_token_pack(p, p, p, p, p, p, 0, 0, 0, None) == 0
    assert ys_lib.bload_ys_rows(p, None, 10, 8 * 16 * 20, 3, 20, p, None) == 1     # rows per wave: 1, 2 or 4
    assert ys_lib.bload_ys_rows(p, None, 10, 8 * 16 * 20, 2, 33, p, None) == 1     # more lanes than a row has
    assert ys_lib.bload_ys_rows(p, None, 10, 8 * 16 * 20 + 16, 2, 20, p, None) == 1  # not whole batches
    assert ys_lib.bload_ys_rows(p, None, 0, 8 * 16 * 20, 2, 20, p, None) == 0
