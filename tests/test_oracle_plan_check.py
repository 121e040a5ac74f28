"""Pins for the oracle's plan check (Methods section: a block is whole sequences laid one
after another from its first slot, none beyond its end).  Independent of its own rules:
every plan the planners make is accepted, planted mistakes are found at the position where
they were planted, and whatever it accepts is, cell by cell, a layout in which no two
sequences share a slot and none leaves its block."""
import numpy as np
import pytest

import oracle
from paper_2310_10879_amd import workloads


def tables(L, T, seed=3, planner="next-fit"):
    n = len(L)
    pl = oracle.plan(L, T, oracle.order(n, seed)) if planner == "next-fit" else oracle.plan_random_fit(L, T, seed)
    bf = np.zeros(n + 1, dtype=np.int32)
    bf[:pl.num_blocks + 1] = pl.block_first
    return dict(so=workloads.src_offsets(L), L=L.copy(), order=pl.order.copy(), block=pl.block_of_seq.copy(),
                off=pl.offset_of_seq.copy(), bf=bf, B=pl.num_blocks, T=T, total=int(L.sum()))


def check(t):
    return oracle.plan_check(t["so"], t["L"], t["order"], t["block"], t["off"], t["bf"], t["B"], t["T"],
                             t["total"])


def layout_is_sound(t):
    """Brute force: paint every listed sequence into a [B, T] grid of cells."""
    grid = np.zeros((t["B"], t["T"]), dtype=np.int32)
    listed = t["bf"][t["B"]]
    seen = set()
    for p in range(listed):
        i = int(t["order"][p])
        if i in seen or not (0 <= i < len(t["L"])):
            return False
        seen.add(i)
        b, o, n = int(t["block"][i]), int(t["off"][i]), int(t["L"][i])
        if not (0 <= b < t["B"]) or o < 0 or o + n > t["T"] or n < 1:
            return False
        grid[b, o:o + n] += 1
    if grid.max() > 1:
        return False
    # valid cells form a prefix of every block (sequences one after another from slot 0)
    fill = grid.sum(axis=1)
    return bool(np.all(grid == (np.arange(t["T"])[None, :] < fill[:, None])))


@pytest.mark.parametrize("planner", ["next-fit", "random-fit"])
@pytest.mark.parametrize("n,T,kind", [(1, 5, "uniform"), (7, 9, "uniform"), (300, 33, "mixed"),
                                      (2000, 64, "short"), (500, 700, "long")])
def test_planners_make_plans_that_pass(planner, n, T, kind):
    L = workloads.random_lengths(np.random.default_rng(n + T), n, T, kind)
    t = tables(L, T, planner=planner)
    assert check(t) == -1 and layout_is_sound(t)


@pytest.mark.parametrize("world", [2, 3, 8])
def test_worker_shares_pass(world):
    L = workloads.random_lengths(np.random.default_rng(world), 400, 50, "mixed")
    pl = oracle.plan(L, 50, oracle.order(400, 1))
    so = workloads.src_offsets(L)
    for rank in range(world):
        sh = oracle.plan_shard(pl, rank, world)
        bf = np.zeros(401, dtype=np.int32)
        bf[:sh.num_blocks + 1] = sh.block_first
        assert oracle.plan_check(so, L, sh.order, sh.block_of_seq, sh.offset_of_seq, bf, sh.num_blocks, 50,
                                 int(L.sum())) == -1


def test_planted_mistakes_are_found_where_they_are():
    L = workloads.random_lengths(np.random.default_rng(4), 200, 40, "uniform")
    base = tables(L, 40)
    assert check(base) == -1
    p = 57
    i = int(base["order"][p])
    b = int(base["block"][i])

    def with_(**kw):
        t = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in base.items()}
        for name, (idx, val) in kw.items():
            t[name][idx] = val
        return t

    assert check(with_(off=(i, base["off"][i] + 1))) == p                 # a gap in front of it
    assert check(with_(off=(i, -1))) == p
    assert check(with_(block=(i, b + 1))) == p                            # in a block that does not list it
    assert check(with_(block=(i, base["B"]))) == p
    assert check(with_(order=(p, -1))) == p
    assert check(with_(order=(p, 200))) == p
    assert check(with_(order=(p, int(base["order"][p + 5])))) == p        # a sequence listed twice
    assert check(with_(L=(i, 0))) == p
    assert check(with_(so=(i, base["so"][i] + 1))) <= p                   # source range does not match L
    # a sequence pushed beyond the block's end: make the block's last one longer
    last_p = int(base["bf"][b + 1]) - 1
    j = int(base["order"][last_p])
    longer = with_(L=(j, 40 - base["off"][j] + 1))
    assert check(longer) == last_p
    # block ranges: not starting at 0, decreasing, beyond n
    assert check(with_(bf=(0, 1))) == 0
    assert check(with_(bf=(3, int(base["bf"][2]) - 1))) == 2
    t = with_(bf=(base["B"], 201))
    assert check(t) == base["B"] - 1
    # the source ends too early
    short = dict(base)
    short["total"] = base["total"] - 1
    assert 0 <= check(short) < 200


def test_accepted_tables_are_sound_layouts_under_random_damage():
    rng = np.random.default_rng(11)
    accepted = rejected = 0
    for trial in range(400):
        n, T = int(rng.integers(1, 30)), int(rng.integers(1, 12))
        L = workloads.random_lengths(rng, n, T, "uniform")
        t = tables(L, T, seed=trial)
        for _ in range(int(rng.integers(0, 3))):            # 0, 1 or 2 random edits
            name = ["order", "block", "off", "bf", "L"][int(rng.integers(0, 5))]
            idx = int(rng.integers(0, (t["B"] + 1) if name == "bf" else n))
            t[name][idx] = int(rng.integers(-1, max(n, T) + 2))
        t["so"] = workloads.src_offsets(np.maximum(t["L"], 0))
        t["total"] = int(t["so"][-1])
        ok = check(t) == -1
        if ok:
            accepted += 1
            assert layout_is_sound(t), f"trial {trial}: accepted tables that are not a layout"
        else:
            rejected += 1
    assert accepted > 50 and rejected > 50
