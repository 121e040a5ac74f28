"""bload_pack_check on the GPU against the oracle's plan check: the same verdict and the same
first failing index on sound tables, on a worker's share, and on tables damaged at random.
(Only the check runs on damaged tables; nothing is packed from them.)"""
import numpy as np
import pytest
import torch

import oracle
from paper_2310_10879_amd import workloads
from gpu_util import binding, gpu_plan, to_dev

pytestmark = pytest.mark.gpu


def gpu_check(bl, so, L, order, block, off, bf, B, T, total):
    plan = bl.Plan(to_dev(order), to_dev(block), to_dev(off), to_dev(bf), B, total, T)
    return bl.bload_pack_check(to_dev(so), to_dev(L), plan, total)


@pytest.mark.parametrize("n,T,kind", [(1, 5, "uniform"), (300, 33, "mixed"), (5000, 64, "short"),
                                      (70000, 700, "uniform")])
def test_plans_of_the_planners_pass(n, T, kind):
    bl = binding()
    L = workloads.random_lengths(np.random.default_rng(n), n, T, kind)
    so = workloads.src_offsets(L)
    for make in (bl.bload_plan, bl.bload_plan_random_fit):
        plan = make(to_dev(L), T, 9)
        assert bl.bload_pack_check(to_dev(so), to_dev(L), plan) == -1
        share = bl.bload_plan_shard(plan, 1, 3)
        assert bl.bload_pack_check(to_dev(so), to_dev(L), share) == -1


def test_damaged_tables_fail_where_the_oracle_says():
    bl = binding()
    rng = np.random.default_rng(21)
    verdicts = set()
    for trial in range(150):
        n, T = int(rng.integers(1, 3000)), int(rng.integers(1, 90))
        L = workloads.random_lengths(rng, n, T, "uniform")
        pl = oracle.plan(L, T, oracle.order(n, trial))
        bf = np.zeros(n + 1, dtype=np.int32)
        bf[:pl.num_blocks + 1] = pl.block_first
        t = dict(order=pl.order.copy(), block=pl.block_of_seq.copy(), off=pl.offset_of_seq.copy(), bf=bf,
                 L=L.copy())
        for _ in range(int(rng.integers(0, 3))):
            name = ["order", "block", "off", "bf", "L"][int(rng.integers(0, 5))]
            idx = int(rng.integers(0, (pl.num_blocks + 1) if name == "bf" else n))
            t[name][idx] = int(rng.integers(-1, max(n, T) + 2))
        so = workloads.src_offsets(np.maximum(t["L"], 0))
        total = int(so[-1])
        want = oracle.plan_check(so, t["L"], t["order"], t["block"], t["off"], t["bf"], pl.num_blocks, T, total)
        got = gpu_check(bl, so, t["L"], t["order"], t["block"], t["off"], t["bf"], pl.num_blocks, T, total)
        assert got == want, f"trial {trial}: GPU says {got}, oracle {want}"
        verdicts.add(want >= 0)
    assert verdicts == {True, False}


def test_check_of_a_full_size_plan():
    bl = binding()
    L = workloads.lengths(5)
    so = workloads.src_offsets(L)
    plan = gpu_plan(L, 4096, 0)
    d_so, d_L = to_dev(so), to_dev(L)
    assert bl.bload_pack_check(d_so, d_L, plan) == -1
    i = int(plan.order[777777].item())
    plan.offset_of_seq[i] += 1
    assert bl.bload_pack_check(d_so, d_L, plan) == 777777
