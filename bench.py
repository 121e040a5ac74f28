#!/usr/bin/env python3
"""Benchmark of the BLoad block packer on one MI355X.

A step is one pass of the whole path over one synthetic workload that is
already resident in HBM: bload_plan (order + next-fit; --plan random-fit takes
the paper's sampler instead), bload_pack (gather, zero padding, start table)
and bload_segment_reduce (per-sequence reduction over the packed blocks).
The recurrent consumer (bload_segment_scan) is timed in a loop of its own
behind the steps.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 4] [--only]
                    [--plan next-fit] [--no-cpu-baseline] [--no-scan]

The headline (`value`, `config`, `roofline`) is workload 4, the largest of the
five (59 GB of traffic per pack); `per_workload` carries all five, each with
the launch time, the algorithmic bytes and the fraction of the HBM roofline of
bload_pack, bload_segment_reduce and bload_segment_scan, and -- for the two
workloads that fit or nearly fit the 256 MB last-level cache -- the same
figures with the buffers rotated so that every step starts cache-cold.

value         valid frames packed per second over the whole path (all K steps)
roofline      the gather/pad kernel against the HBM roofline: algorithmic bytes
              of one launch / its mean duration measured with events on the
              stream it runs on
cpu_baseline  the CPU oracle, one thread, timed on a bounded sample of the
              headline workload
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
CSRC = os.path.join(ROOT, "paper_2310_10879_amd", "csrc")
LAST_LEVEL_CACHE_BYTES = 256 << 20

LENGTHS = {
    1: "uniform integers in [2, 32]",
    2: "lognormal(mu=ln 60, sigma=1) rounded, clipped to [1, 600]",
    3: "floor(8 * (1 + Lomax(1.5))) clipped to [8, 3000]",
    4: "uniform integers in [100, 3000]",
    5: "Zipf(1.2) clipped to [1, 4096]",
}


def measured_traffic(workload: int, family: str):
    """HBM bytes per call of one kernel family ("pack", "reduce", "scan") from the committed
    rocprofv3 counter summary of this workload, or None when there is none or the family's
    source file changed since the counters were taken."""
    path = os.path.join(ROOT, "profiles", f"bload_workload{workload}_hbm_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        rec = json.load(f)
    fam = rec.get("families", {}).get(family)
    if not fam:
        return None
    with open(os.path.join(CSRC, fam["source"]), "rb") as f:
        if hashlib.sha256(f.read()).hexdigest() != fam["source_sha256"]:
            return None
    return fam["hbm_bytes_per_call"]


def roofline_block(kernel, nbytes, ms, traffic):
    gbps = nbytes / (ms * 1e-3) / 1e9
    return {"kernel": kernel, "bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": gbps / HBM_PEAK_GBPS, "algorithmic_bytes_per_launch": int(nbytes), "launch_ms": ms,
            "traffic": traffic}


def run_workload(args, wid: int, cold_sets: int = 0) -> dict:
    """Time `args.steps` steps of workload `wid` (and the scan behind them).  cold_sets > 1:
    the source, the packed outputs and the reduction rows exist that many times and the steps
    rotate through them, so that no step finds its data in a cache."""
    import numpy as np
    import torch

    from paper_2310_10879_amd import bload, workloads

    t_setup = time.perf_counter()
    w = workloads.WORKLOADS[wid]
    dev = torch.device("cuda:0")
    L = workloads.lengths(w.wid)
    so = workloads.src_offsets(L)
    total_frames = int(so[-1])
    src = workloads.source(w.wid, 0, total_frames, threads=16)
    F, T, N, D = w.frame_bytes, w.t_blk, w.n_seq, w.frame_elems
    n_sets = max(1, cold_sets)
    d_srcs = [torch.from_numpy(src.view(np.uint8).reshape(-1)).to(dev) for _ in range(n_sets)]
    del src
    d_so = torch.from_numpy(so).to(dev)
    d_L = torch.from_numpy(L).to(dev)
    seed = 0

    # everything the steps write is allocated once, outside the timed region
    if args.plan == "random-fit":
        make_plan, plan_ws_bytes = bload.bload_plan_random_fit, bload.bload_plan_random_fit_workspace_bytes(N)
    else:
        make_plan, plan_ws_bytes = bload.bload_plan, bload.bload_plan_workspace_bytes(N)
    plan_ws = torch.empty(max(16, plan_ws_bytes), dtype=torch.uint8, device=dev)
    plan = make_plan(d_L, T, seed, workspace=plan_ws)
    sharded = args.world > 1
    if sharded:
        share = bload.bload_plan_shard(plan, args.rank, args.world)
        mine = share.block_of_seq >= 0
        local_frames = int(d_L[mine].sum().item())
        local_seqs = int(mine.sum().item())
    else:
        share, local_frames, local_seqs = plan, total_frames, N
    B = share.num_blocks
    packs = [bload.alloc_packed(B, T, F, dev) for _ in range(n_sets)]
    pack_ws = torch.empty(max(32, bload.bload_pack_workspace_bytes(N, B, T, F)), dtype=torch.uint8, device=dev)
    red_ws = torch.empty(max(16, bload.bload_segment_reduce_workspace_bytes(B, T, D, w.dtype)),
                         dtype=torch.uint8, device=dev)
    reds = [torch.zeros((N, D), dtype=torch.int64 if w.dtype == "i32" else torch.float32, device=dev)
            for _ in range(n_sets)]
    setup_s = time.perf_counter() - t_setup

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]

    def step(k, events=None):
        d_src, packed, red = d_srcs[k % n_sets], packs[k % n_sets], reds[k % n_sets]
        if events:
            events[0].record()
        make_plan(d_L, T, seed, workspace=plan_ws, out=plan)
        todo = bload.bload_plan_shard(plan, args.rank, args.world) if sharded else plan
        if events:
            events[1].record()
        bload.bload_pack(d_src, d_so, d_L, todo, F, out=packed, workspace=pack_ws)
        if events:
            events[2].record()
        bload.bload_segment_reduce(packed.packed, packed.seq_id, packed.reset, packed.valid,
                                   todo.num_blocks, T, D, w.dtype, w.op, N, out=red, workspace=red_ws)
        if events:
            events[3].record()

    if args.calibrate_copy:
        a = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        for _ in range(3):
            torch.mul(a, 1.0, out=b)
        torch.cuda.synchronize()
        del a, b

    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(args.warmup + k, ev[k])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert share.num_blocks == B and plan.total_frames == total_frames

    ms = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(3)] for e in ev])   # plan, pack, reduce
    plan_ms, pack_ms, reduce_ms = (float(x) for x in ms.mean(axis=0))
    slots = B * T
    acc = 8 if w.dtype == "i32" else 4
    # what the method itself has to move (bytes per launch):
    #   pack    valid payload read + every packed byte written + 10 bytes of start table per slot
    #           + 16 bytes of plan tables per sequence
    #   reduce  valid payload + both flag planes read, the sequence id once per sequence, the rows written
    #   scan    valid payload + both flag planes read, a float32 per packed element written
    bytes_pack = local_frames * F + slots * F + 10 * slots + 16 * local_seqs
    bytes_reduce = local_frames * F + 2 * slots + 4 * local_seqs + local_seqs * D * acc
    bytes_scan = local_frames * F + 2 * slots + 4 * slots * D
    whole = args.plan == "next-fit" and not sharded     # what the committed counters were taken on
    wide = bload.bload_pack_tile_bytes(N, B, T, F, d_srcs[0].data_ptr() % 16 == 0)
    out = {
        "workload": f"{w.wid}: N={N} {w.name}, T_blk={T}, frame_bytes={F}, seed={seed}, {args.plan} plan"
                    + (f", share of worker {args.rank} of {args.world}" if sharded else ""),
        "n_seq": N, "t_blk": T, "frame_bytes": F, "total_frames": total_frames, "num_blocks": B,
        "lengths": LENGTHS[w.wid], "dtype": w.dtype,
        "ms_per_step": elapsed / args.steps * 1e3,
        "frames_per_s": local_frames * args.steps / elapsed,
        "work_frames": local_frames,
        "phases_ms": {"plan": plan_ms, "pack": pack_ms, "segment_reduce": reduce_ms},
        # the planner is a latency-bound chain: per sequence it costs
        "plan_ns_per_sequence": plan_ms * 1e6 / max(1, N),
        # the whole call: pack_prepare_kernel, the copy kernel and, for 4 KiB tiles over 2^21 slots or more,
        # the pass that writes the start table (pack_narrow_kernel<unsigned char, false, false>)
        "pack": dict(roofline_block(("pack_wide_kernel + start-table pass" if slots >= 1 << 21 else "pack_wide_kernel")
                                    if wide else "pack_narrow_kernel", bytes_pack, pack_ms,
                                    measured_traffic(w.wid, "pack") if whole else None),
                     frames_per_s=local_frames / (pack_ms * 1e-3), min_ms=float(ms[:, 1].min()),
                     median_ms=float(np.median(ms[:, 1]))),
        "segment_reduce": roofline_block("reduce_*_kernel (+ reduce_stitch_kernel)", bytes_reduce, reduce_ms,
                                         measured_traffic(w.wid, "reduce") if whole else None),
        "padding": {
            "fill": local_frames / slots,
            "pad_blocks_frames": slots - local_frames,
            "pad_to_longest_frames": local_seqs * T - local_frames,
            "pad_ratio_blocks": (slots - local_frames) / slots,
            "pad_ratio_to_longest": (local_seqs * T - local_frames) / (local_seqs * T),
            "reduction_vs_pad_to_longest": (local_seqs * T - local_frames) / max(1, slots - local_frames),
        },
        "buffer_sets": n_sets,
        "setup_s": setup_s,
    }

    if not args.no_scan and w.dtype != "i32" and n_sets == 1:
        scan_out = torch.empty((B, T, D), dtype=torch.float32, device=dev)
        scan_ws = torch.empty(max(16, bload.bload_segment_scan_workspace_bytes(B, T, D, w.dtype)),
                              dtype=torch.uint8, device=dev)
        sev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
        packed = packs[0]
        for k in range(args.warmup + args.steps):
            e = sev[k - args.warmup] if k >= args.warmup else None
            if e:
                e[0].record()
            bload.bload_segment_scan(packed.packed, packed.reset, packed.valid, B, T, D, w.dtype, 0.9,
                                     out=scan_out, workspace=scan_ws)
            if e:
                e[1].record()
        torch.cuda.synchronize()
        scan_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in sev]))
        out["phases_ms"]["segment_scan"] = scan_ms
        out["segment_scan"] = dict(roofline_block("scan_apply_kernel (+ scan_tail_kernel, scan_chain_kernel)",
                                                  bytes_scan, scan_ms,
                                                  measured_traffic(w.wid, "scan") if whole else None), decay=0.9)
        del scan_out, scan_ws

    if n_sets == 1 and not sharded:
        # the strategies of the paper's Table 1 on the same lengths (outside the timed region)
        t_chunk = max(1, total_frames // N)               # pieces of the average length
        out["strategy_counts"] = dict(bload.bload_strategy_counts(d_L, t_chunk, T, plan.num_blocks, T),
                                      t_chunk=t_chunk)
    del d_srcs, packs, reds, pack_ws, red_ws, plan_ws
    torch.cuda.empty_cache()
    return out


def yardsticks() -> dict:
    """What plain kernels reach on this GPU in this run, as same-run references for the roofline
    fractions: torch's elementwise copy (1 GiB read + 1 GiB written) and fill (1 GiB written),
    and the streaming kernels of libbload_yardsticks.so, which move bytes in the patterns of the
    pack, the reduction and the scan without doing anything else."""
    import torch

    dev = torch.device("cuda:0")
    a = torch.ones(1 << 28, dtype=torch.float32, device=dev)
    b = torch.empty_like(a)
    gib = float(1 << 30)

    def gbps(fn, nbytes):
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return nbytes * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9

    out = {"copy_GBps": gbps(lambda: torch.mul(a, 1.0, out=b), 2 * gib),
           "fill_GBps": gbps(lambda: b.fill_(0.0), gib),
           "what": "torch elementwise copy (1 GiB read + 1 GiB written) and fill (1 GiB written)"}
    del a, b
    torch.cuda.empty_cache()
    # what the kernels' access patterns alone reach: plain streaming kernels of the same shapes
    try:
        from paper_2310_10879_amd import yardsticks as ys
        out["patterns"] = ys.measure(dev)
    except Exception as exc:                          # a reference figure, never a reason to fail
        out["patterns"] = {"error": f"{type(exc).__name__}: {exc}"}
    torch.cuda.empty_cache()
    return out


def cpu_baseline(args, wid: int, budget_frames: int) -> dict:
    """The oracle as it stands, one thread: order + plan + pack + reduce of the first sequences
    of the workload (as many as hold about `budget_frames` frames), with the workload's T_blk."""
    import numpy as np

    import oracle
    from paper_2310_10879_amd import workloads

    w = workloads.WORKLOADS[wid]
    L_all = workloads.lengths(wid)
    so_all = workloads.src_offsets(L_all)
    n = int(min(w.n_seq, max(1, np.searchsorted(so_all, budget_frames, side="right") - 1)))
    L, so = L_all[:n], so_all[:n + 1]
    frames = int(so[-1])
    src = workloads.source(wid, 0, frames, threads=16)
    c0 = time.perf_counter()
    ref_plan = (oracle.plan_random_fit(L, w.t_blk, 0) if args.plan == "random-fit"
                else oracle.plan(L, w.t_blk, oracle.order(n, 0)))
    out = oracle.alloc_pack_outputs(ref_plan.num_blocks, w.t_blk, w.frame_bytes)
    c1 = time.perf_counter()
    oracle.pack(src, so, L, ref_plan, w.frame_bytes, out=out)
    c2 = time.perf_counter()
    oracle.segment_reduce(src, so, L, w.frame_elems, w.dtype, w.op)
    c3 = time.perf_counter()
    return {
        "value": frames / (c3 - c0),
        "unit": "frames/s",
        "cores": 1,
        "kind": "oracle",
        "sample": f"the first {n} of the {w.n_seq} sequences of workload {wid} ({frames} of its frames, "
                  f"{ref_plan.num_blocks} blocks of {w.t_blk}), once: plan and output allocation {c1 - c0:.3f} s, "
                  f"pack {c2 - c1:.3f} s, reduce {c3 - c2:.3f} s",
        "host_cores_visible": os.cpu_count(),
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=4, choices=[1, 2, 3, 4, 5],
                    help="the workload of the headline (value, config, roofline)")
    ap.add_argument("--only", action="store_true",
                    help="time the headline workload only (no per_workload sweep, no cache-cold runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-scan", action="store_true", help="leave out bload_segment_scan")
    ap.add_argument("--plan", choices=["next-fit", "random-fit"], default="next-fit",
                    help="block builder: next-fit over the seeded order (default, parallel) or the "
                         "paper's sampler, uniform among the remaining sequences that fit "
                         "(bload_plan_random_fit, a sequential chain of draws)")
    ap.add_argument("--world", type=int, default=1,
                    help="time the share of one data-parallel worker (blocks rank mod world, "
                         "bload_plan_shard) instead of the whole workload; still one GPU")
    ap.add_argument("--rank", type=int, default=0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain elementwise copy of 1 GiB (read 1 GiB, write 1 GiB) "
                         "three times before the steps, as the known-size kernel that the "
                         "rocprofv3 HBM counters are scaled by")
    ap.add_argument("--yardsticks-only", action="store_true",
                    help="time nothing but the yardstick kernels (torch copy and fill, and the streaming "
                         "kernels of libbload_yardsticks.so) and print their figures as one JSON line")
    args = ap.parse_args()
    if args.yardsticks_only:
        print(json.dumps({"yardsticks": yardsticks()}))
        return 0
    if args.gpus != 1:
        print("bench.py measures one GPU: the packer runs on a single MI355X and the library has "
              "no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    head = run_workload(args, args.workload)
    result = {
        "metric": "packed_frames_per_s",
        "value": head["frames_per_s"],
        "unit": "frames/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": head["dtype"],
        "data": "synthetic",
        "config": {k: head[k] for k in ("workload", "n_seq", "t_blk", "frame_bytes", "total_frames",
                                        "num_blocks", "lengths")},
        "phases_ms": head["phases_ms"],
        "plan_ns_per_sequence": head["plan_ns_per_sequence"],
        "pack": head["pack"],
        "segment_reduce": head["segment_reduce"],
        "padding": head["padding"],
        "roofline": {k: v for k, v in head["pack"].items() if k not in ("frames_per_s", "min_ms", "median_ms")},
    }
    for k in ("segment_scan", "strategy_counts"):
        if k in head:
            result[k] = head[k]

    if not args.only and args.world == 1:
        keep = ("workload", "ms_per_step", "frames_per_s", "phases_ms", "plan_ns_per_sequence", "pack",
                "segment_reduce", "segment_scan", "padding", "setup_s")
        per = {}
        for wid in (1, 2, 3, 4, 5):
            r = head if wid == args.workload else run_workload(args, wid)
            per[str(wid)] = {k: r[k] for k in keep if k in r}
        # workloads whose traffic fits or nearly fits the last-level cache: the same steps over
        # rotating buffer sets, enough of them that a set has left every cache before its turn
        # comes again
        for wid in (1, 3):
            one = per[str(wid)]
            set_bytes = one["pack"]["algorithmic_bytes_per_launch"]
            sets = int(min(160, max(4, -(-4 * LAST_LEVEL_CACHE_BYTES // set_bytes))))
            cold_args = argparse.Namespace(**vars(args))
            cold_args.steps = max(args.steps, sets)
            cold_args.no_scan = True
            r = run_workload(cold_args, wid, cold_sets=sets)
            one["cache_cold"] = {"buffer_sets": sets, "steps": cold_args.steps, "ms_per_step": r["ms_per_step"],
                                 "phases_ms": r["phases_ms"], "pack_frac": r["pack"]["frac"],
                                 "segment_reduce_frac": r["segment_reduce"]["frac"]}
        result["per_workload"] = per

    if not args.only:
        result["yardsticks"] = yardsticks()
    if not args.no_cpu_baseline and args.world == 1:
        # the oracle on the whole workload, on the GPU machine's host: about 7 s of its time for workload 4
        # (25 GB of source and 34 GB of packed tensor in host memory meanwhile)
        result["cpu_baseline"] = cpu_baseline(args, args.workload, 1 << 40)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
