#!/usr/bin/env python3
"""Diagnostic: how far the eight XCDs drift apart during one sync of a workload.

Runs one ddl_plan_merge of a one-fragment workload on the diagnostic build of the library
(``libddlsync_trace.so``, the same sources compiled with -DDDL_TRACE), in which every merge
workgroup records the 100 MHz wall clock at its start, the XCD it runs on and its tile.  From
those records it prints, at several points of the sync, how many workgroups each XCD has
started and how wide the range of tile indices started within the last 20 us is -- the window
of addresses in flight, which is what DRAM efficiency depends on.

    python paper_2604_21428_amd/trace_tiles.py --workload large_dense --max-tiles-per-launch 0
    python paper_2604_21428_amd/trace_tiles.py --workload large_dense          # library default

Run as a script (not with -m): it must choose the library before the package is imported.
"""
import argparse
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
TRACE_LIB = os.path.join(HERE, "libddlsync_trace.so")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="large_dense",
                    choices=["dense_block", "large_dense", "moe", "moe_stacked"])
    ap.add_argument("--max-tiles-per-launch", type=int, default=None,
                    help="0: the whole sync as one grid; default: the library's own choice")
    args = ap.parse_args()
    if not os.path.exists(TRACE_LIB):
        sys.exit(f"{TRACE_LIB} is missing: build it first (python paper_2604_21428_amd/build.py)")
    os.environ["DDLSYNC_LIBRARY"] = TRACE_LIB
    sys.path.insert(0, ROOT)
    import numpy as np
    import torch

    import ddl_synth
    import paper_2604_21428_amd as ddl

    dev = "cuda:0"
    wl = ddl_synth.WORKLOADS[args.workload]()
    f = wl.fragments[0]
    segs = ddl_synth.make_fragment(wl, f, dev)
    tiles = sum((s.theta.numel() + 1023) // 1024 for s in segs)
    plan = ddl.Plan([ddl.Fragment([(s.theta, s.v, s.learners) for s in segs], M=f.M,
                                  learner_dtype=torch.bfloat16)])
    call = plan.prepare([(0, f.token_counts, f.quorum_mask, f.lr, f.mu)])
    if args.max_tiles_per_launch is not None:
        ddl.set_option("max_tiles_per_launch", args.max_tiles_per_launch)
    trace = torch.zeros(2 * tiles, dtype=torch.int64, device=dev)   # one record per workgroup
    for _ in range(3):
        plan.merge(call)
    torch.cuda.synchronize()
    g0 = ddl.get_option("grids_enqueued")
    ddl.set_option("trace_buffer", trace.data_ptr())
    plan.merge(call)
    torch.cuda.synchronize()
    ddl.set_option("trace_buffer", 0)
    grids = ddl.get_option("grids_enqueued") - g0

    rec = trace.cpu().numpy().reshape(-1, 2)
    clk = rec[:, 0] - rec[:, 0].min()               # 10 ns ticks
    xcd = (rec[:, 1] >> 32) & 0xF
    tile = rec[:, 1] & 0xFFFFFFFF
    assert sorted(tile.tolist()) == list(range(tiles)), "every tile exactly once"
    span = int(clk.max())
    print(f"workload {wl.name}: {wl.numel:,} params, Mq={f.Mq}, {tiles} tiles in {grids} grid(s) "
          f"(max_tiles_per_launch {ddl.get_option('max_tiles_per_launch')}); first to last "
          f"workgroup start {span / 100:.0f} us; XCDs seen {sorted(set(xcd.tolist()))}")
    print("  at      workgroups started per XCD (min .. max, spread)   tile range started in the "
          "last 20 us")
    for frac in (0.10, 0.25, 0.50, 0.75, 0.90):
        cut = span * frac
        started = clk <= cut
        cnt = [int((started & (xcd == x)).sum()) for x in range(8)]
        recent = started & (clk > cut - 2000)
        rng = int(tile[recent].max() - tile[recent].min()) if recent.any() else 0
        print(f"  {frac:4.0%}   {min(cnt):7d} .. {max(cnt):7d}   spread {max(cnt) - min(cnt):5d}"
              f"            {int(recent.sum()):5d} tiles over an index range of {rng}")
    # How unevenly the XCDs reach the end of each grid: per grid, when each XCD started its last
    # workgroup; the gap between the first and the last XCD to get there is time the early ones
    # spend idle before the next grid may start.
    unit = 64                                       # parts are whole rotation groups
    part = -(-(-(-tiles // grids)) // unit) * unit if grids > 1 else tiles
    gaps = []
    for g in range(grids):
        sel = (tile >= g * part) & (tile < (g + 1) * part)
        last = [int(clk[sel & (xcd == x)].max()) for x in range(8) if (sel & (xcd == x)).any()]
        if len(last) == 8:
            gaps.append((max(last) - min(last)) / 100.0)
    if gaps:
        print(f"  last workgroup start per XCD, first to last XCD: mean {sum(gaps) / len(gaps):.1f} us, "
              f"max {max(gaps):.1f} us per grid ({len(gaps)} grids of about {span / 100 / grids:.0f} us)")
    plan.destroy()


if __name__ == "__main__":
    main()
