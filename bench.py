#!/usr/bin/env python3
"""Benchmark of the synchronizer hot path on one MI355X.

A "step" is one sync of the whole workload: per fragment, quorum weights from the token
counters and the mask, compaction of the contributing learners, and the fused merge + outer
Nesterov step over every tensor of the fragment (ddl_plan_merge on a resident plan; the
streaming workload issues one call per arriving fragment, in its seeded arrival order).
All inputs are resident in HBM before the timed region starts.

Prints ONE JSON line: merged params/s (``value``), the HBM roofline of the merge kernel
(``roofline``) and the fp64 CPU oracle timed on this machine's host cores (``cpu_baseline``).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload dense_block]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published peak

# HBM bytes per merge launch measured with rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE, each
# scaled by what the same counter reads for ddl_copy_probe of known size); the runs are
# summarised under profiles/.  None where no counter run exists for the workload.
MEASURED_TRAFFIC_BYTES = {
    "dense_block": 1107103355,   # profiles/ddl_merge_kernel_dense_block.txt
    "large_dense": 27240647788,  # profiles/ddl_merge_kernel_large_workloads.txt
}
# The same for one sync with the RDA merge through the plan, one norm per row.
MEASURED_TRAFFIC_BYTES_Q4_BLOCK128 = {
    "dense_block": 899423517,    # profiles/ddl_q4_kernels.txt
}
MEASURED_TRAFFIC_BYTES_RDA_ROWS = {
    "dense_block": 1107403362,   # profiles/ddl_rda_kernels.txt
}

METRIC = "merged params/sec and achieved HBM GB/s (% of peak), merge+outer Nesterov"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="dense_block",
                    choices=["tiny", "dense_block", "large_dense", "moe", "moe_stacked",
                             "streaming_model", "small_fragments"])
    ap.add_argument("--syncs-per-call", type=int, default=1,
                    help="fragments handed to one ddl_plan_merge call (plan API, avg merge): "
                         "the library covers up to sixteen fragments with one launch")
    ap.add_argument("--api", default="plan", choices=["plan", "batch", "tensor"],
                    help="resident plan (default); the one-shot ddl_merge_batch per fragment; "
                         "or, for --merge rda, one ddl_rda_merge_fragment call per tensor")
    ap.add_argument("--replicas", type=int, default=None,
                    help="independent copies of the workload visited round-robin, one per step, "
                         "so that no step finds its data in the 256 MB last-level cache "
                         "(default: enough copies for a 3 GiB rotating footprint)")
    ap.add_argument("--balanced", type=int, default=0, metavar="P",
                    help="regroup the workload's tensors into P balanced fragments with "
                         "ddl_balanced_fragments (the paper uses P = 24)")
    ap.add_argument("--merge", default="avg", choices=["avg", "rda", "q4"],
                    help="avg: weighted direct averaging (the metric's path); rda: "
                         "radial-directional averaging; q4: merge of 4-bit block-wise outer "
                         "gradients (each fragment stored as one flat array)")
    ap.add_argument("--q4-block", type=int, default=128, help="elements per scale block (q4)")
    ap.add_argument("--rda-group", default="row", choices=["row", "tensor"],
                    help="one norm per row of the last dimension, or one per tensor")
    ap.add_argument("--bcast", action="store_true",
                    help="also write the new Theta as bf16 in the same pass (+2 B/param)")
    ap.add_argument("--tile-rotate", type=int, default=None)
    ap.add_argument("--streams", type=int, default=1,
                    help="issue the calls of a step round-robin on this many HIP streams "
                         "(fragments are independent; call i of every step uses stream i mod N)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time replays (plan API, avg merge)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tiles-per-block", type=int, default=None)
    ap.add_argument("--max-blocks-per-cu", type=int, default=None)
    ap.add_argument("--rda-blocks-per-cu", type=int, default=None)
    return ap.parse_args()


def time_copy_probe(ddl, torch, nbytes=1 << 30, reps=20):
    """GB/s (read + write bytes) of the plain streaming copy kernel."""
    src = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda:0").normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        ddl.copy_probe(dst, src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        ddl.copy_probe(dst, src)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    del src, dst
    return 2 * nbytes / (ms * 1e-3) / 1e9


def cpu_baseline(torch, ddl_synth, wl, data, budget_s=20.0, gpu_merge=None):
    """The oracle as it stands, timed on the host: the plain scalar fp64 loop on one core and
    the same loop chunked over all cores.  Sample: whole tensors of the workload, in order,
    until about ``budget_s`` seconds of single-core work have been spent.

    The oracle's results are not thrown away: if ``gpu_merge(fragment_index)`` is given, every
    fragment whose tensors were all run through the oracle is then synced once more on the GPU
    from that same state, and the two are compared on windows of every tensor (first, middle
    and last 4096 elements of what the oracle saw): ``max_abs_err_vs_oracle``."""
    import numpy as np
    import oracle
    cores = len(os.sched_getaffinity(0))
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)) or cores)
    done_params = 0
    t_single = 0.0
    t_multi = 0.0
    tensors = 0
    worst_err, worst_rel, checked = 0.0, 0.0, 0
    for fi in wl.arrival_order:
        f = wl.fragments[fi]
        kept = []                       # (segment, lo, hi, theta_ref, v_ref) of this fragment
        for s in data[fi]:
            n = s.theta.numel()
            cap = 1 << 26               # at most 64 Mi elements of a tensor: bounds host memory
            th = ddl_synth.to_host_array(s.theta[:cap])
            v = ddl_synth.to_host_array(s.v[:cap])
            ls = [ddl_synth.to_host_array(x[:cap]) if (x is not None and q and t > 0) else None
                  for x, q, t in zip(s.learners, f.quorum_mask, f.token_counts)]
            t0 = time.perf_counter()
            oracle.merge_fragment(th, v, ls, f.token_counts, f.quorum_mask, f.lr, f.mu)
            t1 = time.perf_counter()
            ref = oracle.merge_fragment(th, v, ls, f.token_counts, f.quorum_mask, f.lr, f.mu,
                                        nthreads=cores)
            t2 = time.perf_counter()
            t_single += t1 - t0
            t_multi += t2 - t1
            m = min(n, cap)
            done_params += m
            tensors += 1
            for lo in sorted({0, max(0, m // 2 - 2048), max(0, m - 4096)}):
                hi = min(m, lo + 4096)
                kept.append((s, lo, hi, ref[0][lo:hi].copy(), ref[1][lo:hi].copy()))
            del ref, th, v, ls
            if t_single >= budget_s:
                break
        whole_fragment = len({id(k[0]) for k in kept}) == len(data[fi])
        if gpu_merge is not None and whole_fragment and kept:
            gpu_merge(fi)
            torch.cuda.synchronize()
            for s, lo, hi, th_ref, v_ref in kept:
                for got, want in ((s.theta[lo:hi], th_ref), (s.v[lo:hi], v_ref)):
                    err = np.abs(got.cpu().numpy().astype(np.float64) - want)
                    worst_err = max(worst_err, float(err.max()))
                    worst_rel = max(worst_rel, float((err / (1.0 + np.abs(want))).max()))
                    checked += err.size
        if t_single >= budget_s:
            break
    model = ""
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {
        "value": done_params / t_multi,
        "unit": "params/s",
        "cores": cores,
        "cpu_model": model,
        "host_cpus": os.cpu_count(),
        "kind": "oracle",
        "sample": (f"{tensors} tensor(s), {done_params} params of workload {wl.name} "
                   f"(of {wl.numel}); same fp64 scalar loop chunked over {cores} threads"),
        "value_1core": done_params / t_single,
        "seconds_1core": round(t_single, 3),
        "seconds_allcores": round(t_multi, 3),
        # one more sync of the same state on the GPU against the oracle's result just timed
        "max_abs_err_vs_oracle": worst_err if checked else None,
        "max_err_over_bound": (worst_rel / 1e-6) if checked else None,   # bound 1e-6 (1 + |ref|)
        "elements_compared": checked,
    }


def detail_pass(torch, launch_lists, counter, replicas, reps, extra_bytes_per_step):
    """After the timed region: ``reps`` more steps with a HIP event before every launch, for
    the spread over steps (median, best) and, for workloads of several fragments, the time
    and rate of each fragment (median over the repetitions).  The extra events put small
    gaps between launches, so these figures are a little below the headline ones."""
    import statistics
    per_step, per_launch = [], {}
    for _ in range(reps):
        ll = launch_lists[counter[0] % replicas]
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(len(ll) + 1)]
        for (_, _, fn), ev in zip(ll, evs):
            ev.record()
            fn()
        evs[-1].record()
        counter[0] += 1
        torch.cuda.synchronize()
        per_step.append(evs[0].elapsed_time(evs[-1]))
        for k, (fi, nb, _) in enumerate(ll):
            per_launch.setdefault((k, fi, nb), []).append(evs[k].elapsed_time(evs[k + 1]))
    step_bytes = sum(nb for _, nb, _ in launch_lists[0]) + extra_bytes_per_step
    med, best = statistics.median(per_step), min(per_step)
    out = {
        "steps": reps,
        "gpu_ms_per_step_median": med,
        "gpu_ms_per_step_best": best,
        "gbps_median": step_bytes / (med * 1e-3) / 1e9,
        "gbps_best": step_bytes / (best * 1e-3) / 1e9,
    }
    if 1 < len(launch_lists[0]) <= 64 and extra_bytes_per_step == 0:
        out["per_launch"] = [
            {"order": k, "fragment": fi, "ms": round(statistics.median(ts), 5),
             "gbps": round(nb / (statistics.median(ts) * 1e-3) / 1e9, 1)}
            for (k, fi, nb), ts in sorted(per_launch.items())]
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        sys.stderr.write(
            "bench.py: this build is single-GPU by design (the synchronizer path is element-wise "
            "and has no collectives here); run with --gpus 1.\n")
        sys.exit(2)

    import torch

    import ddl_synth
    import paper_2604_21428_amd as ddl

    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible; the HIP path has no CPU fallback.\n")
        sys.exit(3)
    torch.cuda.set_device(0)
    if args.tiles_per_block is not None:
        ddl.set_option("tiles_per_block", args.tiles_per_block)
    if args.tile_rotate is not None:
        ddl.set_option("tile_rotate", args.tile_rotate)
    if args.max_blocks_per_cu is not None:
        ddl.set_option("max_blocks_per_cu", args.max_blocks_per_cu)
    if args.rda_blocks_per_cu is not None:
        ddl.set_option("rda_blocks_per_cu", args.rda_blocks_per_cu)

    wl = ddl_synth.WORKLOADS[args.workload]()
    if args.balanced:
        sizes = [t.numel for f in wl.fragments for t in f.tensors]
        wl = ddl_synth.regroup(wl, ddl.balanced_fragments(sizes, args.balanced), args.balanced)
    big = wl.numel > 2_000_000_000
    steps = args.steps if args.steps is not None else (20 if big else 300)
    warmup = args.warmup if args.warmup is not None else (2 if big else 20)

    # ---- inputs, resident in HBM ----------------------------------------------------------
    # Every step syncs ONE copy of the workload.  Small workloads are replicated and the
    # copies visited round-robin: a real syncer touches a fragment once every H steps, so its
    # data never sits in the last-level cache, and a loop over one 0.8 GB copy would.
    footprint = sum(f.numel * ((2 if f.learner_dtype == "bf16" else 4) * f.M + 8)
                    for f in wl.fragments)
    replicas = args.replicas if args.replicas is not None else max(
        1, min(8, -(-3 * (1 << 30) // footprint)))
    dt = {"bf16": torch.bfloat16, "f32": torch.float32}
    copies = []
    for r in range(replicas):
        data = [ddl_synth.make_fragment(wl, f, "cuda:0", absent="valid") for f in wl.fragments]
        for segs in data:
            for s in segs:
                s.bcast = (torch.empty(s.theta.numel(), dtype=torch.bfloat16, device="cuda:0")
                           if args.bcast else None)
        if args.merge == "q4":
            # Each fragment as ONE flat array (its tensors back to back); the learners' outer
            # gradients are encoded once, outside the timed region, as a learner would send them.
            calls = []
            for fi in wl.arrival_order:
                f = wl.fragments[fi]
                theta = torch.cat([s.theta for s in data[fi]])
                v = torch.cat([s.v for s in data[fi]])
                codes, scales = [], []
                for m in range(f.M):
                    if not (f.quorum_mask[m] and f.token_counts[m] > 0):
                        codes.append(None)
                        scales.append(None)
                        continue
                    c, sc = ddl.q4_encode(theta, torch.cat([s.learners[m] for s in data[fi]]),
                                          args.q4_block)
                    codes.append(c)
                    scales.append(sc)
                calls.append((f, theta, v, codes, scales))
                data[fi] = None
            torch.cuda.synchronize()
            torch.cuda.empty_cache()
            copies.append((data, "q4", calls))
        elif args.merge == "rda" and args.api == "plan":
            plan = ddl.Plan([ddl.Fragment([(s.theta, s.v, s.learners, s.bcast) for s in segs], M=f.M,
                                          learner_dtype=dt[f.learner_dtype])
                             for f, segs in zip(wl.fragments, data)])
            plan.set_rda_groups([t.shape[-1] if args.rda_group == "row" else 0
                                 for f in wl.fragments for t in f.tensors])
            ws = torch.empty(max(256, plan.rda_workspace_bytes), dtype=torch.uint8,
                             device="cuda:0")
            calls = [plan.prepare([(fi, wl.fragments[fi].token_counts,
                                    wl.fragments[fi].quorum_mask, wl.fragments[fi].lr,
                                    wl.fragments[fi].mu)]) for fi in wl.arrival_order]
            copies.append((data, ("rda-plan", plan, ws), calls))
        elif args.merge == "rda":
            calls = []
            for fi in wl.arrival_order:
                f = wl.fragments[fi]
                for s, t in zip(data[fi], f.tensors):
                    g = t.shape[-1] if args.rda_group == "row" else t.numel
                    ws = torch.empty(ddl.rda_workspace_bytes(t.numel, g, f.M), dtype=torch.uint8,
                                     device="cuda:0")
                    calls.append((s, f, g, ws))
            copies.append((data, "rda", calls))
        elif args.api == "plan":
            plan = ddl.Plan([ddl.Fragment([(s.theta, s.v, s.learners, s.bcast) for s in segs], M=f.M,
                                          learner_dtype=dt[f.learner_dtype])
                             for f, segs in zip(wl.fragments, data)])
            k = max(1, args.syncs_per_call)
            groups = [wl.arrival_order[i:i + k] for i in range(0, len(wl.arrival_order), k)]
            calls = [plan.prepare([(fi, wl.fragments[fi].token_counts,
                                    wl.fragments[fi].quorum_mask, wl.fragments[fi].lr,
                                    wl.fragments[fi].mu) for fi in grp]) for grp in groups]
            copies.append((data, plan, calls))
        else:
            frs = [ddl.Fragment([(s.theta, s.v, s.learners, s.bcast) for s in segs], f.token_counts,
                                f.quorum_mask, f.lr, f.mu, M=f.M,
                                learner_dtype=dt[f.learner_dtype])
                   for f, segs in zip(wl.fragments, data)]
            copies.append((data, None, frs))
    data = copies[0][0]
    counter = [0]

    def launch_list(copy):
        """One step over one copy as a list of (fragment index, bytes, callable)."""
        _, plan, calls = copy
        out = []
        if isinstance(plan, tuple):
            _, rplan, ws = plan
            for fi, c in zip(wl.arrival_order, calls):
                out.append((fi, wl.fragments[fi].numel * wl.fragments[fi].bytes_per_param,
                            lambda c=c, rplan=rplan, ws=ws: rplan.rda_merge(c, ws)))
        elif plan == "q4":
            for f, theta, v, codes, scales in calls:
                nb = theta.numel() * 16 + sum(c.numel() + 4 * sc.numel()
                                              for c, sc in zip(codes, scales) if c is not None)
                out.append((f.index, nb, lambda f=f, theta=theta, v=v, codes=codes, scales=scales:
                            ddl.q4_merge_fragment(theta, v, codes, scales, f.token_counts,
                                                  f.quorum_mask, args.q4_block, f.lr, f.mu)))
        elif plan == "rda":
            for s, f, g, ws in calls:
                nb = s.theta.numel() * f.bytes_per_param
                out.append((f.index, nb, lambda s=s, f=f, g=g, ws=ws: ddl.rda_merge_fragment(
                    s.theta, s.v, s.learners, f.token_counts, f.quorum_mask, g, f.lr, f.mu, ws)))
        elif plan is not None:
            k = max(1, args.syncs_per_call)
            groups = [wl.arrival_order[i:i + k] for i in range(0, len(wl.arrival_order), k)]
            for grp, c in zip(groups, calls):
                out.append((grp[0], sum(wl.fragments[fi].numel * wl.fragments[fi].bytes_per_param
                                        for fi in grp), lambda c=c, plan=plan: plan.merge(c)))
        else:
            for fi in wl.arrival_order:
                out.append((fi, wl.fragments[fi].numel * wl.fragments[fi].bytes_per_param,
                            lambda fr=calls[fi]: ddl.merge_batch([fr])))
        return out

    launch_lists = [launch_list(c) for c in copies]

    streams = [torch.cuda.Stream() for _ in range(args.streams)] if args.streams > 1 else None

    def step():
        if streams is None:
            for _, _, fn in launch_lists[counter[0] % replicas]:
                fn()
        else:
            for i, (_, _, fn) in enumerate(launch_lists[counter[0] % replicas]):
                with torch.cuda.stream(streams[i % len(streams)]):
                    fn()
        counter[0] += 1

    def fork():     # the side streams start after what the main stream has done so far
        if streams is not None:
            for st in streams:
                st.wait_stream(torch.cuda.current_stream())

    def join():     # ... and the main stream continues after all of them
        if streams is not None:
            for st in streams:
                torch.cuda.current_stream().wait_stream(st)

    if args.graph:
        if args.api != "plan" or args.merge != "avg":
            sys.stderr.write("bench.py: --graph needs the plan API and the avg merge\n")
            sys.exit(2)
        eager_step = step
        graphs = []
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(replicas):
                eager_step()                    # warm-up outside capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        for _ in range(replicas):               # one graph per replica, in visiting order
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                eager_step()
            graphs.append(g)
        gcount = [0]

        def step():
            graphs[gcount[0] % replicas].replay()
            gcount[0] += 1

    if args.merge == "q4" and (args.bcast or args.balanced or args.api != "plan"):
        sys.stderr.write("bench.py: --merge q4 takes none of --bcast, --balanced, --api\n")
        sys.exit(2)
    if args.merge == "rda" and args.api == "batch":
        sys.stderr.write("bench.py: --merge rda goes with --api plan or --api tensor\n")
        sys.exit(2)
    if args.merge == "avg" and args.api == "tensor":
        sys.stderr.write("bench.py: --api tensor is for --merge rda\n")
        sys.exit(2)
    launches_per_step = wl.num_segments if args.api == "tensor" else len(launch_lists[0])
    torch.cuda.synchronize()

    # ---- timed region ---------------------------------------------------------------------
    fork()
    for _ in range(warmup):
        step()
    join()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()          # on torch's current stream: the stream the kernels are launched on
    fork()
    for _ in range(steps):
        step()
    join()
    ev1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall_ms = (t1 - t0) * 1e3 / steps
    gpu_ms = ev0.elapsed_time(ev1) / steps

    detail = None if args.graph or streams is not None else detail_pass(torch, launch_lists, counter, replicas,
                                                 min(steps, 40), 2 * wl.numel if args.bcast else 0)

    params_per_s = wl.numel / (wall_ms * 1e-3)
    if args.merge == "q4":
        alg_bytes = sum(nb for _, nb, _ in launch_lists[0])
    else:
        alg_bytes = wl.algorithmic_bytes + (2 * wl.numel if args.bcast else 0)
    # The step consists of merge-kernel launches only (no copies, no other kernels), so the
    # event time per step divided by the launches per step is the average launch duration,
    # gaps between back-to-back launches included.
    kernel_ms = gpu_ms / launches_per_step
    achieved = alg_bytes / launches_per_step / (kernel_ms * 1e-3) / 1e9
    copy_gbps = time_copy_probe(ddl, torch)
    if args.bcast or args.balanced:
        traffic = None
    elif args.merge == "avg":
        traffic = MEASURED_TRAFFIC_BYTES.get(wl.name)
    elif args.merge == "q4" and args.q4_block == 128:
        traffic = MEASURED_TRAFFIC_BYTES_Q4_BLOCK128.get(wl.name)
    elif args.merge == "rda" and args.api == "plan" and args.rda_group == "row":
        traffic = MEASURED_TRAFFIC_BYTES_RDA_ROWS.get(wl.name)
    else:
        traffic = None

    out = {
        "metric": METRIC,
        "value": params_per_s,
        "unit": "params/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": wall_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": wl.name,
            "params": wl.numel,
            "tensors": wl.num_segments,
            "fragments": len(wl.fragments),
            "M": wl.fragments[0].M,
            "Mq": sorted({f.Mq for f in wl.fragments}),
            "learner_dtype": wl.fragments[0].learner_dtype,
            "state_dtype": "f32",
            "lr": wl.fragments[0].lr,
            "mu": wl.fragments[0].mu,
            "api": ("ddl_q4_merge_fragment" if args.merge == "q4" else
                    "ddl_rda_merge_fragment" if args.api == "tensor" else
                    "ddl_plan_rda_merge" if args.merge == "rda" else
                    "ddl_plan_merge" if args.api == "plan" else "ddl_merge_batch"),
            "merge": (args.merge if args.merge == "avg" else
                      f"q4/block{args.q4_block}" if args.merge == "q4" else
                      f"rda/{args.rda_group}"),
            "launches_per_step": launches_per_step,
            "syncs_per_call": args.syncs_per_call,
            "streams": args.streams,
            "replicas": replicas,
            "bf16_broadcast_copy": bool(args.bcast),
            "hip_graph": bool(args.graph),
            "tiles_per_block": ddl.get_option("tiles_per_block"),
            "tile_rotate": ddl.get_option("tile_rotate"),
            "max_blocks_per_cu": ddl.get_option("max_blocks_per_cu"),
        },
        "achieved_gbps": alg_bytes / (wall_ms * 1e-3) / 1e9,
        "algorithmic_bytes_per_step": alg_bytes,
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS,
            "traffic": traffic,
            "kernel": ("ddl_merge_kernel" if args.merge == "avg" else
                       "q4_merge_kernel" if args.merge == "q4" else
                       "rda kernel(s) of one tensor" if args.api == "tensor" else
                       "rda kernel(s) of one fragment"),
            "avg_launch_ms": kernel_ms,
            "algorithmic_bytes_per_launch": alg_bytes / launches_per_step,
            "copy_probe_gbps": copy_gbps,
            "frac_of_copy_probe": achieved / copy_gbps,
        },
    }
    if detail is not None:
        out["detail"] = detail
    if not args.no_cpu_baseline and args.merge != "q4":   # the oracle leg times the bf16 path
        gpu_merge = None
        if (args.api == "plan" and args.merge == "avg" and args.syncs_per_call == 1 and
                not args.graph and streams is None):
            fns = {fi: fn for fi, _, fn in launch_lists[0]}
            gpu_merge = lambda fi: fns[fi]()
        out["cpu_baseline"] = cpu_baseline(torch, ddl_synth, wl, data, gpu_merge=gpu_merge)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
