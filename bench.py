#!/usr/bin/env python3
"""Benchmark of the synchronizer hot path on one MI355X.

A "step" is one sync of the whole workload: per fragment, quorum weights from the token
counters and the mask, compaction of the contributing learners, and the fused merge + outer
Nesterov step over every tensor of the fragment (ddl_plan_merge on a resident plan; the
streaming workload issues one call per arriving fragment, in its seeded arrival order).
All inputs are resident in HBM before the timed region starts.

The default workload is the largest single-GPU one, ``streaming_model`` (8.3 B parameters in
33 fragments, 166 GB resident).  Before it, the default run also measures the three one-fragment
workloads of at least 50 M parameters (``dense_block``, ``large_dense``, ``moe``) the same way
and reports them under ``per_config``.

Parity rides along: before anything is timed, fragments are synced once from their fresh state
and EVERY element of the new Theta and v is compared with the fp64 CPU oracle (all fragments of
the per-config workloads; for the streaming model whole fragments, in arrival order after the
embedding and one fragment of each quorum size, under a time budget).  That oracle run is also
the ``cpu_baseline``.

Prints ONE JSON line: merged params/s (``value``), the HBM roofline of the merge kernel
(``roofline``), the oracle timed on this machine's host cores (``cpu_baseline``) and ``per_config``.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload streaming_model]
"""
from __future__ import annotations

import argparse
import json
import math
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published peak
METRIC = "merged params/sec and achieved HBM GB/s (% of peak), merge+outer Nesterov"
DEFAULT_WORKLOAD = "streaming_model"
PER_CONFIG = ("dense_block", "large_dense", "moe")
PARITY_CHUNK = 1 << 26          # elements copied to the host and run through the oracle at a time
TOL = 1e-6                      # parity bar: |err| <= TOL (1 + |oracle|), Theta and v alike


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD,
                    choices=["tiny", "dense_block", "large_dense", "moe", "moe_stacked",
                             "streaming_model", "small_fragments"])
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the per_config measurements of dense_block, large_dense and moe "
                         "(they are taken only in the default configuration anyway)")
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
    ap.add_argument("--merge", default="avg", choices=["avg", "rda", "q4", "q4rda"],
                    help="avg: weighted direct averaging (the metric's path); rda: "
                         "radial-directional averaging; q4: merge of 4-bit block-wise outer "
                         "gradients")
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
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="skip the oracle: no cpu_baseline, no parity figures")
    ap.add_argument("--parity-budget", type=float, default=45.0,
                    help="seconds of wall time the oracle/parity leg of the main workload may "
                         "take before it stops adding fragments (whole fragments only)")
    ap.add_argument("--tiles-per-block", type=int, default=None)
    ap.add_argument("--max-blocks-per-cu", type=int, default=None)
    ap.add_argument("--rda-blocks-per-cu", type=int, default=None)
    ap.add_argument("--max-tiles-per-launch", type=int, default=None)
    ap.add_argument("--part-megabytes", type=int, default=None)
    return ap.parse_args()


# ------------------------------------------------------------------------------------------
# HBM traffic from the committed counter runs
# ------------------------------------------------------------------------------------------
def profiled_traffic(ddl, workload, merge, default_shape):
    """(HBM bytes of one step or None, source string).  The figure comes from a line
    ``TRAFFIC workload=<w> merge=<m> bytes_per_step=<int> build_id=<id>`` of a summary under
    profiles/ (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of this script, each scaled by the
    same counter's reading for ddl_copy_probe, summed over the kernel launches of a step).  It is reported only if it was taken on the
    very kernel sources the loaded library was built from (ddl_kernel_build_id) and in the
    default launch shape; otherwise
    the value is null and the source string says why."""
    if not default_shape:
        return None, "not reported: launch-shape options differ from the profiled defaults"
    here = ddl.kernel_build_id("rda" if merge.startswith(("rda", "q4rda")) else
                               "q4" if merge.startswith("q4") else "merge")
    stale = None
    pdir = os.path.join(ROOT, "profiles")
    for name in sorted(os.listdir(pdir)) if os.path.isdir(pdir) else []:
        if not name.endswith((".txt", ".md")):
            continue
        with open(os.path.join(pdir, name)) as fh:
            for line in fh:
                if not line.startswith("TRAFFIC "):
                    continue
                kv = dict(re.findall(r"(\w+)=(\S+)", line))
                if kv.get("workload") != workload or kv.get("merge") != merge:
                    continue
                if kv.get("build_id") == here:
                    return int(kv["bytes_per_step"]), f"profiles/{name} (build {here})"
                stale = (f"profiles/{name} holds a figure taken on build {kv.get('build_id')}; "
                         f"this library is build {here}: not reported")
    return None, stale or "no counter run for this workload under profiles/"


# ------------------------------------------------------------------------------------------
# set-up of one workload: resident inputs, plans, the list of calls of a step
# ------------------------------------------------------------------------------------------
class Setup:
    pass


def merge_label(args):
    """How the merge of this run is named in the JSON line and in the profile summaries."""
    if args.merge == "avg":
        return "avg"
    if args.merge == "q4":
        return f"q4/block{args.q4_block}"
    if args.merge == "q4rda":
        return f"q4rda/block{args.q4_block}/{args.rda_group}"
    return f"rda/{args.rda_group}"


def build_setup(args, wl, ddl, ddl_synth, torch, replicas=None):
    """Generates ``replicas`` copies of the workload in HBM and marshals the calls of a step."""
    su = Setup()
    su.wl = wl
    footprint = sum(f.numel * ((2 if f.learner_dtype == "bf16" else 4) * f.M + 8)
                    for f in wl.fragments)
    # Every step syncs ONE copy of the workload.  Small workloads are replicated and the
    # copies visited round-robin: a real syncer touches a fragment once every H steps, so its
    # data never sits in the last-level cache, and a loop over one 0.8 GB copy would.
    if replicas is None:
        replicas = max(1, min(8, -(-3 * (1 << 30) // footprint)))
    su.replicas = replicas
    dt = {"bf16": torch.bfloat16, "f32": torch.float32}
    rda_groups = None
    if args.merge in ("rda", "q4rda"):
        rda_groups = [[t.shape[-1] if args.rda_group == "row" else t.numel for t in f.tensors]
                      for f in wl.fragments]
    su.rda_groups = rda_groups
    copies = []
    for _ in range(replicas):
        data = [ddl_synth.make_fragment(wl, f, "cuda:0", absent="valid") for f in wl.fragments]
        for segs in data:
            for s in segs:
                s.bcast = (torch.empty(s.theta.numel(), dtype=torch.bfloat16, device="cuda:0")
                           if args.bcast else None)
        if args.merge in ("q4", "q4rda"):
            # The learners' outer gradients are encoded once, tensor by tensor, outside the
            # timed region, as a learner would send them; the parameter copies are then dropped
            # (the 4-bit merge reads codes and scales only).
            sources = []
            for f, segs in zip(wl.fragments, data):
                for s in segs:
                    codes, scales = [], []
                    for m in range(f.M):
                        if f.quorum_mask[m] and f.token_counts[m] > 0:
                            c, sc = ddl.q4_encode(s.theta, s.learners[m], args.q4_block)
                        else:
                            c, sc = None, None
                        codes.append(c)
                        scales.append(sc)
                    s.learners = [None] * f.M
                    s.q4 = (codes, scales)
                    sources.append((codes, scales))
            torch.cuda.synchronize()
            torch.cuda.empty_cache()
            plan = ddl.Plan([ddl.Fragment([(s.theta, s.v, s.learners, s.bcast) for s in segs],
                                          M=f.M, learner_dtype=dt[f.learner_dtype])
                             for f, segs in zip(wl.fragments, data)])
            plan.set_q4_sources(sources, args.q4_block)
            ws = None
            if args.merge == "q4rda":     # RDA as the merge of the 4-bit outer gradients
                plan.set_rda_groups([g for gs in rda_groups for g in gs])
                ws = torch.empty(max(256, plan.rda_workspace_bytes), dtype=torch.uint8,
                                 device="cuda:0")
            calls = [plan.prepare([(fi, wl.fragments[fi].token_counts,
                                    wl.fragments[fi].quorum_mask, wl.fragments[fi].lr,
                                    wl.fragments[fi].mu)]) for fi in wl.arrival_order]
            copies.append((data, ("q4-plan", plan, ws), calls))
        elif args.merge == "rda" and args.api == "plan":
            plan = ddl.Plan([ddl.Fragment([(s.theta, s.v, s.learners, s.bcast) for s in segs],
                                          M=f.M, learner_dtype=dt[f.learner_dtype])
                             for f, segs in zip(wl.fragments, data)])
            plan.set_rda_groups([g for gs in rda_groups for g in gs])
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
                for s, t, g in zip(data[fi], f.tensors, rda_groups[fi]):
                    ws = torch.empty(ddl.rda_workspace_bytes(t.numel, g, f.M), dtype=torch.uint8,
                                     device="cuda:0")
                    calls.append((s, f, g, ws))
            copies.append((data, "rda", calls))
        elif args.api == "plan":
            plan = ddl.Plan([ddl.Fragment([(s.theta, s.v, s.learners, s.bcast) for s in segs],
                                          M=f.M, learner_dtype=dt[f.learner_dtype])
                             for f, segs in zip(wl.fragments, data)])
            k = max(1, args.syncs_per_call)
            groups = [wl.arrival_order[i:i + k] for i in range(0, len(wl.arrival_order), k)]
            calls = [plan.prepare([(fi, wl.fragments[fi].token_counts,
                                    wl.fragments[fi].quorum_mask, wl.fragments[fi].lr,
                                    wl.fragments[fi].mu) for fi in grp]) for grp in groups]
            copies.append((data, plan, calls))
        else:
            frs = [ddl.Fragment([(s.theta, s.v, s.learners, s.bcast) for s in segs],
                                f.token_counts, f.quorum_mask, f.lr, f.mu, M=f.M,
                                learner_dtype=dt[f.learner_dtype])
                   for f, segs in zip(wl.fragments, data)]
            copies.append((data, None, frs))
    su.copies = copies

    def launch_list(copy):
        """One step over one copy as a list of (fragment index, bytes, callable)."""
        _, plan, calls = copy
        out = []
        if isinstance(plan, tuple) and plan[0] == "q4-plan":
            _, qplan, qws = plan
            for fi, c in zip(wl.arrival_order, calls):
                nb = sum(s.theta.numel() * (16 + (2 if s.bcast is not None else 0)) +
                         sum(cc.numel() + 4 * sc.numel()
                             for cc, sc in zip(*s.q4) if cc is not None)
                         for s in copy[0][fi])
                if qws is None:
                    out.append((fi, nb, lambda c=c, qplan=qplan: qplan.q4_merge(c)))
                else:
                    out.append((fi, nb, lambda c=c, qplan=qplan, qws=qws:
                                qplan.q4_rda_merge(c, qws)))
        elif isinstance(plan, tuple):
            _, rplan, ws = plan
            for fi, c in zip(wl.arrival_order, calls):
                out.append((fi, wl.fragments[fi].numel * wl.fragments[fi].bytes_per_param,
                            lambda c=c, rplan=rplan, ws=ws: rplan.rda_merge(c, ws)))
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

    su.launch_lists = [launch_list(c) for c in copies]
    su.launches_per_step = (wl.num_segments if args.api == "tensor" else len(su.launch_lists[0]))
    if args.merge in ("q4", "q4rda"):   # codes and scales as stored; the bf16 copy is counted too
        su.alg_bytes = sum(nb for _, nb, _ in su.launch_lists[0])
    else:
        su.alg_bytes = wl.algorithmic_bytes + (2 * wl.numel if args.bcast else 0)
    su.counter = [0]
    return su


def free_setup(su, torch):
    for _, plan, _ in su.copies:
        p = plan[1] if isinstance(plan, tuple) else plan
        if hasattr(p, "destroy"):
            p.destroy()
    su.copies = su.launch_lists = None
    torch.cuda.synchronize()
    torch.cuda.empty_cache()


# ------------------------------------------------------------------------------------------
# oracle leg: parity over every element of whole fragments, and the CPU baseline
# ------------------------------------------------------------------------------------------
def host_cores():
    cores = len(os.sched_getaffinity(0))
    return max(1, min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)) or cores))


def parity_supported(args):
    return (args.merge in ("avg", "rda", "q4", "q4rda") and args.api in ("plan", "batch") and
            args.syncs_per_call == 1 and not (args.merge == "rda" and args.api == "batch"))


def oracle_leg(args, su, torch, ddl_synth, budget_s, single_core_s, must_cover=()):
    """Syncs fragments of copy 0 once from their fresh state, through the very calls the timed
    region uses, and compares every element of the new Theta and v with the fp64 oracle run on
    host copies of the same inputs.  Fragments are taken whole: first those in ``must_cover``,
    then the rest in arrival order until ``budget_s`` seconds of wall time are spent.  The
    oracle's own time (its plain scalar loop chunked over all host cores, and for the first
    ``single_core_s`` seconds of work the same loop on one core) is the CPU baseline."""
    import numpy as np
    import oracle
    wl = su.wl
    data = su.copies[0][0]
    fns = {fi: fn for fi, _, fn in su.launch_lists[0]}
    cores = host_cores()
    order = list(must_cover) + [fi for fi in wl.arrival_order if fi not in must_cover]
    t_multi = t_single = 0.0
    n_multi = n_single = 0
    worst_abs = worst_rel = 0.0
    compared = 0
    covered = []
    t_start = time.perf_counter()
    for k, fi in enumerate(order):
        if k >= len(must_cover) and time.perf_counter() - t_start > budget_s:
            break
        f = wl.fragments[fi]
        segs = data[fi]
        before = [(s.theta.clone(), s.v.clone()) for s in segs]   # device copies, freed below
        fns[fi]()
        torch.cuda.synchronize()
        present = [bool(q) and t > 0 for q, t in zip(f.quorum_mask, f.token_counts)]
        for si, (s, (th0, v0)) in enumerate(zip(segs, before)):
            n = th0.numel()
            g = (su.rda_groups[fi][si] if su.rda_groups else
                 args.q4_block if args.merge == "q4" else 1)   # chunks end on these boundaries
            if args.merge == "q4rda" and g < n:                # ... of groups and scale blocks
                g = g * args.q4_block // math.gcd(g, args.q4_block)
            # chunks end on group boundaries; a group longer than a chunk is taken whole
            chunk = max(g, PARITY_CHUNK // g * g) if g > 1 else PARITY_CHUNK
            for lo in range(0, n, chunk):
                hi = min(n, lo + chunk)
                th = ddl_synth.to_host_array(th0[lo:hi])
                vv = ddl_synth.to_host_array(v0[lo:hi])
                ls = [ddl_synth.to_host_array(x[lo:hi]) if (p and x is not None) else None
                      for x, p in zip(s.learners, present)]
                if args.merge in ("q4", "q4rda"):
                    B = args.q4_block
                    cs = [c[lo // 2:(hi + 1) // 2].cpu().numpy() if c is not None else None
                          for c in s.q4[0]]
                    ss = [x[lo // B:-(-hi // B)].cpu().numpy() if x is not None else None
                          for x in s.q4[1]]
                    t0 = time.perf_counter()
                    ref = oracle.q4_merge_fragment(
                        th, vv, cs, ss, f.token_counts, f.quorum_mask, B, f.lr, f.mu,
                        rda_group_len=(min(su.rda_groups[fi][si], hi - lo)
                                       if args.merge == "q4rda" else 0))
                    t_single += time.perf_counter() - t0
                    n_single += hi - lo
                elif args.merge == "rda":
                    t0 = time.perf_counter()
                    ref = oracle.rda_merge_fragment(th, vv, ls, f.token_counts, f.quorum_mask,
                                                    min(g, hi - lo), f.lr, f.mu)
                    t_single += time.perf_counter() - t0
                    n_single += hi - lo
                else:
                    if t_single < single_core_s:
                        t0 = time.perf_counter()
                        oracle.merge_fragment(th, vv, ls, f.token_counts, f.quorum_mask, f.lr,
                                              f.mu)
                        t_single += time.perf_counter() - t0
                        n_single += hi - lo
                    t0 = time.perf_counter()
                    ref = oracle.merge_fragment(th, vv, ls, f.token_counts, f.quorum_mask, f.lr,
                                                f.mu, nthreads=cores)
                    t_multi += time.perf_counter() - t0
                    n_multi += hi - lo
                # The comparison itself (fp64 subtract, abs, max) runs on the GPU: plumbing.
                for got, want in ((s.theta[lo:hi], ref[0]), (s.v[lo:hi], ref[1])):
                    w = torch.from_numpy(want).to("cuda:0")
                    err = (got.double() - w).abs_()
                    worst_abs = max(worst_abs, float(err.max()))
                    rel = float(err.div_(w.abs_().add_(1.0)).max())
                    worst_rel = rel if math.isnan(rel) else max(worst_rel, rel)
                    compared += hi - lo
                    del w, err
                del ref, th, vv, ls
        del before
        covered.append(fi)
    model = ""
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    done = sum(wl.fragments[fi].numel for fi in covered)
    multi = n_multi > 0
    out = {
        "value": (n_multi / t_multi) if multi else (n_single / t_single if n_single else None),
        "unit": "params/s",
        "cores": cores if multi else 1,
        "cpu_model": model,
        "host_cpus": os.cpu_count(),
        "kind": "oracle",
        "sample": (f"{len(covered)} whole fragment(s) of workload {wl.name} (fragment indices "
                   f"{covered}): {done} of {wl.numel} params; "
                   + (f"fp64 scalar loop chunked over {cores} threads" if multi else
                      "fp64 scalar loop on one core (this oracle function has no threaded form)")),
        "fragments_covered": covered,
        "params_covered": done,
        "value_1core": (n_single / t_single) if n_single else None,
        "seconds_1core": round(t_single, 3),
        "seconds_allcores": round(t_multi, 3),
        "seconds_wall": round(time.perf_counter() - t_start, 1),
        # every element of the new Theta and of the new v of the covered fragments
        "elements_compared": compared // 2,
        "max_abs_err_vs_oracle": worst_abs if compared else None,
        "max_err_over_bound": (worst_rel / TOL) if compared else None,
        "parity_ok": bool(compared and worst_rel <= TOL),
    }
    return out


# ------------------------------------------------------------------------------------------
# timing
# ------------------------------------------------------------------------------------------
def detail_pass(torch, su, reps, extra_bytes_per_step):
    """After the timed region: ``reps`` more steps with a HIP event before every launch, for
    the spread over steps (median, best) and, for workloads of several fragments, the time
    and rate of each fragment (median over the repetitions).  The extra events put small
    gaps between launches, so these figures are a little below the headline ones."""
    import statistics
    per_step, per_launch = [], {}
    for _ in range(reps):
        ll = su.launch_lists[su.counter[0] % su.replicas]
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(len(ll) + 1)]
        for (_, _, fn), ev in zip(ll, evs):
            ev.record()
            fn()
        evs[-1].record()
        su.counter[0] += 1
        torch.cuda.synchronize()
        per_step.append(evs[0].elapsed_time(evs[-1]))
        for k, (fi, nb, _) in enumerate(ll):
            per_launch.setdefault((k, fi, nb), []).append(evs[k].elapsed_time(evs[k + 1]))
    step_bytes = sum(nb for _, nb, _ in su.launch_lists[0]) + extra_bytes_per_step
    med, best = statistics.median(per_step), min(per_step)
    out = {
        "steps": reps,
        "gpu_ms_per_step_median": med,
        "gpu_ms_per_step_best": best,
        "gbps_median": step_bytes / (med * 1e-3) / 1e9,
        "gbps_best": step_bytes / (best * 1e-3) / 1e9,
    }
    if 1 < len(su.launch_lists[0]) <= 64 and extra_bytes_per_step == 0:
        out["per_launch"] = [
            {"order": k, "fragment": fi, "ms": round(statistics.median(ts), 5),
             "gbps": round(nb / (statistics.median(ts) * 1e-3) / 1e9, 1)}
            for (k, fi, nb), ts in sorted(per_launch.items())]
    return out


def timed_region(args, su, ddl, torch, steps, warmup):
    """W untimed steps, then exactly K steps between synchronisations.  Returns (wall ms per
    step, event ms per step, several streams?, kernel grids per step); the events are recorded
    on torch's current stream, which is the stream every call of a step is enqueued on."""
    streams = [torch.cuda.Stream() for _ in range(args.streams)] if args.streams > 1 else None

    def step():
        ll = su.launch_lists[su.counter[0] % su.replicas]
        if streams is None:
            for _, _, fn in ll:
                fn()
        else:
            for i, (_, _, fn) in enumerate(ll):
                with torch.cuda.stream(streams[i % len(streams)]):
                    fn()
        su.counter[0] += 1

    def fork():     # the side streams start after what the main stream has done so far
        if streams is not None:
            for st in streams:
                st.wait_stream(torch.cuda.current_stream())

    def join():     # ... and the main stream continues after all of them
        if streams is not None:
            for st in streams:
                torch.cuda.current_stream().wait_stream(st)

    # How many kernel grids a step enqueues (a long fragment goes out as several): counted by
    # the library, over one untimed eager step.
    g0 = ddl.get_option("grids_enqueued")
    step()
    grids_per_step = ddl.get_option("grids_enqueued") - g0

    if args.graph:
        eager_step = step
        graphs = []
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(su.replicas):
                eager_step()                    # warm-up outside capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        for _ in range(su.replicas):            # one graph per replica, in visiting order
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                eager_step()
            graphs.append(g)
        gcount = [0]

        def step():                             # noqa: F811 (replaces the eager step)
            graphs[gcount[0] % su.replicas].replay()
            gcount[0] += 1

    torch.cuda.synchronize()
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
    return ((t1 - t0) * 1e3 / steps, ev0.elapsed_time(ev1) / steps, streams is not None,
            grids_per_step)


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


def measure(args, name, ddl, ddl_synth, torch, steps, warmup, parity_budget, must_cover_fn=None,
            with_detail=False, default_shape=True):
    """Generate one workload, check it against the oracle from its fresh state, time it, free
    it.  Returns (summary dict, cpu/parity dict or None, detail or None)."""
    wl = ddl_synth.WORKLOADS[name]()
    if args.balanced:
        sizes = [t.numel for f in wl.fragments for t in f.tensors]
        wl = ddl_synth.regroup(wl, ddl.balanced_fragments(sizes, args.balanced), args.balanced)
    su = build_setup(args, wl, ddl, ddl_synth, torch, args.replicas)
    cpu = None
    if not args.no_cpu_baseline and parity_supported(args):
        must = must_cover_fn(wl) if must_cover_fn else ()
        cpu = oracle_leg(args, su, torch, ddl_synth, parity_budget,
                         single_core_s=5.0, must_cover=must)
    wall_ms, gpu_ms, multi_stream, grids = timed_region(args, su, ddl, torch, steps, warmup)
    detail = None
    if with_detail and not args.graph and not multi_stream:
        detail = detail_pass(torch, su, min(steps, 40),
                             2 * wl.numel if (args.bcast and not args.merge.startswith("q4")) else 0)
    # A step consists of merge-kernel grids only (no copies, no other kernels), so the event
    # time per step divided by the grids per step is the average duration of one kernel launch,
    # the gaps between back-to-back launches included.
    kernel_ms = gpu_ms / grids
    achieved = su.alg_bytes / grids / (kernel_ms * 1e-3) / 1e9
    merge_tag = merge_label(args)
    plain = default_shape and not (args.bcast or args.balanced or args.graph or multi_stream or
                                   args.api != "plan" or args.syncs_per_call != 1)
    traffic, traffic_source = profiled_traffic(ddl, wl.name, merge_tag, plain)
    if traffic is not None:
        traffic = round(traffic / grids)      # per launch, like `achieved`
    summary = {
        "workload": wl.name,
        "params": wl.numel,
        "tensors": wl.num_segments,
        "fragments": len(wl.fragments),
        "M": wl.fragments[0].M,
        "Mq": sorted({f.Mq for f in wl.fragments}),
        "steps": steps,
        "warmup": warmup,
        "replicas": su.replicas,
        "ms_per_step": wall_ms,
        "params_per_s": wl.numel / (wall_ms * 1e-3),
        "calls_per_step": su.launches_per_step,
        "launches_per_step": grids,
        "avg_launch_ms": kernel_ms,
        "algorithmic_bytes_per_step": su.alg_bytes,
        "achieved": achieved,
        "frac": achieved / HBM_PEAK_GBPS,
        "traffic": traffic,
        "traffic_source": traffic_source,
    }
    if cpu is not None:
        summary["elements_compared"] = cpu["elements_compared"]
        summary["max_err_over_bound"] = cpu["max_err_over_bound"]
        summary["parity_ok"] = cpu["parity_ok"]
    free_setup(su, torch)
    return summary, cpu, detail, wl


def main():
    args = parse_args()
    if args.gpus != 1:
        sys.stderr.write(
            "bench.py: this build is single-GPU by design (the synchronizer path is element-wise "
            "and has no collectives here); run with --gpus 1.\n")
        sys.exit(2)
    if args.merge in ("q4", "q4rda") and args.api != "plan":
        sys.stderr.write("bench.py: --merge q4 / q4rda go through the plan\n")
        sys.exit(2)
    if args.merge == "rda" and args.api == "batch":
        sys.stderr.write("bench.py: --merge rda goes with --api plan or --api tensor\n")
        sys.exit(2)
    if args.merge == "avg" and args.api == "tensor":
        sys.stderr.write("bench.py: --api tensor is for --merge rda\n")
        sys.exit(2)
    if args.graph and (args.api != "plan" or args.merge != "avg"):
        sys.stderr.write("bench.py: --graph needs the plan API and the avg merge\n")
        sys.exit(2)

    import torch

    import ddl_synth
    import paper_2604_21428_amd as ddl

    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible; the HIP path has no CPU fallback.\n")
        sys.exit(3)
    torch.cuda.set_device(0)
    default_shape = True
    for opt, val in (("tiles_per_block", args.tiles_per_block), ("tile_rotate", args.tile_rotate),
                     ("max_blocks_per_cu", args.max_blocks_per_cu),
                     ("rda_blocks_per_cu", args.rda_blocks_per_cu),
                     ("max_tiles_per_launch", args.max_tiles_per_launch),
                     ("part_megabytes", args.part_megabytes)):
        if val is not None:
            default_shape = default_shape and ddl.get_option(opt) == val
            ddl.set_option(opt, val)

    big = ddl_synth.WORKLOADS[args.workload]().numel > 2_000_000_000
    steps = args.steps if args.steps is not None else (20 if big else 300)
    warmup = args.warmup if args.warmup is not None else (2 if big else 20)

    # ---- the other configurations of at least 50 M parameters, measured the same way ------
    per_config = []
    plain_default = (args.workload == DEFAULT_WORKLOAD and args.merge == "avg" and
                     args.api == "plan" and not (args.no_per_config or args.balanced or
                                                 args.bcast or args.graph or args.streams > 1 or
                                                 args.syncs_per_call != 1))
    if plain_default:
        for name in PER_CONFIG:
            # at least 50 ms of timed work, so that a handful of slow launches cannot move it
            n_steps = {"dense_block": 400, "large_dense": 30, "moe": 30}[name]
            summary, _, _, _ = measure(args, name, ddl, ddl_synth, torch, n_steps,
                                       max(3, n_steps // 10), parity_budget=1e9,
                                       default_shape=default_shape)
            per_config.append(summary)

    # ---- the workload the headline figure is quoted on -------------------------------------
    def must_cover(wl):
        """Streaming model: the embedding and one fragment of each quorum size first."""
        if wl.name != "streaming_model":
            return ()
        out = [len(wl.fragments) - 1]
        for mq in sorted({f.Mq for f in wl.fragments}):
            cand = [fi for fi in wl.arrival_order if wl.fragments[fi].Mq == mq and fi not in out]
            if cand:
                out.append(cand[0])
        return tuple(out)

    budget = args.parity_budget if big else 1e9
    main_summary, cpu, detail, wl = measure(args, args.workload, ddl, ddl_synth, torch, steps,
                                            warmup, budget, must_cover_fn=must_cover,
                                            with_detail=True, default_shape=default_shape)
    copy_gbps = time_copy_probe(ddl, torch)

    out = {
        "metric": METRIC,
        "value": main_summary["params_per_s"],
        "unit": "params/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": main_summary["ms_per_step"],
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
            "api": ("ddl_plan_q4_merge" if args.merge == "q4" else
                    "ddl_plan_q4_rda_merge" if args.merge == "q4rda" else
                    "ddl_rda_merge_fragment" if args.api == "tensor" else
                    "ddl_plan_rda_merge" if args.merge == "rda" else
                    "ddl_plan_merge" if args.api == "plan" else "ddl_merge_batch"),
            "merge": merge_label(args),
            "calls_per_step": main_summary["calls_per_step"],
            "launches_per_step": main_summary["launches_per_step"],
            "syncs_per_call": args.syncs_per_call,
            "streams": args.streams,
            "replicas": main_summary["replicas"],
            "bf16_broadcast_copy": bool(args.bcast),
            "hip_graph": bool(args.graph),
            "tiles_per_block": ddl.get_option("tiles_per_block"),
            "tile_rotate": ddl.get_option("tile_rotate"),
            "max_blocks_per_cu": ddl.get_option("max_blocks_per_cu"),
            "library_build": ddl.build_id(),
            "kernel_build": ddl.kernel_build_id("rda" if args.merge in ("rda", "q4rda") else
                                                "q4" if args.merge == "q4" else "merge"),
        },
        "achieved_gbps": main_summary["algorithmic_bytes_per_step"] /
                         (main_summary["ms_per_step"] * 1e-3) / 1e9,
        "algorithmic_bytes_per_step": main_summary["algorithmic_bytes_per_step"],
        "roofline": {
            "bound": "hbm",
            "achieved": main_summary["achieved"],
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": main_summary["frac"],
            "traffic": main_summary["traffic"],
            "traffic_source": main_summary["traffic_source"],
            "kernel": ("ddl_merge_kernel" if args.merge == "avg" else
                       "ddl_merge_kernel on 4-bit codes" if args.merge == "q4" else
                       "rda kernel(s) of one tensor" if args.api == "tensor" else
                       "rda kernel(s) of one fragment"),
            "avg_launch_ms": main_summary["avg_launch_ms"],
            "algorithmic_bytes_per_launch": (main_summary["algorithmic_bytes_per_step"] /
                                             main_summary["launches_per_step"]),
            "copy_probe_gbps": copy_gbps,
            "frac_of_copy_probe": main_summary["achieved"] / copy_gbps,
        },
    }
    if cpu is not None:
        out["cpu_baseline"] = cpu
    if per_config:
        out["per_config"] = per_config
    if detail is not None:
        out["detail"] = detail
    print(json.dumps(out))
    bad = [s["workload"] for s in per_config + [main_summary] if s.get("parity_ok") is False]
    if bad:
        sys.stderr.write(f"bench.py: GPU result off the oracle on {bad}\n")
        sys.exit(4)


if __name__ == "__main__":
    main()
