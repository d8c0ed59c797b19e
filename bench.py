#!/usr/bin/env python3
"""Benchmark of the Slow Momentum hot path on one MI355X.

A "step" is one outer iteration (round) of Algorithm 1 over the whole tensor
list: tau local steps on all m workers plus the outer step.  All inputs
(replicas, state, tau pre-generated gradient sets) are resident in HBM before
the timed region starts; gradients stand in for the backward pass and are not
regenerated inside it.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet50]
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

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak
LIB = os.path.join(ROOT, "paper_1910_00643_amd", "libslowmo.so")
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")


def mangled(kernel: str) -> str:
    """The symbol-name fragment of a kernel given as rocprofv3 prints it, e.g.
    'k_local_step<0, false, true>' -> '12k_local_stepILi0ELb0ELb1EEE' (integer
    and bool template arguments only, which is all the library's kernels have)."""
    name, _, rest = kernel.partition("<")
    args = [a.strip() for a in rest.rstrip(">").split(",")] if rest else []
    enc = "".join("Lb1E" if a == "true" else "Lb0E" if a == "false" else f"Li{int(a)}E"
                  for a in args)
    return f"{len(name)}{name}" + (f"I{enc}E" if args else "")


def measured_traffic(workload: str, variant: str):
    """HBM bytes per launch of the variant's dominant kernel from the rocprofv3
    --pmc runs recorded in profiles/traffic.json (written together with the
    profile summaries by slowmo_inputs/profile_summary.py), or None: nothing
    recorded, or the library no longer contains the kernel it was measured for
    (the number would be stale)."""
    try:
        entries = json.load(open(TRAFFIC_FILE))["entries"]
        lib = open(LIB, "rb").read()
    except (OSError, ValueError, KeyError):
        return None
    for e in entries:
        if e["workload"] == workload and e["variant"] == variant:
            return e["bytes_per_launch"] if mangled(e["kernel"]).encode() in lib else None
    return None


def local_bytes_per_update(w, first: bool, last: bool = False) -> int:
    """Algorithmic HBM bytes of one base-optimizer update of one (worker,
    element): x, h (and v) read and written, the gradient read; the first step
    after a reset does not read the buffers, the last step before a reset does
    not write them."""
    g = 2 if w.grad_dtype == "bf16" else 4
    nbuf = 2 if w.base == "adam" else 1
    reads = 4 + (0 if first else 4 * nbuf) + g
    writes = 4 + (0 if last else 4 * nbuf)
    return reads + writes


def outer_bytes_per_element(w) -> int:
    if not w.exact_average:     # per worker: x, x0, u read and written
        return 24 * w.m
    b = 8 * w.m + 16            # m replicas + x0 + u read, the same written
    if w.policy == "average":   # + every worker's h (and v) read and written
        b += 8 * w.m * (2 if w.base == "adam" else 1)
    return b


def fused_bytes_per_element(w) -> int:
    """Last local step + outer step in one kernel: per worker x, h (and v), g
    read and x written; x0, u read and written; the buffers written once per
    worker unless the policy discards them."""
    g = 2 if w.grad_dtype == "bf16" else 4
    nbuf = 2 if w.base == "adam" else 1
    first = w.policy == "reset" and w.tau == 1
    reads = w.m * (4 + (0 if first else 4 * nbuf) + g) + 8
    writes = 4 * w.m + 8 + (0 if w.policy == "reset" else 4 * nbuf * w.m)
    return reads + writes


BIG_TILE = 65536                # elements of a big tile (kBigTile of the library)


def big_elements(w, fused: bool) -> int:
    """Elements that the big-tile kernels take in the outer step (fused with
    the last local step or not): the whole 65 536-element pieces of every
    tensor, from 8 workers on for the fused kernel and from 16 for the plain
    outer step, if there are at least 160 such pieces; the fused kernel only
    under the "reset" buffer strategy, the plain one unless the buffers are
    averaged (the library's rule; every tensor of the benchmark is 16-byte
    aligned)."""
    if not w.exact_average or w.policy == "average" or w.m < (8 if fused else 16):
        return 0
    if fused and w.policy != "reset":
        return 0
    tiles = sum(n // BIG_TILE for n in w.numel)
    return tiles * BIG_TILE if tiles >= 160 else 0


def fusable(w) -> bool:
    return w.exact_average and w.mix == "none"


def round_bytes(w, fused: bool = False, fused_mix: bool = False) -> int:
    """Algorithmic HBM bytes of one outer iteration as it is executed."""
    reset = w.policy == "reset"
    steps = range(w.tau - 1) if fused else range(w.tau)
    # the fused local+gossip kernel always stores the buffers
    per_worker_elem = sum(local_bytes_per_update(w, reset and k == 0,
                                                 reset and k == w.tau - 1 and not fused_mix)
                          for k in steps)
    if w.mix != "none" and not fused_mix:   # every replica read and written once per gossip step
        per_worker_elem += 8 * w.tau
    tail = fused_bytes_per_element(w) if fused else outer_bytes_per_element(w)
    return w.d * (w.m * per_worker_elem + tail)


PARAM_LAYOUT = "separate"       # --param-layout


def build_problem(w, ring):
    import torch
    from slowmo_inputs.gpu_problem import GpuProblem
    from paper_1910_00643_amd.optimizer import SlowMo, make_config
    # parameters: one allocation per tensor and worker; gradients: every tensor
    # 512-byte aligned, as separately allocated .grad tensors would be
    prob = GpuProblem(w, "cuda:0", ring=ring, grad_layout="padded", param_layout=PARAM_LAYOUT)
    cfg = make_config(m=w.m, tau=w.tau, alpha=w.alpha, beta=w.beta, base=w.base,
                      policy=w.policy, grad_dtype=w.grad_dtype, momentum=w.momentum,
                      weight_decay=w.weight_decay, beta1=w.beta1, beta2=w.beta2, eps=w.eps,
                      no_average=not w.exact_average)
    opt = SlowMo(prob.params, cfg)
    for s in range(ring):
        prob.fill_grads(s, s)
    torch.cuda.synchronize()
    return prob, opt


def _bracket(events, kind):
    """Context manager: HIP events on torch's current stream -- the stream the
    library's kernels are launched on -- around one library call."""
    import contextlib
    import torch

    @contextlib.contextmanager
    def cm():
        if events is None:
            yield
            return
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        yield
        b.record()
        events[kind].append((a, b))
    return cm()


def run_rounds(w, opt, arrays, rounds, events=None, marks=None, fused=False, fused_mix=False,
               z=None):
    """`rounds` outer iterations.  With `events`, brackets every call with HIP
    events; with `marks`, records one event at the start of every outer
    iteration and one after the last (per-iteration durations without any
    synchronization inside the timed region).  With `z` (a pointer array of
    destination tensors) the de-biased parameters are written after every gossip
    step, as a gradient evaluation at z would need them."""
    import torch
    import paper_1910_00643_amd as P
    ring = len(arrays)
    peers = None
    if w.mix == "expgraph":
        peers = [P.slowmo_expgraph_in_peers(w.m, s) for s in range(16)]
    elif w.mix == "random":     # any in-neighbour map: the general (push-sum) kernel
        from slowmo_inputs.workloads import in_peers
        peers = [in_peers(w, s).tolist() for s in range(16)]
    reset = w.policy == "reset"

    def mark():
        if marks is not None:
            e = torch.cuda.Event(enable_timing=True)
            e.record()
            marks.append(e)

    for _ in range(rounds):
        mark()
        for k in range(w.tau):
            if fused and k == w.tau - 1:        # last local step + outer step, one call
                with _bracket(events, "fused_last_outer"):
                    opt.local_outer_step(arrays[k % ring], w.lr)
                break
            if peers is not None and fused_mix:     # local step + gossip step, one call
                with _bracket(events, "local_mix_first" if (reset and k == 0) else "local_mix"):
                    opt.local_mix_step(arrays[k % ring], w.lr, peers[k % len(peers)])
                if z is not None:
                    with _bracket(events, "debias"):
                        opt.debias(z)
                continue
            kind = ("local_first" if (reset and k == 0) else
                    "local_last" if (reset and k == w.tau - 1) else "local")
            with _bracket(events, kind):
                opt.local_step(arrays[k % ring], w.lr)
            if peers is not None:           # SGP as base optimizer: gossip after every step
                with _bracket(events, "mix"):
                    opt.mix_step(peers[k % len(peers)])
                if z is not None:
                    with _bracket(events, "debias"):
                        opt.debias(z)
        else:
            with _bracket(events, "outer"):
                opt.outer_step(w.lr)
    mark()


def time_workload(w, steps, warmup, ring=None, fused=False, fused_mix=False, kernel_rounds=None,
                  debias=False):
    """Returns (wall seconds of the `steps` timed outer iterations, their
    individual durations in ms from HIP events, average ms per call kind from a
    second pass of `kernel_rounds` iterations with events around every call)."""
    import torch
    ring = ring or w.tau
    prob, opt = build_problem(w, ring)
    arrays = [opt.grad_pointer_array(prob.grads[s]) for s in range(ring)]
    z = None
    if debias:
        zt = [[torch.empty_like(t) for t in p] for p in prob.params]
        z = opt.param_pointer_array(zt)
    run_rounds(w, opt, arrays, warmup, fused=fused, fused_mix=fused_mix, z=z)
    torch.cuda.synchronize()
    marks = []
    t0 = time.perf_counter()
    run_rounds(w, opt, arrays, steps, marks=marks, fused=fused, fused_mix=fused_mix, z=z)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    round_ms = [a.elapsed_time(b) for a, b in zip(marks[:-1], marks[1:])]
    # second pass: per-kernel durations from HIP events around every launch
    events = {"local": [], "local_first": [], "local_last": [], "outer": [], "mix": [],
              "fused_last_outer": [], "local_mix": [], "local_mix_first": [], "debias": []}
    run_rounds(w, opt, arrays, kernel_rounds or steps, events, fused=fused, fused_mix=fused_mix,
               z=z)
    torch.cuda.synchronize()
    kern_ms = {k: (sum(a.elapsed_time(b) for a, b in v) / len(v) if v else None)
               for k, v in events.items()}
    opt.close()
    del prob, opt
    torch.cuda.empty_cache()
    return wall, round_ms, kern_ms


def graph_replay(w, steps, warmup):
    """The launch-bound case: one whole outer iteration (tau-1 local steps and
    the fused last step, all on one gradient set) captured into a HIP graph and
    replayed.  With unchanged gradient pointers the library only launches
    kernels, and for the SGD base with the reset policy every outer iteration
    is the same sequence of launches with the same arguments, so a replay is one
    more outer iteration.  Returns ms per replayed iteration (median, min) --
    a launch-overhead figure, not a bandwidth claim."""
    import torch
    assert w.base == "sgd_nesterov" and w.policy == "reset" and fusable(w)
    prob, opt = build_problem(w, 1)
    arr = opt.grad_pointer_array(prob.grads[0])

    def one_round():
        for _ in range(w.tau - 1):
            opt.local_step(arr, w.lr)
        opt.local_outer_step(arr, w.lr)

    one_round()                                 # eager: uploads the pointer table
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    cap = torch.cuda.Stream()
    cap.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=cap):
        one_round()
    torch.cuda.synchronize()
    for _ in range(warmup):
        graph.replay()
    torch.cuda.synchronize()
    marks = []
    for _ in range(steps + 1):
        e = torch.cuda.Event(enable_timing=True)
        e.record()
        marks.append(e)
        graph.replay()
    torch.cuda.synchronize()
    ms = [a.elapsed_time(b) for a, b in zip(marks[:-1], marks[1:])]
    opt.close()
    del prob, opt, graph
    torch.cuda.empty_cache()
    return {"median": _median(ms), "min": min(ms), "n": len(ms),
            "what": "ms per outer iteration replayed from a HIP graph (tau kernel launches)"}


def _median(v):
    v = sorted(v)
    n = len(v)
    return None if not n else v[n // 2] if n % 2 else 0.5 * (v[n // 2 - 1] + v[n // 2])


def variant_name(w) -> str:
    """Key of a workload variant in profiles/traffic.json."""
    if w.mix != "none":
        return "mix_" + w.mix
    if not w.exact_average:
        return "no_average"
    return "default" if w.policy in ("reset", "maintain") else "policy_" + w.policy


def describe(w) -> str:
    return (f"{w.name}-shaped tensor list ({len(w.numel)} tensors, d={w.d}), m={w.m}, tau={w.tau}, "
            f"base={w.base}, grads={w.grad_dtype}, policy={w.policy}, alpha={w.alpha}, "
            f"beta={w.beta}" + ("" if w.exact_average else ", no exact average")
            + ("" if w.mix == "none" else f", gossip={w.mix}"))


def measure(w, steps, warmup, ring, unfused=False, kernel_rounds=None, debias=False):
    """One workload variant: throughput over `steps` outer iterations (one
    timed region, synchronized on both sides), the spread of the individual
    iterations, and the roofline of every kernel kind that ran."""
    fused = fusable(w) and not unfused
    fused_mix = w.mix != "none" and not unfused
    wall, round_ms, kern_ms = time_workload(w, steps, warmup, ring, fused=fused,
                                            fused_mix=fused_mix, kernel_rounds=kernel_rounds,
                                            debias=debias)
    rb = round_bytes(w, fused, fused_mix) + (8 * w.m * w.d * w.tau if debias else 0)
    reset = w.policy == "reset"
    per_launch = {          # algorithmic HBM bytes of one call of each kind
        "local": local_bytes_per_update(w, False) * w.m * w.d,
        "local_first": local_bytes_per_update(w, True) * w.m * w.d,
        "local_last": local_bytes_per_update(w, reset and w.tau == 1, True) * w.m * w.d,
        # the fused local+gossip kernel moves the local step's bytes (gossip adds none)
        "local_mix": local_bytes_per_update(w, False) * w.m * w.d,
        "local_mix_first": local_bytes_per_update(w, True) * w.m * w.d,
        "mix": 8 * w.m * w.d,
        "outer": outer_bytes_per_element(w) * w.d,
        "fused_last_outer": fused_bytes_per_element(w) * w.d,
        "debias": 8 * w.m * w.d,
    }
    names = {"local": "k_local_step (steady state)", "local_first": "k_local_step (buffers read as zero)",
             "local_last": "k_local_step (buffers not stored)",
             "local_mix": "k_local_mix_step (steady state; all launches of one step)",
             "local_mix_first": "k_local_mix_step (buffers read as zero)",
             "mix": "k_mix_step (all launches of one step)",
             "outer": "k_outer_noavg" if not w.exact_average else
                      "k_outer_big + k_outer_step (whole 65 536-element pieces + rest)"
                      if big_elements(w, False) else "k_outer_step",
             "fused_last_outer": "k_local_outer_big + k_local_outer_step (whole 65 536-element "
                                 "pieces + rest)" if big_elements(w, True) else "k_local_outer_step",
             "debias": "k_debias"}
    kernels = {}
    for kind, ms in kern_ms.items():
        if ms:
            gbps = per_launch[kind] / (ms * 1e-3) / 1e9
            kernels[kind] = {"kernel": names[kind], "ms": ms, "achieved": gbps, "unit": "GB/s",
                             "frac": gbps / HBM_PEAK_GBPS,
                             "algorithmic_bytes_per_launch": per_launch[kind]}
    # the kernel kind the round spends most of its time in
    calls = {"local": w.tau - (2 if reset else 0) - (1 if fused and not reset else 0),
             "local_mix": w.tau - (1 if reset else 0)}
    dominant = "local_mix" if "local_mix" in kernels else "local" if "local" in kernels else \
        max(kernels, key=lambda k: kernels[k]["ms"] * calls.get(k, 1))
    dom = kernels[dominant]
    med = _median(round_ms)
    return {
        "workload": describe(w),
        "value": w.updates_per_round * steps / wall, "unit": "updates/s", "steps": steps,
        "ms_per_step": 1e3 * wall / steps,
        "round_ms": {"median": med, "min": min(round_ms), "max": max(round_ms), "n": len(round_ms),
                     "how": "HIP events at the start of every outer iteration inside the one "
                            "timed region (no synchronization between them)"},
        "value_at_median_round": w.updates_per_round / (med * 1e-3),
        "hbm_gbps_whole_round": rb / wall * steps / 1e9,
        "hbm_frac_whole_round": rb / wall * steps / 1e9 / HBM_PEAK_GBPS,
        "algorithmic_bytes_per_round": rb,
        "fused_calls": {"last_local_plus_outer": fused, "local_plus_gossip": fused_mix},
        "roofline": {"bound": "hbm", "kernel": dom["kernel"], "achieved": dom["achieved"],
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": dom["frac"],
                     "algorithmic_bytes_per_launch": dom["algorithmic_bytes_per_launch"],
                     "traffic": measured_traffic(w.name, variant_name(w))},
        "kernels": kernels,
        "gradient_sets_resident": ring,
    }


def cpu_baseline(w, budget_s=12.0):
    """The fp32 build of the CPU oracle, as it stands, timed on this host's
    cores over whole outer iterations of a contiguous slice of the workload
    (about budget_s seconds of oracle time; gradient generation not timed)."""
    import numpy as np
    import torch
    from oracle import slowmo_oracle as O
    from slowmo_inputs import device, generator as G
    lib = O.load("f32")
    cores = int(lib.oracle_num_threads())
    bf16 = w.grad_dtype == "bf16"
    # slice: the first n elements of the flat range, all m workers; n bounded
    # so that the oracle's state (x, h[, v], g per worker) stays near 2 GiB
    n = int(min(w.d, (2 << 30) // (16 * w.m)))
    idx = np.arange(n, dtype=np.int64)
    o = O.SlowMoOracle(G.initial_params(w.seed, idx), m=w.m, tau=w.tau, alpha=w.f32("alpha"),
                       beta=w.f32("beta"), base=w.base, policy=w.policy,
                       momentum=w.f32("momentum"), weight_decay=w.f32("weight_decay"),
                       beta1=w.f32("beta1"), beta2=w.f32("beta2"), eps=w.f32("eps"), prec="f32",
                       exact_average=w.exact_average)
    g_dev = torch.empty((w.m, n), dtype=torch.bfloat16 if bf16 else torch.float32, device="cuda:0")
    sets = []                                   # four gradient sets, used in turn (not timed)
    for s in range(4):
        device.fill(g_dev if w.m > 1 else g_dev[0], 0, w.seed, 0, s, w.sigma, n_workers=w.m)
        sets.append(g_dev.to(torch.float32).cpu().numpy())
    del g_dev
    spent, rounds, step = 0.0, 0, 0
    while spent < budget_s and rounds < 200:
        t0 = time.perf_counter()
        for k in range(w.tau):
            o.local_step(sets[step % 4], w.f32("lr"))
            if w.mix == "expgraph":
                o.mix_step(O.exponential_graph_in_peers(w.m, step))
            elif w.mix == "random":
                from slowmo_inputs.workloads import in_peers
                o.mix_step(in_peers(w, step))
            step += 1
        o.outer_step(w.f32("lr"))
        spent += time.perf_counter() - t0
        rounds += 1
    return {"value": w.m * n * w.tau * rounds / spent, "unit": "updates/s", "cores": cores,
            "kind": "oracle",
            "sample": f"fp32 build of the oracle (gcc -O2, OpenMP over elements, {cores} threads), "
                      f"{rounds} outer iterations (tau={w.tau} local steps + outer step each) of "
                      f"the first {n} elements of the flat range on all m={w.m} workers, "
                      f"{spent:.1f} s of oracle time"}


def default_ring(w) -> int:
    return min(w.tau, 16 if w.name == "transformer_big" else w.tau, 2 if w.name == "stress" else w.tau)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="resnet50",
                    choices=["tiny", "resnet18", "resnet50", "transformer_big", "stress"])
    ap.add_argument("--ring", type=int, default=0, help="gradient sets kept in HBM (default tau)")
    ap.add_argument("--policy", default=None, choices=["reset", "maintain", "average"],
                    help="override the workload's buffer strategy")
    ap.add_argument("--mix", default=None, choices=["expgraph", "random"],
                    help="stochastic gradient push as base: a gossip step on the one-peer "
                         "exponential graph after every local step")
    ap.add_argument("--no-average", action="store_true",
                    help="the variant without the exact average (Section 6 of the paper)")
    ap.add_argument("--unfused", action="store_true",
                    help="end every outer iteration with slowmo_local_step + slowmo_outer_step "
                         "instead of the single call slowmo_local_outer_step (same results)")
    ap.add_argument("--debias", action="store_true",
                    help="with --mix: also write the de-biased parameters z = x / w after every "
                         "gossip step (slowmo_debias)")
    ap.add_argument("--param-layout", default="separate", choices=["separate", "arena"],
                    help="separate (the benchmark's layout): every parameter tensor of every "
                         "worker is its own allocation; arena: one allocation for all workers, "
                         "tensors 512-byte aligned (reported in addition, never instead)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the short runs of the other workloads and variants (reported "
                         "under 'other_workloads')")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB copy kernel three times (a kernel of known "
                         "traffic for scaling rocprofv3 counters)")
    ap.add_argument("--ladder", action="store_true",
                    help="instead of the benchmark: the microbenchmark ladder of access shapes "
                         "(slowmo_inputs/ladder.py), m and floats per stream from --ladder-m/-n")
    ap.add_argument("--placement", action="store_true",
                    help="instead of the benchmark: three launches of the stream microbenchmark on "
                         "40 buffers allocated one after the other (how much the place of the "
                         "operands in memory matters)")
    ap.add_argument("--ladder-m", type=int, default=32)
    ap.add_argument("--ladder-n", type=int, default=25_559_040)
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (m logical workers share it); "
                 "--gpus N with N > 1 is not supported and no multi-GPU figure is reported")
    import dataclasses

    import torch
    from slowmo_inputs import workloads as W
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    if args.placement:
        from slowmo_inputs import ladder
        ladder.placement(args.ladder_m, args.ladder_n)
        return
    if args.ladder:
        from slowmo_inputs import ladder
        ladder.main(args.ladder_m, args.ladder_n)
        return
    global PARAM_LAYOUT
    PARAM_LAYOUT = args.param_layout
    w = W.BY_NAME[args.workload]()
    if args.policy:
        w = dataclasses.replace(w, policy=args.policy)
    if args.no_average:
        w = dataclasses.replace(w, exact_average=False)
    if args.mix:
        w = dataclasses.replace(w, mix=args.mix)
    if args.calibrate_copy:
        from slowmo_inputs import device
        a = torch.zeros(1 << 28, dtype=torch.float32, device="cuda:0")      # 1 GiB
        b = torch.empty_like(a)
        for _ in range(3):
            device.calib_copy(a, b)
        torch.cuda.synchronize()
        del a, b
        torch.cuda.empty_cache()
    res = measure(w, args.steps, args.warmup, args.ring or default_ring(w), unfused=args.unfused,
                  debias=args.debias and w.mix != "none")
    out = {
        "metric": "param-element updates/s (m*d*tau per round)",
        "value": res["value"], "unit": "updates/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": res["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": res["workload"],
                   "step": "one outer iteration: tau local steps on all m workers + outer step"
                           + (" (the last local step and the outer step as one fused call)"
                              if res["fused_calls"]["last_local_plus_outer"] else "")
                           + (" (every local step and the gossip step after it as one fused call)"
                              if res["fused_calls"]["local_plus_gossip"] else ""),
                   "gradient_sets_resident": res["gradient_sets_resident"]},
    }
    for key in ("round_ms", "value_at_median_round", "hbm_gbps_whole_round", "hbm_frac_whole_round",
                "algorithmic_bytes_per_round", "roofline", "kernels"):
        out[key] = res[key]
    if (not args.no_others and args.workload == "resnet50" and not args.policy
            and not args.no_average and not args.mix and not args.unfused):
        # Short runs of the other configurations and of the variants beyond the
        # base path, so that every figure quoted for them is measured here.
        r50 = W.resnet50()
        others = [(W.transformer_big(), 3, 1, 2), (W.tiny(), 10, 2, None), (W.resnet18(), 5, 1, None),
                  (W.stress(), 3, 1, 1),
                  (dataclasses.replace(r50, policy="average"), 3, 1, 2),
                  (dataclasses.replace(r50, exact_average=False), 3, 1, 2),
                  (dataclasses.replace(r50, mix="expgraph"), 3, 1, 2),
                  (dataclasses.replace(r50, mix="random"), 3, 1, 2),
                  (dataclasses.replace(W.transformer_big(), mix="expgraph"), 2, 1, 1)]
        out["other_workloads"] = []
        for w2, steps2, warm2, krounds in others:
            r2 = measure(w2, steps2, warm2, default_ring(w2), kernel_rounds=krounds)
            r2["variant"] = variant_name(w2)
            if w2.name == "tiny":       # launch-bound: also as a captured graph
                r2["hip_graph_replay_ms"] = graph_replay(w2, 50, 5)
            if w2.name == "transformer_big" and w2.mix == "none" and not args.no_cpu_baseline:
                r2["cpu_baseline"] = cpu_baseline(w2, budget_s=10.0)
            out["other_workloads"].append(r2)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
