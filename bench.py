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

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc runs
# (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of known size); see
# profiles/.  None until measured for a workload.
MEASURED_TRAFFIC_BYTES = {
    "resnet50": 16407838272,            # profiles/resnet50_local_step_outer_step.md
    "transformer_big": 43766547359,     # profiles/transformer_big_local_step_outer_step.md
    # k_local_mix_step, per step (all its launches), profiles/resnet50_average_noaverage_mixing.md
    ("resnet50", "expgraph"): 16366373785,
    ("resnet50", "random"): 17971173213,
}


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


def build_problem(w, ring):
    import torch
    from slowmo_inputs.gpu_problem import GpuProblem
    from paper_1910_00643_amd.optimizer import SlowMo, make_config
    # parameters: one allocation per tensor and worker; gradients: every tensor
    # 512-byte aligned, as separately allocated .grad tensors would be
    prob = GpuProblem(w, "cuda:0", ring=ring, grad_layout="padded")
    cfg = make_config(m=w.m, tau=w.tau, alpha=w.alpha, beta=w.beta, base=w.base,
                      policy=w.policy, grad_dtype=w.grad_dtype, momentum=w.momentum,
                      weight_decay=w.weight_decay, beta1=w.beta1, beta2=w.beta2, eps=w.eps,
                      no_average=not w.exact_average)
    opt = SlowMo(prob.params, cfg)
    for s in range(ring):
        prob.fill_grads(s, s)
    torch.cuda.synchronize()
    return prob, opt


def run_rounds(w, opt, arrays, rounds, events=None, fused=False, fused_mix=False):
    """`rounds` outer iterations.  With `events`, brackets every call with HIP
    events on the stream the kernels are launched on (torch's current one)."""
    import torch
    import paper_1910_00643_amd as P
    ring = len(arrays)
    peers = None
    if w.mix == "expgraph":
        peers = [P.slowmo_expgraph_in_peers(w.m, s) for s in range(16)]
    elif w.mix == "random":     # any in-neighbour map: the general (push-sum) kernel
        from slowmo_inputs.workloads import in_peers
        peers = [in_peers(w, s).tolist() for s in range(16)]
    for _ in range(rounds):
        for k in range(w.tau):
            if fused and k == w.tau - 1:        # last local step + outer step, one call
                if events is not None:
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record()
                opt.local_outer_step(arrays[k % ring], w.lr)
                if events is not None:
                    b.record()
                    events["fused_last_outer"].append((a, b))
                break
            if peers is not None and fused_mix:     # local step + gossip step, one call
                if events is not None:
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record()
                opt.local_mix_step(arrays[k % ring], w.lr, peers[k % len(peers)])
                if events is not None:
                    b.record()
                    reset = w.policy == "reset"
                    events["local_mix_first" if (reset and k == 0) else "local_mix"].append((a, b))
                continue
            if events is not None:
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
            opt.local_step(arrays[k % ring], w.lr)
            if events is not None:
                b.record()
                reset = w.policy == "reset"
                kind = ("local_first" if (reset and k == 0) else
                        "local_last" if (reset and k == w.tau - 1) else "local")
                events[kind].append((a, b))
            if peers is not None:           # SGP as base optimizer: gossip after every step
                if events is not None:
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record()
                opt.mix_step(peers[k % len(peers)])
                if events is not None:
                    b.record()
                    events["mix"].append((a, b))
        else:
            if events is not None:
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
            opt.outer_step(w.lr)
            if events is not None:
                b.record()
                events["outer"].append((a, b))


def time_workload(w, steps, warmup, ring=None, fused=False, fused_mix=False):
    import torch
    ring = ring or w.tau
    prob, opt = build_problem(w, ring)
    arrays = [opt.grad_pointer_array(prob.grads[s]) for s in range(ring)]
    run_rounds(w, opt, arrays, warmup, fused=fused, fused_mix=fused_mix)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_rounds(w, opt, arrays, steps, fused=fused, fused_mix=fused_mix)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    # second pass: per-kernel durations from HIP events around every launch
    events = {"local": [], "local_first": [], "local_last": [], "outer": [], "mix": [],
              "fused_last_outer": [], "local_mix": [], "local_mix_first": []}
    run_rounds(w, opt, arrays, steps, events, fused=fused, fused_mix=fused_mix)
    torch.cuda.synchronize()
    kern_ms = {k: (sum(a.elapsed_time(b) for a, b in v) / len(v) if v else None)
               for k, v in events.items()}
    opt.close()
    del prob, opt
    torch.cuda.empty_cache()
    return wall, kern_ms


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
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the short extra run of the other target workload "
                         "(Transformer-big-shaped, reported under 'other_workloads')")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB copy kernel three times (a kernel of known "
                         "traffic for scaling rocprofv3 counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (m logical workers share it); "
                 "--gpus N with N > 1 is not supported and no multi-GPU figure is reported")
    import torch
    from slowmo_inputs import workloads as W
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    w = W.BY_NAME[args.workload]()
    import dataclasses
    if args.policy:
        w = dataclasses.replace(w, policy=args.policy)
    if args.no_average:
        w = dataclasses.replace(w, exact_average=False)
    if args.mix:
        w = dataclasses.replace(w, mix=args.mix)
    ring = args.ring or min(w.tau, 16 if w.name == "transformer_big" else w.tau,
                            2 if w.name == "stress" else w.tau)
    if args.calibrate_copy:
        from slowmo_inputs import device
        a = torch.zeros(1 << 28, dtype=torch.float32, device="cuda:0")      # 1 GiB
        b = torch.empty_like(a)
        for _ in range(3):
            device.calib_copy(a, b)
        torch.cuda.synchronize()
        del a, b
        torch.cuda.empty_cache()
    fused = fusable(w) and not args.unfused
    fused_mix = w.mix != "none" and not args.unfused
    wall, kern_ms = time_workload(w, args.steps, args.warmup, ring, fused=fused, fused_mix=fused_mix)
    ms_per_step = 1e3 * wall / args.steps
    value = w.updates_per_round * args.steps / wall
    local_bytes = local_bytes_per_update(w, False) * w.m * w.d
    # with gossip fused into the local step that kernel is the dominant one: same
    # algorithmic bytes as a local step (the gossip adds no traffic)
    dominant = "local_mix" if fused_mix and kern_ms.get("local_mix") else "local"
    achieved = local_bytes / (kern_ms[dominant] * 1e-3) / 1e9
    out = {
        "metric": "param-element updates/s (m*d*tau per round)",
        "value": value, "unit": "updates/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}-shaped tensor list ({len(w.numel)} tensors, d={w.d}), "
                               f"m={w.m}, tau={w.tau}, base={w.base}, grads={w.grad_dtype}, "
                               f"policy={w.policy}, alpha={w.alpha}, beta={w.beta}"
                               + ("" if w.exact_average else ", no exact average")
                               + ("" if w.mix == "none" else f", gossip={w.mix}"),
                   "step": "one outer iteration: tau local steps on all m workers + outer step"
                           + (" (the last local step and the outer step as one fused call)"
                              if fused else "")
                           + (" (every local step and the gossip step after it as one fused call)"
                              if fused_mix else ""),
                   "gradient_sets_resident": ring},
        "hbm_gbps_whole_round": round_bytes(w, fused, fused_mix) / wall * args.steps / 1e9,
        "hbm_frac_whole_round": round_bytes(w, fused, fused_mix) / wall * args.steps / 1e9
                                / HBM_PEAK_GBPS,
        "algorithmic_bytes_per_round": round_bytes(w, fused, fused_mix),
        "kernel_ms": kern_ms,
        "roofline": {"bound": "hbm", "kernel": ("k_local_mix_step (steady state)" if dominant == "local_mix"
                                                else "k_local_step (steady state)"),
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "algorithmic_bytes_per_launch": local_bytes,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(w.name if dominant == "local"
                                                           else (w.name, w.mix))},
    }
    if kern_ms.get("outer"):
        ob = outer_bytes_per_element(w) * w.d
        out["outer_kernel"] = {"achieved": ob / (kern_ms["outer"] * 1e-3) / 1e9, "unit": "GB/s",
                               "frac": ob / (kern_ms["outer"] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                               "algorithmic_bytes_per_launch": ob}
    if kern_ms.get("fused_last_outer"):
        fb = fused_bytes_per_element(w) * w.d
        ms = kern_ms["fused_last_outer"]
        out["fused_last_outer_kernel"] = {"achieved": fb / (ms * 1e-3) / 1e9, "unit": "GB/s",
                                          "frac": fb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                          "algorithmic_bytes_per_launch": fb}
    if kern_ms.get("mix"):
        mb = 8 * w.m * w.d
        out["mix_kernel"] = {"achieved": mb / (kern_ms["mix"] * 1e-3) / 1e9, "unit": "GB/s",
                             "frac": mb / (kern_ms["mix"] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                             "algorithmic_bytes_per_launch": mb}
    if (not args.no_others and args.workload == "resnet50" and not args.policy
            and not args.no_average and not args.mix):
        # the second workload the bandwidth target is stated for, three timed iterations
        w2 = W.transformer_big()
        f2 = fusable(w2) and not args.unfused
        wall2, k2 = time_workload(w2, 3, 1, 16, fused=f2)
        lb2 = local_bytes_per_update(w2, False) * w2.m * w2.d
        out["other_workloads"] = [{
            "workload": f"{w2.name}-shaped tensor list ({len(w2.numel)} tensors, d={w2.d}), "
                        f"m={w2.m}, tau={w2.tau}, base={w2.base}, grads={w2.grad_dtype}, "
                        f"policy={w2.policy}",
            "value": w2.updates_per_round * 3 / wall2, "unit": "updates/s", "steps": 3,
            "ms_per_step": 1e3 * wall2 / 3,
            "hbm_frac_whole_round": round_bytes(w2, f2) / wall2 * 3 / 1e9 / HBM_PEAK_GBPS,
            "roofline": {"bound": "hbm", "kernel": "k_local_step (steady state)",
                         "achieved": lb2 / (k2["local"] * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS,
                         "unit": "GB/s", "frac": lb2 / (k2["local"] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                         "algorithmic_bytes_per_launch": lb2,
                         "traffic": MEASURED_TRAFFIC_BYTES.get(w2.name)},
            "kernel_ms": k2}]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
