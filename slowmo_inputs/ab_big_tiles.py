"""Big tiles against single-wave tiles for the outer step and the fused last
step, measured in ONE process on the SAME replicas and gradients: two contexts
(created with SLOWMO_BIG_TILES=0 and =1) whose calls are timed in alternation
with HIP events.  Separate processes get different physical pages, and the
kernels that walk all workers differ by up to 15 % between placements, so a
comparison across processes says little.

    python -m slowmo_inputs.ab_big_tiles            # the table of profiles/outer_step_two_pass_and_wide_tiles.md
    python -m slowmo_inputs.ab_big_tiles --sweep    # one tensor of k big tiles, k = 4 .. 1024: where they start to pay

Measurement only."""
from __future__ import annotations

import dataclasses
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _context(w, prob, big: int):
    from paper_1910_00643_amd.optimizer import SlowMo, make_config
    old = os.environ.get("SLOWMO_BIG_TILES")
    os.environ["SLOWMO_BIG_TILES"] = str(big)       # read by slowmo_create
    try:
        cfg = make_config(m=w.m, tau=w.tau, alpha=w.alpha, beta=w.beta, base=w.base,
                          policy=w.policy, grad_dtype=w.grad_dtype, momentum=w.momentum,
                          weight_decay=w.weight_decay, beta1=w.beta1, beta2=w.beta2, eps=w.eps,
                          no_average=not w.exact_average)
        return SlowMo(prob.params, cfg)
    finally:
        if old is None:
            os.environ.pop("SLOWMO_BIG_TILES", None)
        else:
            os.environ["SLOWMO_BIG_TILES"] = old


def compare(name: str, fused: bool, reps: int = 6, **changes):
    """Median and minimum ms of the call with single-wave tiles and with big
    tiles.  fused: slowmo_local_outer_step (tau = 2: a first step, then the
    fused last step), else slowmo_outer_step (tau = 1).  name: a workload of
    slowmo_inputs.workloads, or "mini" (the small SGD configuration of the
    parity tests, for use with shapes=...)."""
    import torch
    from . import workloads as W
    from .gpu_problem import GpuProblem
    base = W.ragged_mini(m=changes.pop("m", 3)) if name == "mini" else W.BY_NAME[name]()
    w = dataclasses.replace(base, tau=2 if fused else 1, **changes)
    prob = GpuProblem(w, "cuda:0", ring=1, grad_layout="padded", param_layout="separate")
    prob.fill_grads(0, 0)
    opts = {b: _context(w, prob, b) for b in (0, 1)}
    arr = {b: o.grad_pointer_array(prob.grads[0]) for b, o in opts.items()}
    events = {0: [], 1: []}
    for r in range(reps + 1):                    # the first repetition is not timed
        for b in (0, 1):
            o = opts[b]
            o.local_step(arr[b], w.lr)
            a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            if fused:
                o.local_outer_step(arr[b], w.lr)
            else:
                o.outer_step(w.lr)
            e.record()
            if r:
                events[b].append((a, e))
    torch.cuda.synchronize()
    ms = {b: sorted(a.elapsed_time(e) for a, e in events[b]) for b in events}
    for o in opts.values():
        o.close()
    del prob, opts, arr
    torch.cuda.empty_cache()
    return w, {b: (v[len(v) // 2], v[0]) for b, v in ms.items()}


CASES = [("resnet50", True, {}), ("resnet50", True, dict(m=16)), ("resnet50", True, dict(m=8)),
         ("resnet50", True, dict(m=4)), ("resnet18", True, {}), ("resnet18", True, dict(m=32)),
         ("transformer_big", True, {}), ("transformer_big", True, dict(policy="reset")),
         ("resnet50", True, dict(policy="maintain")),
         ("resnet50", False, {}), ("resnet50", False, dict(m=8)), ("resnet18", False, {}),
         ("transformer_big", False, {})]


def main(repetitions: int = 2):
    for rep in range(repetitions):
        for name, fused, changes in CASES:
            w, ms = compare(name, fused, **changes)
            call = "last local step + outer step" if fused else "outer step"
            print(f"{name}-shaped m={w.m} {w.base} policy={w.policy}, {call}: single-wave tiles "
                  f"{ms[0][0]:.4f} ms (min {ms[0][1]:.4f}), big tiles {ms[1][0]:.4f} ms "
                  f"(min {ms[1][1]:.4f}), ratio {ms[1][0] / ms[0][0]:.3f}", flush=True)


def sweep():
    """One tensor of k whole big tiles: a big tile keeps one CU busy, so few of
    them leave the chip idle."""
    for m in (8, 32):
        for k in (4, 16, 32, 64, 96, 128, 192, 256, 384, 512, 1024):
            shapes = (("a", (k * 65536,)),)
            _, f = compare("mini", True, reps=8, m=m, shapes=shapes)
            _, o = compare("mini", False, reps=8, m=m, shapes=shapes)
            print(f"m={m} big tiles={k:5d}: last local step + outer step {f[0][0]:.4f} -> {f[1][0]:.4f} ms "
                  f"(ratio {f[1][0] / f[0][0]:.3f}); outer step {o[0][0]:.4f} -> {o[1][0]:.4f} ms "
                  f"(ratio {o[1][0] / o[0][0]:.3f})", flush=True)


if __name__ == "__main__":
    sweep() if "--sweep" in sys.argv[1:] else main()
