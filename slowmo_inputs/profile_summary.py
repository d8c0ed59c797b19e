"""Turns the output of three rocprofv3 runs of one bench.py command into a
summary under profiles/ and records the measured HBM traffic of the dominant
kernel in profiles/traffic.json (which bench.py reads for `roofline.traffic`).

The three runs, each with `-f csv -d <dir>/<pass>` and the same bench.py command
(which must include --calibrate-copy, --no-others and --no-cpu-baseline):
    <dir>/kt     rocprofv3 --kernel-trace --stats
    <dir>/fetch  rocprofv3 --pmc FETCH_SIZE
    <dir>/write  rocprofv3 --pmc WRITE_SIZE
and <dir>/kt.log holding bench.py's output of the kernel-trace run.

    python -m slowmo_inputs.profile_summary <dir> <bench.py arguments ...>

Measurement tooling; no optimizer arithmetic."""
from __future__ import annotations

import argparse
import collections
import csv
import dataclasses
import glob
import json
import os
import re
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

KERNEL = re.compile(r"(k_[a-z_]+(?:<[^>]*>)?)")


def _newest(pattern):
    files = sorted(glob.glob(pattern), key=os.path.getmtime)
    if not files:
        raise FileNotFoundError(pattern)
    return files[-1]


def _kernel(name):
    m = KERNEL.search(name)
    return m.group(1) if m else None


def _counter(path):
    """{kernel: [counter value of every dispatch]} of a counter_collection.csv."""
    out = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        k = _kernel(r["Kernel_Name"])
        if k:
            out[k].append(float(r["Counter_Value"]))
    return out


def _durations(path):
    """{kernel: [duration in ns of every dispatch]} of a kernel_trace.csv."""
    out = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        k = _kernel(r["Kernel_Name"])
        if k:
            out[k].append(float(r["End_Timestamp"]) - float(r["Start_Timestamp"]))
    return out


def _targs(kernel):
    inner = kernel.partition("<")[2].rstrip(">")
    return [a.strip() for a in inner.split(",")] if inner else []


def family(kernel):
    """(kind of library call the kernel belongs to, steady): steady = not a
    first-step / last-step variant."""
    name = kernel.partition("<")[0]
    a = _targs(kernel)
    fam = {"k_local_step": "local", "k_local_outer_step": "local_outer", "k_outer_step": "outer",
           "k_local_outer_big": "local_outer", "k_outer_big": "outer",
           "k_mix_step": "mix", "k_local_mix_step": "local_mix", "k_outer_noavg": "outer_noavg",
           "k_debias": "debias", "k_calib_copy": "copy"}.get(name)
    steady = True
    if name == "k_local_step":
        steady = a[2] == "false" and a[3] == "false"
    elif name in ("k_local_mix_step", "k_local_outer_step", "k_local_outer_big"):
        steady = a[2] == "false"
    return fam, steady


def algorithmic_bytes(kernel, w, rounds, dispatches):
    """(read bytes, written bytes, library calls) of ALL dispatches of this
    kernel instance in a run of `rounds` outer iterations; None for kernels that
    are not the library's.  Every kernel but the gossip kernels is launched once
    per call."""
    import bench
    name = kernel.partition("<")[0]
    a = _targs(kernel)
    g = 2 if w.grad_dtype == "bf16" else 4
    nbuf = 2 if w.base == "adam" else 1
    reset = w.policy == "reset"
    d = w.d
    md = w.m * d

    def local(first, last):
        return 4 + (0 if first else 4 * nbuf) + g, 4 + (0 if last else 4 * nbuf)

    calls = dispatches
    if name == "k_local_step":
        r, wr = local(a[2] == "true", a[3] == "true")
        return r * md * calls, wr * md * calls, calls
    if name == "k_local_mix_step":
        first = a[2] == "true"
        r, wr = local(first, False)
        calls = (rounds if reset else 1) if first else rounds * w.tau - (rounds if reset else 1)
        return r * md * calls, wr * md * calls, calls
    if name == "k_mix_step":
        calls = rounds * w.tau
        return 4 * md * calls, 4 * md * calls, calls
    # the outer step and the fused last step run as two kernels when big tiles
    # are in use: the whole 65 536-element pieces, and the rest
    if name in ("k_local_outer_step", "k_local_outer_big"):
        first = a[2] == "true"
        r = w.m * (4 + (0 if first else 4 * nbuf) + g) + 8
        wr = 4 * w.m + 8 + (0 if reset else 4 * nbuf * w.m)
        big = bench.big_elements(w, True)
        n = big if name == "k_local_outer_big" else d - big
        return r * n * calls, wr * n * calls, calls
    if name in ("k_outer_step", "k_outer_big"):
        b = bench.outer_bytes_per_element(w)
        big = bench.big_elements(w, False)
        n = big if name == "k_outer_big" else d - big
        return b // 2 * n * calls, b // 2 * n * calls, calls
    if name == "k_outer_noavg":
        return 12 * md * calls, 12 * md * calls, calls
    if name == "k_debias":
        return 4 * md * calls, 4 * md * calls, calls
    if name == "k_calib_copy":
        return calls << 30, calls << 30, calls
    return None


def summarize(directory, bench_args, out_md, title, extra_note=""):
    import bench
    from slowmo_inputs import workloads as W
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="resnet50")
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--policy", default=None)
    ap.add_argument("--mix", default=None)
    ap.add_argument("--no-average", action="store_true")
    ap.add_argument("--unfused", action="store_true")
    a, _ = ap.parse_known_args(bench_args)
    w = W.BY_NAME[a.workload]()
    if a.policy:
        w = dataclasses.replace(w, policy=a.policy)
    if a.no_average:
        w = dataclasses.replace(w, exact_average=False)
    if a.mix:
        w = dataclasses.replace(w, mix=a.mix)
    rounds = a.warmup + 2 * a.steps          # warm-up, timed pass, per-kernel pass
    dur = _durations(_newest(f"{directory}/kt/*/*_kernel_trace.csv"))
    try:
        fetch = _counter(_newest(f"{directory}/fetch/*/*_counter_collection.csv"))
        write = _counter(_newest(f"{directory}/write/*/*_counter_collection.csv"))
    except FileNotFoundError:       # a kernel-trace-only profile: traffic not measured
        fetch = write = None
    line = [ln for ln in open(f"{directory}/kt.log") if ln.startswith("{")][-1]
    j = json.loads(line)
    cal = "k_calib_copy"
    counters = fetch is not None
    fs = 1048576.0 / (sum(fetch[cal]) / len(fetch[cal])) if counters else 0.0
    ws = 1048576.0 / (sum(write[cal]) / len(write[cal])) if counters else 0.0
    fetch, write = fetch or {}, write or {}
    cmd = "python3 $R/bench.py " + " ".join(bench_args)
    name = os.path.basename(os.path.normpath(directory))
    where = "$R/" + os.path.relpath(os.path.abspath(directory), ROOT)   # as given on the command line
    out = [f"# rocprofv3 summary: {title}\n",
           f"Workload: {bench.describe(w)}. One MI355X; {a.warmup} warm-up + {a.steps} timed + "
           f"{a.steps} per-kernel-timed outer iterations per run; three runs of the same command "
           "under different rocprofv3 options.\n",
           "Commands (run from /tmp with TMPDIR=/tmp; `$R` is the repository root):\n",
           "```",
           f"rocprofv3 --kernel-trace --stats -f csv -d {where}/kt -- {cmd}",
           *([f"rocprofv3 --pmc FETCH_SIZE -f csv -d {where}/fetch -- {cmd}",
              f"rocprofv3 --pmc WRITE_SIZE -f csv -d {where}/write -- {cmd}"]
             if counters else []),
           f"python3 -m slowmo_inputs.profile_summary {where} {' '.join(bench_args)}",
           "```\n",
           ("Counter scaling: `k_calib_copy` moves exactly 1 048 576 KiB each way per launch; "
            f"FETCH_SIZE reads {sum(fetch[cal]) / len(fetch[cal]):.2f} for it (factor {fs:.5f}), "
            f"WRITE_SIZE {sum(write[cal]) / len(write[cal]):.2f} (factor {ws:.5f}).\n") if counters
           else "Kernel trace only: the HBM counters were not collected for this command.\n",
           "A library call may launch its kernel several times (the gossip kernels run once per "
           "connected group of workers): durations, traffic and algorithmic bytes below are "
           "summed over all dispatches of a kernel and divided by the number of library calls.\n",
           "| kernel | dispatches | calls | ms per call (kernel trace) | min / max ms per dispatch | "
           "algorithmic bytes per call | GB/s | of 8 TB/s | fetched (scaled) / algorithmic read | "
           "written (scaled) / algorithmic written | traffic bytes per call | traffic / algorithmic |",
           "|---|---|---|---|---|---|---|---|---|---|---|---|"]
    fam_traffic = collections.defaultdict(float)      # steady-state families: bytes per call
    fam_biggest = {}
    for k in sorted(dur):
        ab = algorithmic_bytes(k, w, rounds, len(dur[k]))
        if ab is None or ab[2] <= 0 or ab[0] + ab[1] <= 0:
            continue
        ar, aw, calls = ab
        total_ms = sum(dur[k]) / 1e6
        fr = sum(fetch.get(k, [])) * fs * 1024
        wr = sum(write.get(k, [])) * ws * 1024
        gbps = (ar + aw) / calls / (total_ms / calls * 1e-3) / 1e9
        tr = (f"{fr / ar:.4f} | {wr / aw:.4f} | {(fr + wr) / calls:.0f} | {(fr + wr) / (ar + aw):.4f}"
              if k in fetch and k in write else "not measured | not measured | | ")
        out.append(f"| `{k}` | {len(dur[k])} | {calls} | {total_ms / calls:.4f} | "
                   f"{min(dur[k]) / 1e6:.4f} / {max(dur[k]) / 1e6:.4f} | {(ar + aw) // calls} | "
                   f"{gbps:.0f} | {gbps / 8000:.3f} | {tr} |")
        fam, steady = family(k)
        if steady and k in fetch and k in write:
            fam_traffic[fam] += (fr + wr) / calls
            if fam not in fam_biggest or ar + aw > fam_biggest[fam][1]:
                fam_biggest[fam] = (k, ar + aw)
    km = {k: v for k, v in j.get("kernels", {}).items()}
    out.append("\nHIP-event averages per library call printed by bench.py in the kernel-trace run: "
               + ", ".join(f"{k} {v['ms']:.4f} ms ({v['frac']:.3f} of peak)" for k, v in km.items())
               + f"; {j['ms_per_step']:.3f} ms per outer iteration "
               f"(median {j['round_ms']['median']:.3f}, min {j['round_ms']['min']:.3f}).\n")
    if extra_note:
        out.append(extra_note + "\n")
    open(out_md, "w").write("\n".join(out))
    # the dominant call kind's measured traffic, for bench.py's roofline.traffic
    dom = {"k_local_step": "local", "k_local_mix_step": "local_mix"}.get(
        j["roofline"]["kernel"].split(" ")[0])
    traffic = dict(fam_traffic)
    if dom in fam_traffic and not a.unfused:      # bench.py's default run is the fused one
        tf = os.path.join(ROOT, "profiles", "traffic.json")
        try:
            data = json.load(open(tf))
        except (OSError, ValueError):
            data = {"what": "HBM bytes per library call of the dominant kernel (all its launches), "
                            "FETCH_SIZE + WRITE_SIZE scaled by a copy kernel of known size; "
                            "written by slowmo_inputs/profile_summary.py", "entries": []}
        variant = bench.variant_name(w)
        data["entries"] = [e for e in data["entries"]
                           if not (e["workload"] == w.name and e["variant"] == variant)]
        data["entries"].append({"workload": w.name, "variant": variant,
                                "kernel": fam_biggest[dom][0],
                                "bytes_per_launch": int(fam_traffic[dom]),
                                "source": os.path.relpath(out_md, ROOT)})
        data["entries"].sort(key=lambda e: (e["workload"], e["variant"]))
        json.dump(data, open(tf, "w"), indent=1)
    return traffic


if __name__ == "__main__":
    d = sys.argv[1]
    rest = sys.argv[2:]
    title = "kernels of `bench.py " + " ".join(x for x in rest if x not in
                                              ("--no-cpu-baseline", "--no-others",
                                               "--calibrate-copy")) + "`"
    nm = os.path.basename(os.path.normpath(d))
    nm = nm[5:] if nm.startswith("prof_") else nm
    note = ""
    if "--no-average" in rest:
        note = ("HBM counters for this variant are deliberately not collected.  The one attempt "
                "(`rocprofv3 --pmc FETCH_SIZE` on this command with --steps 5) stopped producing "
                "output right after the profiler's start-up line and was ended from outside after "
                "three minutes; it was the eighth profiler process of that session, the seven "
                "before it (same command line apart from the variant flag) and the kernel-trace "
                "pass of this very command had each finished in about four seconds, and every "
                "other variant was profiled later without incident.  Whether counter collection "
                "or a kernel under counter collection stalled cannot be told from the log, so "
                "the pass has not been repeated; `k_outer_noavg` moves 24 bytes per worker and "
                "element by construction (3 streams read, 3 written, one workgroup per tile).")
    print(summarize(d, rest, os.path.join(ROOT, "profiles", nm + ".md"), title, note))
