"""The microbenchmark ladder behind the kernels' access shape: plain read /
write / copy ceilings, the local step's 3-read/2-write mix under different
workgroup shapes, dispatch orders and cache hints, and the m-stream patterns of
the kernels that walk all workers per workgroup.  Every line is one shape of
csrc/streambench.hip, timed with HIP events on the launch stream
(`python bench.py --ladder`).  Measurement only."""
from __future__ import annotations

import json

HBM_PEAK_GBPS = 8000.0


def cases(m: int, n: int):
    """(label, kwargs of device.streambench, HBM bytes per launch)."""
    out = []

    def add(label, units, S, R, W, in_place=True, **kw):
        out.append((label, dict(units=units, S=S, R=R, W=W, in_place=in_place, **kw),
                    units * (R + W) * 4 * kw.get("n", n)))

    # ceilings.  A workgroup that moves 1 KiB is bound by the rate at which
    # workgroups are dispatched, so the plain streams also run with 16 KiB each.
    add("read,  1 KiB per workgroup (dispatch-bound)", m, 1, 1, 0)
    add("write, 1 KiB per workgroup (dispatch-bound)", m, 1, 0, 1)
    add("read,  256 threads x 4 vec4/lane", m, 1, 1, 0, B=256, VPT=4)
    add("write, 256 threads x 4 vec4/lane", m, 1, 0, 1, B=256, VPT=4)
    add("write, 256 threads x 4 vec4/lane, plain stores", m, 1, 0, 1, B=256, VPT=4, nt=0)
    add("copy (1 read, 1 write), 1 KiB per stream and workgroup", m, 2, 1, 1, in_place=False)
    add("copy, 256 threads x 4 vec4/lane", m, 2, 1, 1, in_place=False, B=256, VPT=4)
    # read : write mixes, one 1 KiB vector load or store per stream and wave
    add("2r/1w  in place", m, 2, 2, 1)
    add("3r/1w  in place", m, 3, 3, 1)
    add("1r/2w  out of place", m, 3, 1, 2, in_place=False)
    add("2r/2w  in place (first local step under \"reset\": x, g read; x, h written)", m, 2, 2, 2)
    add("3r/3w  in place", m, 3, 3, 3)
    add("4r/2w  in place", m, 4, 4, 2)
    add("4r/3w  in place (Adam: x, h, v, g read; x, h, v written)", m, 4, 4, 3)
    add("2 streams written per wave (nothing read)", m, 2, 0, 2)
    add("3 streams read per wave (nothing written)", m, 3, 3, 0)
    # the SGD local step's mix: x, h, g read; x, h written
    add("3r/2w  64 threads, 1 vec4/lane, retire, NT, XCD-contiguous  [library shape]", m, 3, 3, 2)
    add("3r/2w  same, plain loads and stores", m, 3, 3, 2, nt=0)
    add("3r/2w  same, NT loads, plain stores", m, 3, 3, 2, nt=1)
    add("3r/2w  same, plain loads, NT stores", m, 3, 3, 2, nt=2)
    add("3r/2w  same, NT, workgroup b takes tile b (no XCD remap)", m, 3, 3, 2, remap=False)
    add("3r/2w  128 threads", m, 3, 3, 2, B=128)
    add("3r/2w  256 threads", m, 3, 3, 2, B=256)
    add("3r/2w  1024 threads", m, 3, 3, 2, B=1024)
    add("3r/2w  64 threads, 4 vec4/lane (4 KiB per stream and wave)", m, 3, 3, 2, VPT=4)
    add("3r/2w  256 threads, 4 vec4/lane", m, 3, 3, 2, B=256, VPT=4)
    add("3r/2w  64 threads, workgroup loops over 16 consecutive tiles", m, 3, 3, 2, iters=16)
    add("3r/2w  256 threads, workgroup loops over 64 consecutive tiles", m, 3, 3, 2, B=256, iters=64)
    add("3r/2w  library shape, tiles dispatched worker-minor (tile k of every worker, then k+1)",
        m, 3, 3, 2, order=1)
    add("3r/2w  out of place (x, h written to other arrays)", m, 5, 3, 2, in_place=False)
    # all m workers per workgroup (outer step, gossip): m+2 streams read and written in place
    for B, V in ((64, 1), (64, 4), (256, 1), (256, 4), (256, 16), (512, 16), (1024, 4), (1024, 16)):
        add(f"{m + 2} streams in place per workgroup, {B} threads, {V} vec4/lane", 1, m + 2, m + 2,
            m + 2, B=B, VPT=V)
    add(f"{m + 2} streams in place, 1024 threads, 16 vec4/lane, no XCD remap", 1, m + 2, m + 2, m + 2,
        B=1024, VPT=16, remap=False)
    add(f"{m + 2} streams in place, 64 threads, 1 vec4/lane, no XCD remap", 1, m + 2, m + 2, m + 2,
        remap=False)
    add(f"{m + 2} streams in place, 64 threads, NT loads, plain stores", 1, m + 2, m + 2, m + 2, nt=1)
    # the same bytes with the m+2 streams cut into pieces that lie side by side
    # (what a caller could give only by interleaving the replicas)
    for piece in (65536, 16384, 4096, 256):
        if n % piece == 0:
            add(f"{m + 2} streams in place, streams cut into pieces of {piece * 4 // 1024} KiB laid "
                f"side by side", n // piece, m + 2, m + 2, m + 2, n=piece, stride=piece)
    add(f"{m} streams read per workgroup (nothing written)", 1, m, m, 0)
    add(f"{m} streams read, 1024 threads x 16 vec4/lane", 1, m, m, 0, B=1024, VPT=16)
    add(f"{m} streams written per workgroup (nothing read)", 1, m, 0, m)
    add(f"{m} streams written, plain stores", 1, m, 0, m, nt=0)
    add(f"{m} streams written, 1024 threads x 16 vec4/lane", 1, m, 0, m, B=1024, VPT=16)
    add(f"{m + 2} streams read, 2 of them written in place", 1, m + 2, m + 2, 2)
    add(f"{m + 2} streams read, 2 other streams written", 1, m + 4, m + 2, 2, in_place=False)
    add(f"{m + 2} streams read, 2 written in place, plain stores", 1, m + 2, m + 2, 2, nt=1)
    add(f"{m + 2} streams read, 2 written in place, 1024 threads x 16 vec4/lane", 1, m + 2, m + 2, 2,
        B=1024, VPT=16)
    add(f"{3 * m + 2} streams read, 2 written (last local step + average, no copy back)", 1,
        3 * m + 2, 3 * m + 2, 2)
    add(f"{3 * m + 2} streams read, 2 written, 1024 threads x 16 vec4/lane", 1, 3 * m + 2, 3 * m + 2,
        2, B=1024, VPT=16)
    return out


def run(m: int = 32, n: int = 25_559_040, reps: int = 5, device: str = "cuda:0"):
    """Times every case (1 untimed + `reps` timed launches, HIP events on the
    launch stream).  n is a multiple of every tile size used (65 536 floats)."""
    import torch
    from . import device as D
    assert n % 65536 == 0
    stride = n + 65536                         # streams start 256 KiB after the previous one ends
    all_cases = cases(m, n)
    most = max(kw["units"] * kw["S"] * kw.get("stride", stride) for _, kw, _ in all_cases)
    buf = torch.zeros(most, dtype=torch.float32, device=device)
    rows = []
    for label, kw, nbytes in all_cases:
        kw = dict(kw)
        args = (buf, kw.pop("stride", stride))
        kw.setdefault("n", n)
        D.streambench(*args, **kw)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            D.streambench(*args, **kw)
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / reps
        rows.append({"shape": label, "ms": ms, "GB/s": nbytes / ms / 1e6,
                     "frac": nbytes / ms / 1e6 / HBM_PEAK_GBPS, "bytes": nbytes})
    return {"m": m, "floats_per_stream": n, "reps": reps, "rows": rows}


def placement(m: int = 32, n: int = 25_559_040, count: int = 40, device: str = "cuda:0"):
    """The same three launches on `count` buffers allocated one after the other
    and kept (so that each lies in other physical memory): m+2 streams in place
    with single waves and with 1024-thread workgroups, and the local step's
    mix.  Shows how much of a kernel's figure is the place its operands
    happen to lie in (`python bench.py --placement`)."""
    import torch
    from . import device as D
    stride = n + 65536
    S = m + 2

    def frac(buf, **kw):
        D.streambench(buf, stride, n=n, **kw)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(5):
            D.streambench(buf, stride, n=n, **kw)
        b.record()
        torch.cuda.synchronize()
        return kw["units"] * (kw["R"] + kw["W"]) * 4 * n / (a.elapsed_time(b) / 5) / 1e6 / HBM_PEAK_GBPS

    keep = []
    for i in range(count):
        buf = torch.zeros(S * stride, dtype=torch.float32, device=device)
        keep.append(buf)
        f1 = frac(buf, units=1, S=S, R=S, W=S, in_place=True)
        f2 = frac(buf, units=1, S=S, R=S, W=S, in_place=True, B=1024, VPT=16)
        f3 = frac(buf, units=S // 3, S=3, R=3, W=2, in_place=True)
        print(f"buffer {i:2d} ({S * stride * 4 / 2**30:.2f} GiB, after {i * S * stride * 4 / 2**30:6.1f} GiB of "
              f"others): {S} streams in place, single waves {f1:.3f}; 1024 threads x 16 vec4/lane "
              f"{f2:.3f}; 3r/2w {f3:.3f}", flush=True)


def main(m: int = 32, n: int = 25_559_040):
    res = run(m, n)
    for r in res["rows"]:
        print(f"{r['frac']:.3f}  {r['GB/s']:7.0f} GB/s  {r['ms']:7.3f} ms  {r['shape']}", flush=True)
    print(json.dumps(res))
