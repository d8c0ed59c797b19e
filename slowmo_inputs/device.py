"""Device side of the seeded input generator: fills GPU tensors with the same
values generator.py computes on the host (bit for bit).  Test and benchmark
infrastructure; no optimizer arithmetic."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "csrc", "gradgen.hip")
SOURCES = [SRC, os.path.join(_HERE, "csrc", "streambench.hip")]
LIB_PATH = os.path.join(_HERE, "libslowmo_inputs.so")
_lib = None


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB_PATH) and \
            all(os.path.getmtime(LIB_PATH) >= os.path.getmtime(f) for f in SOURCES):
        return LIB_PATH
    hipcc = "/opt/rocm/bin/hipcc" if os.path.exists("/opt/rocm/bin/hipcc") else "hipcc"
    cmd = [hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
           "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-x", "hip", *SOURCES, "-o", LIB_PATH]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + r.stderr)
    return LIB_PATH


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run slowmo_inputs.device.build()")
        _lib = C.CDLL(LIB_PATH)
        _lib.slowmo_inputs_fill.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_uint64,
                                            C.c_int32, C.c_int32, C.c_int64, C.c_int64,
                                            C.c_float, C.c_int32, C.c_void_p]
        _lib.slowmo_inputs_fill.restype = C.c_int
        _lib.slowmo_inputs_calib_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        _lib.slowmo_inputs_calib_copy.restype = C.c_int
        _lib.slowmo_inputs_streambench.argtypes = [C.c_void_p, C.c_int64] + [C.c_int32] * 5 + \
            [C.c_int64] + [C.c_int32] * 7 + [C.c_void_p]
        _lib.slowmo_inputs_streambench.restype = C.c_int
    return _lib


def fill(out, first_index: int, seed: int, worker: int, step: int, scale: float,
         n_workers: int = 1, worker_stride: int = 0) -> None:
    """Fills a contiguous CUDA tensor (fp32 or bf16) with
    scale * n(seed, worker, step, first_index + j).  With n_workers > 1, `out`
    is 2-D [n_workers, n] and row w is filled for worker `worker + w`."""
    import torch
    assert out.is_cuda and out.is_contiguous()
    bf16 = {torch.float32: 0, torch.bfloat16: 1}[out.dtype]
    if n_workers > 1:
        assert out.dim() == 2 and out.shape[0] == n_workers
        n = out.shape[1]
        worker_stride = worker_stride or out.stride(0)
    else:
        n = out.numel()
    if n == 0:
        return
    rc = lib().slowmo_inputs_fill(out.data_ptr(), n, first_index, seed, worker, n_workers,
                                  worker_stride, step, scale, bf16,
                                  torch.cuda.current_stream(out.device).cuda_stream)
    if rc != 0:
        raise RuntimeError(f"slowmo_inputs_fill failed with hipError {rc}")


def fill_strided(buf, col0: int, n: int, first_index: int, seed: int, step: int, scale: float,
                 n_workers: int) -> None:
    """Fills buf[w, col0:col0+n] for workers w = 0..n_workers-1 (buf is a
    contiguous 2-D CUDA tensor with one row per worker) in one launch."""
    import torch
    assert buf.is_cuda and buf.is_contiguous() and buf.dim() == 2 and buf.shape[0] == n_workers
    assert 0 <= col0 and col0 + n <= buf.shape[1]
    bf16 = {torch.float32: 0, torch.bfloat16: 1}[buf.dtype]
    rc = lib().slowmo_inputs_fill(buf.data_ptr() + col0 * buf.element_size(), n, first_index, seed,
                                  0, n_workers, buf.stride(0), step, scale, bf16,
                                  torch.cuda.current_stream(buf.device).cuda_stream)
    if rc != 0:
        raise RuntimeError(f"slowmo_inputs_fill failed with hipError {rc}")


def calib_copy(src, dst) -> None:
    """dst <- src with the plain copy kernel k_calib_copy (known traffic:
    src.nbytes read, the same written), for scaling hardware counters."""
    import torch
    assert src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()
    nbytes = src.numel() * src.element_size()
    assert nbytes == dst.numel() * dst.element_size() and nbytes % 16 == 0
    rc = lib().slowmo_inputs_calib_copy(src.data_ptr(), dst.data_ptr(), nbytes,
                                        torch.cuda.current_stream(src.device).cuda_stream)
    if rc != 0:
        raise RuntimeError(f"slowmo_inputs_calib_copy failed with hipError {rc}")


def streambench(buf, stride: int, units: int, S: int, R: int, W: int, in_place: bool, n: int,
                B: int = 64, VPT: int = 1, nt: int = 3, order: int = 0, remap: bool = True,
                iters: int = 1, lds: int = 0) -> None:
    """One launch of the stream microbenchmark kernel (csrc/streambench.hip) on
    the fp32 CUDA tensor `buf` seen as units x S streams of n floats, `stride`
    floats apart.  nt: 1 = non-temporal loads, 2 = non-temporal stores, 3 = both."""
    import torch
    assert buf.is_cuda and buf.is_contiguous() and buf.dtype == torch.float32
    assert buf.numel() >= units * S * stride
    rc = lib().slowmo_inputs_streambench(buf.data_ptr(), stride, units, S, R, W, int(in_place), n,
                                         B, VPT, int(nt), order, int(remap), iters, lds,
                                         torch.cuda.current_stream(buf.device).cuda_stream)
    if rc != 0:
        raise RuntimeError(f"slowmo_inputs_streambench failed with hipError {rc}")
