"""CPU ORACLE -- test infrastructure, not the product.

Algorithm 1 (Slow Momentum) driven step by step in the paper's order:
outer iteration t -> buffer policy (line 2) -> tau base-optimizer steps of
every worker (lines 3-5, directions of Table C.1) -> exact average, slow
momentum, outer iterate (lines 6-8).  The per-element arithmetic is the plain
C in slowmo_oracle.c, built in fp64 (the reference) and fp32 (noise floor).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this module.  It shares no code with the HIP path and does not import it.

Readings of the paper where it is silent or inconsistent: coupled L2 weight
decay; Adam's bias-correction exponent
counts the current update (starts at 1); eps is added after the square root of
the bias-corrected second moment; the learning rate is a per-call scalar (the
one given to the outer step is gamma_t of Eq. (2)-(3); the two schedules of
Section 4 / Appendix A.3 are plain functions of the step number); the mean is a
left-to-right sum over workers 0..m-1 followed by a division by m; "reset"
zeroes the buffers (and Adam's step counter) at the start of every outer
iteration, "maintain" leaves them alone, "average" replaces every worker's
buffers by their mean over the workers (same summation order as the
parameters; Adam's step counter runs on).  exact_average=False is the
"SlowMo-noaverage" variant of Section 6: no line 6, per-worker x0 and u.

Parity pins: tests/test_oracle_pins.py.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "slowmo_oracle.c")
_LIBS = {"f64": os.path.join(_HERE, "liboracle_f64.so"),
         "f32": os.path.join(_HERE, "liboracle_f32.so")}
_FLAGS = {"f64": ["-DREAL=double"], "f32": ["-DREAL=float", "-DORACLE_F32"]}
_loaded: dict = {}


def build(force: bool = False, src: str = _SRC, out: Optional[dict] = None) -> dict:
    """Compile the C oracle with gcc (both precisions).  Plain -O2, no
    fast-math, no FMA contraction, OpenMP over the element index only."""
    out = out or _LIBS
    for prec, path in out.items():
        if not force and os.path.exists(path) and \
                os.path.getmtime(path) >= os.path.getmtime(src):
            continue
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
               *_FLAGS[prec], "-o", path, src, "-lm"]
        subprocess.run(cmd, check=True)
    return out


def load(prec: str = "f64", path: Optional[str] = None) -> C.CDLL:
    key = (prec, path)
    if key in _loaded:
        return _loaded[key]
    if path is None:
        build()
        path = _LIBS[prec]
    lib = C.CDLL(path)
    want = 8 if prec == "f64" else 4
    lib.oracle_real_bytes.restype = C.c_int
    assert lib.oracle_real_bytes() == want, "oracle library has the wrong precision"
    lib.oracle_num_threads.restype = C.c_int
    p, i64, dbl = C.c_void_p, C.c_int64, C.c_double
    lib.oracle_sgd_nesterov_step.argtypes = [p, p, p, i64, dbl, dbl, dbl]
    lib.oracle_sgd_nesterov_step.restype = None
    lib.oracle_adam_step.argtypes = [p, p, p, p, i64, dbl, dbl, dbl, dbl, dbl, i64]
    lib.oracle_adam_step.restype = None
    lib.oracle_outer_step.argtypes = [p, C.c_int, i64, p, p, dbl, dbl, dbl]
    lib.oracle_outer_step.restype = None
    lib.oracle_average_buffers.argtypes = [p, C.c_int, i64]
    lib.oracle_average_buffers.restype = None
    lib.oracle_mix_step.argtypes = [p, p, C.c_int, i64, p]
    lib.oracle_mix_step.restype = None
    _loaded[key] = lib
    return lib


def exponential_graph_in_peers(m: int, step: int) -> np.ndarray:
    """Appendix C.1: with the workers ordered by rank, each one communicates in
    turn with the peer 2^0, 2^1, ..., 2^floor(log2(m-1)) hops away, one peer
    per iteration.  Worker i receives from worker (i - hop) mod m."""
    if m < 2:
        return np.zeros(max(m, 1), dtype=np.int32)
    n_hops = int(np.floor(np.log2(m - 1))) + 1 if m > 2 else 1
    hop = 1 << (step % n_hops)
    return ((np.arange(m) - hop) % m).astype(np.int32)


def lr_warmup_step_decay(base_lr: float, start_lr: float, warmup_steps: int, milestones,
                         factor: float, step: int) -> float:
    """Section 4 (CIFAR-10, ImageNet): the learning rate rises linearly during
    the warm-up and afterwards drops by a constant factor at every milestone.
    Steps are base-optimizer steps counted from 0; the rate reaches base_lr at
    step warmup_steps.  Where the paper is silent: the warm-up starts at
    start_lr, and a milestone counts from the step that bears its number."""
    if step < warmup_steps:
        return start_lr + (base_lr - start_lr) * step / warmup_steps
    passed = sum(1 for ms in milestones if step >= ms)
    return base_lr * factor ** passed


def lr_warmup_inverse_sqrt(peak_lr: float, init_lr: float, warmup_steps: int, step: int) -> float:
    """Appendix A.3 (WMT'16 En-De): the learning rate rises linearly to peak_lr
    over warmup_steps steps and then decays in proportion to the inverse square
    root of the step number (continuous at step warmup_steps)."""
    if step < warmup_steps:
        return init_lr + (peak_lr - init_lr) * step / warmup_steps
    return peak_lr * (warmup_steps / step) ** 0.5 if step > 0 else peak_lr


def _ptr(a: np.ndarray) -> C.c_void_p:
    assert a.flags["C_CONTIGUOUS"]
    return C.c_void_p(a.ctypes.data)


class SlowMoOracle:
    """State and control flow of Algorithm 1 for m workers over d elements.

    x[i] is worker i's replica, h[i] (and v[i]) its base-optimizer buffers,
    x0 the outer iterate x_{t,0}, u the slow momentum buffer (u_0 = 0).
    All workers start from the same point (Section 2).
    """

    def __init__(self, x_init, m: int, tau: int, alpha: float, beta: float,
                 base: str = "sgd_nesterov", policy: Optional[str] = None,
                 momentum: float = 0.0, weight_decay: float = 0.0,
                 beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
                 prec: str = "f64", lib: Optional[C.CDLL] = None,
                 exact_average: bool = True, tensor_sizes=None,
                 tensor_weight_decay=None, tensor_lr_scale=None):
        assert base in ("sgd_nesterov", "adam")
        if policy is None:      # the paper's defaults (Section 4, Appendix B.4)
            policy = "reset" if base == "sgd_nesterov" else "maintain"
        assert policy in ("reset", "maintain", "average")
        assert m >= 1 and tau >= 1
        self.lib = lib if lib is not None else load(prec)
        self.dtype = np.float64 if prec == "f64" else np.float32
        x_init = np.asarray(x_init)
        self.d = int(x_init.size)
        self.m, self.tau = int(m), int(tau)
        self.alpha, self.beta = float(alpha), float(beta)
        self.base, self.policy = base, policy
        self.momentum, self.weight_decay = float(momentum), float(weight_decay)
        self.beta1, self.beta2, self.eps = float(beta1), float(beta2), float(eps)
        # Optional per-tensor hyper-parameters ("parameter groups"): the flat
        # range is cut into tensors of the given sizes; tensor j uses weight
        # decay tensor_weight_decay[j] and the fast learning rate
        # lr * tensor_lr_scale[j] wherever gamma_t appears (Algorithm 1 lines
        # 4, 7 and 8).  The paper uses one value for all parameters.
        if tensor_sizes is None:
            assert tensor_weight_decay is None and tensor_lr_scale is None
            self.bounds = None
        else:
            sizes = [int(n) for n in tensor_sizes]
            assert sum(sizes) == self.d
            ends = np.cumsum(sizes)
            self.bounds = [(int(e - n), int(e)) for n, e in zip(sizes, ends)]
            nt = len(sizes)
            self.t_wd = [self.weight_decay] * nt if tensor_weight_decay is None \
                else [float(v) for v in tensor_weight_decay]
            self.t_lr = [1.0] * nt if tensor_lr_scale is None \
                else [float(v) for v in tensor_lr_scale]
            assert len(self.t_wd) == nt and len(self.t_lr) == nt
        self.exact_average = bool(exact_average)
        self.x0 = x_init.astype(self.dtype).reshape(self.d).copy()
        self.x = np.tile(self.x0, (self.m, 1))
        self.u = np.zeros(self.d, self.dtype)
        if not self.exact_average:
            # Section 6, "SlowMo-noaverage": line 6 is skipped and every worker
            # keeps its own outer iterate and slow momentum buffer
            self.x0 = self.x.copy()
            self.u = np.zeros((self.m, self.d), self.dtype)
        self.h = np.zeros((self.m, self.d), self.dtype)
        self.v = np.zeros((self.m, self.d), self.dtype) if base == "adam" else None
        self.w = np.ones(self.m, self.dtype)    # push-sum weights (Algorithm C.1), 1 unless mixing
        self.t = 0      # outer iteration
        self.k = 0      # inner step within the outer iteration
        self.l = 0      # Adam moment updates applied so far (bias-correction exponent)

    # Algorithm 1 line 2
    def _apply_buffer_policy(self) -> None:
        if self.policy == "reset":
            self.h[...] = 0
            if self.v is not None:
                self.v[...] = 0
            self.l = 0
        elif self.policy == "average":
            self.lib.oracle_average_buffers(_ptr(self.h), self.m, self.d)
            if self.v is not None:
                self.lib.oracle_average_buffers(_ptr(self.v), self.m, self.d)
        # "maintain": nothing to do

    # Algorithm 1 lines 3-5: one base-optimizer step on every worker
    def local_step(self, grads, lr: float) -> None:
        """grads: (m, d) float32 (bf16 inputs already widened)."""
        assert self.k < self.tau, "tau local steps already taken; outer step is due"
        g = np.ascontiguousarray(grads, dtype=np.float32).reshape(self.m, self.d)
        if self.k == 0:
            self._apply_buffer_policy()
        if self.base == "adam":
            self.l += 1
        for i in range(self.m):
            for a, b, lr_j, wd_j in self._groups(lr):
                if self.base == "sgd_nesterov":
                    self.lib.oracle_sgd_nesterov_step(
                        _ptr(self.x[i][a:b]), _ptr(self.h[i][a:b]), _ptr(g[i][a:b]), b - a,
                        lr_j, self.momentum, wd_j)
                else:
                    self.lib.oracle_adam_step(
                        _ptr(self.x[i][a:b]), _ptr(self.h[i][a:b]), _ptr(self.v[i][a:b]),
                        _ptr(g[i][a:b]), b - a, lr_j, self.beta1, self.beta2, self.eps,
                        wd_j, self.l)
        self.k += 1

    def _groups(self, lr: float):
        """(begin, end, learning rate, weight decay) of every parameter group:
        the whole range unless per-tensor hyper-parameters were given.  The
        scaled learning rate is rounded to fp32, the precision in which it
        reaches the kernels."""
        if self.bounds is None:
            return [(0, self.d, lr, self.weight_decay)]
        return [(a, b, float(np.float32(np.float32(lr) * np.float32(s))), wd)
                for (a, b), s, wd in zip(self.bounds, self.t_lr, self.t_wd) if b > a]

    exponential_graph_in_peers = staticmethod(exponential_graph_in_peers)
    lr_warmup_step_decay = staticmethod(lr_warmup_step_decay)
    lr_warmup_inverse_sqrt = staticmethod(lr_warmup_inverse_sqrt)

    # Algorithm C.1, communication half of a stochastic-gradient-push step
    def mix_step(self, in_peer) -> None:
        """x^{(i)} <- sum_j p(i,j) x^{(j)} and the same for the push-sum
        weights, with the column-stochastic P described by in_peer (worker i
        receives from in_peer[i]; in_peer[i] == i: from nobody)."""
        peers = np.ascontiguousarray(in_peer, dtype=np.int32)
        assert peers.shape == (self.m,) and peers.min() >= 0 and peers.max() < self.m
        self.lib.oracle_mix_step(_ptr(self.x), _ptr(self.w), self.m, self.d, _ptr(peers))

    def debiased(self) -> np.ndarray:
        """z^{(i)} = x^{(i)} / w_i (Algorithm C.1, last line)."""
        return self.x / self.w[:, None]

    # Algorithm 1 lines 6-8 (+ copy of x_{t+1,0} into every replica)
    def outer_step(self, lr: float) -> None:
        assert self.k == self.tau, "outer step needs exactly tau local steps"
        if self.exact_average and self.bounds is None:
            self.lib.oracle_outer_step(_ptr(self.x), self.m, self.d, _ptr(self.x0),
                                       _ptr(self.u), lr, self.alpha, self.beta)
        elif self.exact_average:
            # per tensor, with that tensor's gamma_t; the C routine wants the m
            # replicas of the range contiguous, so the range is copied out and back
            for a, b, lr_j, _ in self._groups(lr):
                xs = np.ascontiguousarray(self.x[:, a:b])
                self.lib.oracle_outer_step(_ptr(xs), self.m, b - a, _ptr(self.x0[a:b]),
                                           _ptr(self.u[a:b]), lr_j, self.alpha, self.beta)
                self.x[:, a:b] = xs
        else:
            # lines 7-8 on each worker's own replica: the "average" over that
            # one replica is the replica itself
            for i in range(self.m):
                for a, b, lr_j, _ in self._groups(lr):
                    self.lib.oracle_outer_step(_ptr(self.x[i][a:b]), 1, b - a,
                                               _ptr(self.x0[i][a:b]), _ptr(self.u[i][a:b]),
                                               lr_j, self.alpha, self.beta)
        if self.exact_average:
            self.w[...] = 1     # all mass is shared equally again after the exact average
        self.k = 0
        self.t += 1

    def run(self, grad_fn, lr, rounds: int) -> None:
        """grad_fn(t, k) -> (m, d) float32; lr a float or a callable lr(t)."""
        for _ in range(rounds):
            t = self.t
            g_t = lr(t) if callable(lr) else lr
            for k in range(self.tau):
                self.local_step(grad_fn(t, k), g_t)
            self.outer_step(g_t)
