"""GPU-resident synthetic problem for a workload: parameter replicas, gradient
buffers and index bookkeeping.  Allocation and input generation only -- the
optimizer itself is not involved (callers hand these tensors to it)."""
from __future__ import annotations

from typing import List, Sequence

import numpy as np

from . import device as _device
from . import generator as _gen
from .workloads import Workload


class IndexPlan:
    """Global element indices grouped by tensor: groups = [(tensor, offsets
    inside it as a device index tensor)], order = positions of those elements
    in the index array, group after group."""

    def __init__(self, prob: "GpuProblem", index: np.ndarray):
        self.index = np.asarray(index, dtype=np.int64)
        tensor, off = prob.locate(self.index)
        order = np.argsort(tensor, kind="stable")
        cuts = np.searchsorted(tensor[order], np.arange(len(prob.numel) + 1))
        self.order = order
        self.groups = []
        for j in range(len(prob.numel)):
            a, b = int(cuts[j]), int(cuts[j + 1])
            if b > a:
                self.groups.append((j, prob.torch.from_numpy(off[order[a:b]]).to(prob.device)))


class GpuProblem:
    """params[i][j]   worker i's replica of tensor j (fp32).  Worker 0 holds
                      the seeded x_{0,0}; the others are zero until the
                      optimizer's create call copies worker 0 into them.
       grads[s][i][j] gradient buffers, `ring` independent sets.

    param_layout / grad_layout:
      "separate"  every tensor is its own allocation (the allocator aligns it);
      "arena"     (parameters) one allocation for all workers, every tensor
                  512-byte aligned;
      "flat"      one allocation per worker, tensors back to back without
                  padding, so tensors after an odd-sized one are not 16-byte
                  aligned; gradients of one step are then produced by a single
                  launch over all workers;
      "padded"    (gradients) one allocation, every tensor starting at a
                  multiple of 512 bytes as the caching allocator would place a
                  separate allocation; one generator launch per tensor covers
                  all workers.
    """

    def __init__(self, w: Workload, device="cuda:0", ring: int = 1,
                 param_layout: str = "separate", grad_layout: str = "flat"):
        import torch
        self.torch = torch
        self.w = w
        self.device = torch.device(device)
        self.numel = w.numel
        self.starts = w.tensor_starts
        self.d = w.d
        self.ring = ring
        self.grad_layout = grad_layout
        self.gdtype = torch.bfloat16 if w.grad_dtype == "bf16" else torch.float32
        dev = self.device

        def views(flat):
            return [flat[int(s):int(s) + n] for s, n in zip(self.starts, self.numel)]

        if param_layout == "separate":
            self.params = [[torch.zeros(n, dtype=torch.float32, device=dev) for n in self.numel]
                           for _ in range(w.m)]
        elif param_layout == "arena":
            # one allocation for all workers, every tensor 512-byte aligned
            sizes = np.asarray(self.numel, dtype=np.int64)
            padded = (sizes + 127) // 128 * 128
            poff = np.concatenate([[0], np.cumsum(padded)[:-1]]).astype(np.int64)
            self._pflat = torch.zeros((w.m, int(max(padded.sum(), 128))), dtype=torch.float32,
                                      device=dev)
            self.params = [[self._pflat[i][int(o):int(o) + n] for o, n in zip(poff, self.numel)]
                           for i in range(w.m)]
        else:
            self._pflat = torch.zeros((w.m, max(self.d, 1)), dtype=torch.float32, device=dev)
            self.params = [views(self._pflat[i]) for i in range(w.m)]
        for j, t in enumerate(self.params[0]):          # x_{0,0} on worker 0
            _device.fill(t, int(self.starts[j]), w.seed ^ _gen.PARAM_SEED_XOR, 0, 0, 0.01)

        if grad_layout == "flat":
            self._gflat = [torch.zeros((w.m, max(self.d, 1)), dtype=self.gdtype, device=dev)
                           for _ in range(ring)]
            self.grads = [[views(g[i]) for i in range(w.m)] for g in self._gflat]
        elif grad_layout == "padded":
            unit = 512 // (2 if w.grad_dtype == "bf16" else 4)
            sizes = np.asarray(self.numel, dtype=np.int64)
            padded = (sizes + unit - 1) // unit * unit
            self._goff = np.concatenate([[0], np.cumsum(padded)[:-1]]).astype(np.int64)
            width = int(max(padded.sum(), unit))
            self._gflat = [torch.zeros((w.m, width), dtype=self.gdtype, device=dev)
                           for _ in range(ring)]
            self.grads = [[[g[i][int(o):int(o) + n] for o, n in zip(self._goff, self.numel)]
                           for i in range(w.m)] for g in self._gflat]
        else:
            self.grads = [[[torch.zeros(n, dtype=self.gdtype, device=dev) for n in self.numel]
                           for _ in range(w.m)] for _ in range(ring)]

    def fill_grads(self, slot: int, step: int) -> None:
        """Gradients of global step `step` (= t * tau + k) into ring slot `slot`."""
        w = self.w
        if self.d == 0:
            return
        if self.grad_layout == "flat":
            g = self._gflat[slot]
            _device.fill(g if w.m > 1 else g[0], 0, w.seed, 0, step, w.sigma, n_workers=w.m)
        elif self.grad_layout == "padded":
            g = self._gflat[slot]
            for j, n in enumerate(self.numel):
                if n:
                    _device.fill_strided(g, int(self._goff[j]), n, int(self.starts[j]), w.seed,
                                         step, w.sigma, w.m)
        else:
            for i in range(w.m):
                for j, t in enumerate(self.grads[slot][i]):
                    _device.fill(t, int(self.starts[j]), w.seed, i, step, w.sigma)

    # ---- index bookkeeping ----------------------------------------------------
    def locate(self, index: np.ndarray):
        """(tensor, offset) of global element indices."""
        index = np.asarray(index, dtype=np.int64)
        ends = self.starts + np.asarray(self.numel, dtype=np.int64)
        tensor = np.searchsorted(ends, index, side="right")
        return tensor, index - self.starts[tensor]

    def plan(self, index: np.ndarray) -> "IndexPlan":
        """Bookkeeping for repeated gathers at the same global indices."""
        return IndexPlan(self, index)

    def gather(self, tensors: Sequence, index) -> np.ndarray:
        """Values of a per-tensor list (e.g. one worker's replica) at global
        element indices (an array, or a plan() of one), as a host float32 array."""
        torch = self.torch
        plan = index if isinstance(index, IndexPlan) else IndexPlan(self, index)
        out = np.empty(plan.index.shape, dtype=np.float32)
        if plan.index.size == 0:
            return out
        parts = [tensors[j].reshape(-1)[idx] for j, idx in plan.groups]
        out[plan.order] = torch.cat(parts).to(torch.float32).cpu().numpy()
        return out

    def gather_all(self, tensors: Sequence) -> np.ndarray:
        """All values of a per-tensor list in global element order (one
        concatenation on the device, one copy), as a host float32 array."""
        torch = self.torch
        if self.d == 0:
            return np.empty(0, dtype=np.float32)
        flat = torch.cat([t.reshape(-1) for t in tensors]).to(torch.float32)
        return flat.cpu().numpy()

    def sample_indices(self, n_random: int, edges: Sequence[int] = (), halo: int = 8,
                       seed: int = 0) -> np.ndarray:
        """Sorted unique global indices: a halo around every tensor boundary
        and around the given extra edges (e.g. tile boundaries), the two ends
        of the range, and n_random uniformly drawn indices."""
        pts: List[np.ndarray] = []
        marks = np.concatenate([self.starts, self.starts + np.asarray(self.numel, np.int64),
                                np.asarray(list(edges), dtype=np.int64)])
        for d in range(-halo, halo):
            pts.append(marks + d)
        rng = np.random.default_rng(seed)
        pts.append(rng.integers(0, max(self.d, 1), size=n_random, dtype=np.int64))
        idx = np.unique(np.concatenate(pts))
        return idx[(idx >= 0) & (idx < self.d)]
