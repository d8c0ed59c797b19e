"""SlowMo: a thin holder around the C ABI for callers that keep their tensors
in PyTorch.  PyTorch supplies device memory and the stream; every step of the
method runs in libslowmo.so.
"""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Sequence

import torch

from . import binding as B

_BASE = {"sgd_nesterov": B.SLOWMO_SGD_NESTEROV, "adam": B.SLOWMO_ADAM}
_POLICY = {"reset": B.SLOWMO_BUF_RESET, "maintain": B.SLOWMO_BUF_MAINTAIN,
           "average": B.SLOWMO_BUF_AVERAGE}
_DTYPE = {"f32": B.SLOWMO_F32, "bf16": B.SLOWMO_BF16}
_TORCH_GRAD = {"f32": torch.float32, "bf16": torch.bfloat16}


def make_config(m: int, tau: int, alpha: float, beta: float, base: str = "sgd_nesterov",
                policy: Optional[str] = None, grad_dtype: str = "f32", momentum: float = 0.0,
                weight_decay: float = 0.0, beta1: float = 0.9, beta2: float = 0.999,
                eps: float = 1e-8, no_average: bool = False) -> B.slowmo_config:
    if policy is None:
        policy = "reset" if base == "sgd_nesterov" else "maintain"
    return B.slowmo_config(m=m, tau=tau, alpha=alpha, beta=beta, base=_BASE[base],
                           policy=_POLICY[policy], grad_dtype=_DTYPE[grad_dtype],
                           momentum=momentum, weight_decay=weight_decay,
                           beta1=beta1, beta2=beta2, eps=eps, no_average=int(no_average))


class SlowMo:
    """params[i][j]: worker i's replica of tensor j (fp32, contiguous, on one
    GPU).  Worker 0's values become the common starting point."""

    def __init__(self, params: Sequence[Sequence[torch.Tensor]], cfg: B.slowmo_config):
        m, n_t = len(params), len(params[0])
        assert m == cfg.m and all(len(p) == n_t for p in params)
        dev = params[0][0].device
        assert dev.type == "cuda", "parameters must live on the GPU"
        for p in params:
            for j, t in enumerate(p):
                assert t.dtype == torch.float32 and t.is_contiguous() and t.device == dev
                assert t.numel() == params[0][j].numel()
        self.cfg, self.m, self.n_tensors, self.device = cfg, m, n_t, dev
        self.params = [list(p) for p in params]          # keeps the memory alive
        self.numel = [int(t.numel()) for t in params[0]]
        self.grad_dtype = _TORCH_GRAD["bf16" if cfg.grad_dtype == B.SLOWMO_BF16 else "f32"]
        nbytes = B.slowmo_state_bytes(cfg, self.numel)
        if nbytes == 0:
            raise B.SlowMoError(B.SLOWMO_ERR_ARG, B.slowmo_last_error(None))
        self.state = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        ptrs = [t.data_ptr() if t.numel() else 0 for p in self.params for t in p]
        with torch.cuda.device(dev):
            self.ctx = B.slowmo_create(cfg, self.numel, ptrs, self.state.data_ptr(), nbytes,
                                       torch.cuda.current_stream(dev).cuda_stream)
        self._grad_key = None
        self._grad_arr = None

    def _pointer_array(self, tensors: Sequence[Sequence[torch.Tensor]], dtype):
        flat = []
        for i, g in enumerate(tensors):
            for j, t in enumerate(g):
                assert t.dtype == dtype and t.is_contiguous() and t.device == self.device
                assert t.numel() == self.numel[j]
                flat.append(t.data_ptr() if t.numel() else 0)
        assert len(flat) == self.m * self.n_tensors
        return (C.c_void_p * len(flat))(*[C.c_void_p(v) if v else None for v in flat])

    def grad_pointer_array(self, grads: Sequence[Sequence[torch.Tensor]]):
        """ctypes array of the m * n_tensors gradient addresses (reusable: building
        it walks every tensor in Python, which costs more than a kernel launch)."""
        return self._pointer_array(grads, self.grad_dtype)

    def param_pointer_array(self, tensors: Sequence[Sequence[torch.Tensor]]):
        """The same for fp32 tensors shaped like the replicas (destinations of debias)."""
        return self._pointer_array(tensors, torch.float32)

    def local_step(self, grads, lr: float) -> None:
        """grads: m lists of tensors, or an array from grad_pointer_array()."""
        arr = grads if isinstance(grads, C.Array) else self.grad_pointer_array(grads)
        B.slowmo_local_step(self.ctx, arr, lr, torch.cuda.current_stream(self.device).cuda_stream)

    def local_outer_step(self, grads, lr: float, outer_lr: Optional[float] = None) -> None:
        """Last local step of the outer iteration + outer step (fused when possible)."""
        arr = grads if isinstance(grads, C.Array) else self.grad_pointer_array(grads)
        B.slowmo_local_outer_step(self.ctx, arr, lr, lr if outer_lr is None else outer_lr,
                                  torch.cuda.current_stream(self.device).cuda_stream)

    def local_mix_step(self, grads, lr: float, in_peer: Sequence[int]) -> None:
        """A local step and the gossip step after it (fused when possible)."""
        arr = grads if isinstance(grads, C.Array) else self.grad_pointer_array(grads)
        B.slowmo_local_mix_step(self.ctx, arr, lr, in_peer,
                                torch.cuda.current_stream(self.device).cuda_stream)

    def mix_step(self, in_peer: Sequence[int]) -> None:
        B.slowmo_mix_step(self.ctx, in_peer, torch.cuda.current_stream(self.device).cuda_stream)

    def pushsum_weights(self):
        return B.slowmo_get_pushsum_weights(self.ctx, self.m)

    def debias(self, z) -> None:
        """z[i][j] <- x^{(i)}_j / w_i (fp32 CUDA tensors shaped like the replicas, or an
        array from param_pointer_array())."""
        arr = z if isinstance(z, C.Array) else self.param_pointer_array(z)
        B.slowmo_debias(self.ctx, arr, torch.cuda.current_stream(self.device).cuda_stream)

    def outer_step(self, lr: float) -> None:
        B.slowmo_outer_step(self.ctx, lr, torch.cuda.current_stream(self.device).cuda_stream)

    def set_tensor_hparams(self, weight_decay=None, lr_scale=None) -> None:
        B.slowmo_set_tensor_hparams(self.ctx, weight_decay, lr_scale,
                                    torch.cuda.current_stream(self.device).cuda_stream)

    def export_state(self) -> torch.Tensor:
        """The optimizer state (x0, u, h, v, counters) as one uint8 CUDA tensor."""
        n = B.slowmo_export_bytes(self.ctx)
        blob = torch.empty(n, dtype=torch.uint8, device=self.device)
        B.slowmo_export_state(self.ctx, blob.data_ptr(), n,
                              torch.cuda.current_stream(self.device).cuda_stream)
        return blob

    def import_state(self, blob: torch.Tensor) -> None:
        assert blob.dtype == torch.uint8 and blob.is_contiguous() and blob.device == self.device
        B.slowmo_import_state(self.ctx, blob.data_ptr(), blob.numel(),
                              torch.cuda.current_stream(self.device).cuda_stream)

    def counters(self):
        return B.slowmo_get_counters(self.ctx)

    def buffer(self, which: str, tensor: int, worker: int = 0) -> torch.Tensor:
        """A view (no copy) of x0 / u / h / v of one tensor inside the workspace."""
        code = {"x0": B.SLOWMO_BUF_X0, "u": B.SLOWMO_BUF_U, "h": B.SLOWMO_BUF_H,
                "v": B.SLOWMO_BUF_V}[which]
        addr = B.slowmo_get_buffer(self.ctx, code, worker, tensor)
        off = addr - self.state.data_ptr()
        n = self.numel[tensor]
        return self.state[off:off + 4 * n].view(torch.float32)

    def close(self) -> None:
        if getattr(self, "ctx", None) is not None:
            torch.cuda.synchronize(self.device)
            B.slowmo_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
