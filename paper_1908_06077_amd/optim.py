"""Alg. 1 as a torch optimizer over a module's parameters, K simulated workers on one device.

The optimizer owns one flat fp32 vector for the parameters and one per worker for the gradients; every parameter's
`.data` becomes a view into the first and, while worker k computes, its `.grad` a view into worker k's vector, so
that autograd writes the K gradients straight into the buffers the encoder reads.  step() is then one call of
DataParallelSGD.step: quantize + ENCODE of the K gradients, DECODE + aggregate + parameter update (plain rule, or
the momentum rule of Sec. 4.2).  Nothing here computes: flattening is done by views, every step of the path runs
in the library's kernels.

    opt = NUQSGD(model.parameters(), K=4, lr=0.1, bucket=512, s=3)
    for k in range(4):
        with opt.worker(k):                  # gradients of this block go to worker k
            loss_fn(model(x[k]), y[k]).backward()
    opt.step()

The diagnostic of App. J (normalized variance of the quantized gradient) is gradient_variance().
"""
from __future__ import annotations

import contextlib

import torch

from . import sgd


class NUQSGD(torch.optim.Optimizer):
    def __init__(self, params, K: int, lr: float, bucket: int = 8192, s: int = 3, sync_stride: int = 256,
                 momentum: float = 0.0, nesterov_l: float = 0.0, seed: int = 0):
        if K < 1:
            raise ValueError("K >= 1 workers")
        super().__init__(params, dict(lr=lr, momentum=momentum, nesterov_l=nesterov_l))
        if len(self.param_groups) != 1:
            raise ValueError("one parameter group: Alg. 1 has one step size")
        self.params = [p for p in self.param_groups[0]["params"] if p.requires_grad]
        if not self.params:
            raise ValueError("no parameters to optimize")
        dev = self.params[0].device
        if any(p.dtype != torch.float32 or p.device != dev or not p.is_cuda for p in self.params):
            raise ValueError("fp32 parameters on one GPU are needed")
        # the flat vectors are the parameters one after the other, in the order given
        self.offsets, d = [], 0
        for p in self.params:
            self.offsets.append(d)
            d += p.numel()
        self.d, self.K = d, K
        self.flat_w = torch.zeros(d, dtype=torch.float32, device=dev)
        self.flat_g = [torch.zeros(d, dtype=torch.float32, device=dev) for _ in range(K)]
        for p, o in zip(self.params, self.offsets):
            view = self.flat_w[o:o + p.numel()].view_as(p)
            view.copy_(p.data)
            p.data = view
        self.engine = sgd.DataParallelSGD(self.flat_w, K, lr, bucket, s, sync_stride=sync_stride, mu=momentum,
                                          l=nesterov_l, seed=seed)
        self.bucket, self.s, self.sync_stride = bucket, s, sync_stride
        self._estimate = None

    def _grad_views(self, k: int):
        return [self.flat_g[k][o:o + p.numel()].view_as(p) for p, o in zip(self.params, self.offsets)]

    @contextlib.contextmanager
    def worker(self, k: int):
        """Inside the block the parameters' .grad are (zeroed) views into worker k's gradient vector."""
        if not 0 <= k < self.K:
            raise ValueError("worker index out of range")
        self.flat_g[k].zero_()
        for p, gv in zip(self.params, self._grad_views(k)):
            p.grad = gv
        try:
            yield
        finally:
            for p, gv in zip(self.params, self._grad_views(k)):
                if p.grad is not None and p.grad.data_ptr() != gv.data_ptr():
                    gv.copy_(p.grad)         # autograd replaced the tensor instead of accumulating into it
                p.grad = None

    @torch.no_grad()
    def step(self, closure=None):
        if closure is not None:
            raise ValueError("closures are not supported: the K gradients are computed in worker() blocks")
        self.engine.alpha = float(self.param_groups[0]["lr"])
        self.engine.step(self.flat_g)

    def zero_grad(self, set_to_none: bool = True):
        for g in self.flat_g:
            g.zero_()
        for p in self.params:
            p.grad = None

    @torch.no_grad()
    def gradient_variance(self, k: int = 0, draws: int = 16, seed: int = 1 << 32) -> float:
        """App. J: mean normalized variance of Q(g_k) over `draws` independent quantizations of worker k's
        current gradient (each draw quantized, ENCODEd and DECODEd by the library)."""
        if self._estimate is None:
            self._estimate = sgd.QuantizedEstimate(self.d, self.bucket, self.s, self.flat_w.device, self.sync_stride)
            self._q = torch.empty(self.d, dtype=torch.float32, device=self.flat_w.device)
        acc = sgd.NormalizedVariance(self.d, self.flat_w.device)
        for m in range(draws):
            acc.add(self._estimate(self.flat_g[k], seed + m, self._q))
        return acc.value()
