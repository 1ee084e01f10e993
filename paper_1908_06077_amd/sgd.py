"""Alg. 1 (data-parallel SGD with coded gradients) on one device, and the variance diagnostic of App. J.

Buffer management around the library calls only: the K workers' gradients of one step are quantized and
ENCODEd in one launch, the K messages are DECODEd and aggregated in one launch, and the parameters move
inside that launch (plain rule: the decoder adds -alpha/K times the sum onto w; momentum rule of Sec. 4.2:
the decoder applies it to w and y^l) or, on request, by the momentum kernel after it.  On several devices each worker would run the encode half on its own gradient, exchange
messages, and run the decode half on the K messages it holds; here the exchange is the identity.
"""
from __future__ import annotations

import torch

from . import binding as nuq


def step_seed(seed0: int, t: int, K: int, k: int) -> int:
    """Quantizer seed of worker k at step t: a separate random stream for every (t, k)."""
    return (seed0 + t * K + k) & (2 ** 64 - 1)


class MessageBuffers:
    """K messages and the encode workspace for gradients of length d, allocated once."""

    def __init__(self, K: int, d: int, bucket: int, s: int, sync_stride: int, device: torch.device):
        B = nuq.nuq_num_buckets(d, bucket)
        nsync = nuq.nuq_num_sync(bucket, sync_stride)
        cap = nuq.nuq_max_words(d, bucket, s)
        self.messages = [nuq.Message(torch.empty(B, dtype=torch.float32, device=device),
                                     torch.empty(B + 1, dtype=torch.int64, device=device),
                                     torch.zeros(cap, dtype=torch.int32, device=device),
                                     torch.empty(max(1, B * nsync), dtype=torch.int32, device=device))
                         for _ in range(K)]
        self.workspace = torch.empty(nuq.nuq_encode_workspace_bytes(K, d, bucket, s), dtype=torch.uint8, device=device)


class DataParallelSGD:
    """Alg. 1 with Omega = R^d on a flat fp32 parameter vector w (updated in place).

    mu = 0 gives the plain aggregate step; mu > 0 the momentum rule of Sec. 4.2 (l = 0 heavy ball, l = 1 Nesterov).
    """

    def __init__(self, w: torch.Tensor, K: int, alpha: float, bucket: int, s: int, sync_stride: int = 256,
                 mu: float = 0.0, l: float = 0.0, seed: int = 0, fused: bool = True):
        if w.dtype != torch.float32 or not w.is_cuda or not w.is_contiguous() or w.dim() != 1:
            raise ValueError("w: flat contiguous fp32 device tensor")
        self.w, self.K, self.alpha, self.mu, self.l = w, K, float(alpha), float(mu), float(l)
        self.bucket, self.s, self.sync_stride, self.seed, self.t = bucket, s, sync_stride, seed, 0
        self.d = w.numel()
        self.buffers = MessageBuffers(K, self.d, bucket, s, sync_stride, w.device)
        self.fused = fused            # momentum rule inside the decoder's launch, or as a kernel of its own
        if self.mu != 0.0:
            self.yl = w.clone()
            if not fused:
                self.avg = torch.empty_like(w)

    def encode(self, grads: list[torch.Tensor]) -> list[nuq.Message]:
        """Transmitter half of one step: K gradients -> K messages."""
        seeds = [step_seed(self.seed, self.t, self.K, k) for k in range(self.K)]
        nuq.nuq_quantize_encode_batch(grads, self.bucket, self.s, seeds, self.sync_stride, self.buffers.messages,
                                      self.buffers.workspace)
        return self.buffers.messages

    def apply(self, messages: list[nuq.Message]) -> None:
        """Receiver half: DECODE the K messages, aggregate, move w."""
        if self.mu == 0.0:
            nuq.nuq_decode_accumulate(messages, self.d, self.bucket, self.s, self.sync_stride,
                                      -self.alpha / self.K, True, self.w)
        elif self.fused:
            nuq.nuq_decode_momentum_step(messages, self.d, self.bucket, self.s, self.sync_stride, 1.0 / self.K,
                                         self.alpha, self.mu, self.l, self.w, self.yl)
        else:
            nuq.nuq_decode_accumulate(messages, self.d, self.bucket, self.s, self.sync_stride, 1.0 / self.K, False,
                                      self.avg)
            nuq.nuq_momentum_step(self.w, self.yl, self.avg, self.alpha, self.mu, self.l)
        self.t += 1

    def step(self, grads: list[torch.Tensor]) -> None:
        if len(grads) != self.K:
            raise ValueError("one gradient per worker")
        self.apply(self.encode(grads))


class QuantizedEstimate:
    """Q(g) of one worker as a dense fp32 vector: quantize + ENCODE + DECODE with fresh randomness per call."""

    def __init__(self, d: int, bucket: int, s: int, device: torch.device, sync_stride: int = 256):
        self.d, self.bucket, self.s, self.sync_stride = d, bucket, s, sync_stride
        self.buffers = MessageBuffers(1, d, bucket, s, sync_stride, device)

    def __call__(self, g: torch.Tensor, seed: int, out: torch.Tensor) -> torch.Tensor:
        nuq.nuq_quantize_encode_batch([g], self.bucket, self.s, [seed], self.sync_stride, self.buffers.messages,
                                      self.buffers.workspace)
        nuq.nuq_decode_accumulate(self.buffers.messages, self.d, self.bucket, self.s, self.sync_stride, 1.0, False, out)
        return out


class NormalizedVariance:
    """Mean normalized variance of App. J over the draws passed to add()."""

    def __init__(self, d: int, device: torch.device):
        self.total = torch.zeros(d, dtype=torch.float64, device=device)
        self.total_sq = torch.zeros(d, dtype=torch.float64, device=device)
        self.workspace = torch.empty(nuq.VARIANCE_WORKSPACE_BYTES, dtype=torch.uint8, device=device)
        self.out2 = torch.empty(2, dtype=torch.float64, device=device)
        self.M = 0

    def add(self, g: torch.Tensor) -> None:
        nuq.nuq_moments_accumulate(g, self.total, self.total_sq)
        self.M += 1

    def value(self) -> float:
        nuq.nuq_normalized_variance(self.total, self.total_sq, self.M, self.workspace, self.out2)
        var, second = self.out2.tolist()
        return var / second
