"""Seeded synthetic gradient workloads shared by the tests, the benchmark and the smoke check.

Holds no arithmetic of the compression method: it only draws input vectors.
The five workloads stand in for the gradients of the paper's experiments
(Sec. 5: ResNets on CIFAR10/ImageNet, bucket sizes 8192 and 512, K simulated
workers); only tensor shapes, bucket sizes and K are borrowed, the values are
random.  Worker k of workload c uses generator seed 1000*c + k for the values
and quantizer seed k.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import torch


def resnet18_shapes() -> list[tuple[int, ...]]:
    """Parameter tensors of an ImageNet ResNet-18 in definition order (62 tensors)."""
    shapes: list[tuple[int, ...]] = [(64, 3, 7, 7), (64,), (64,)]
    inplanes = 64
    for planes, stride in ((64, 1), (128, 2), (256, 2), (512, 2)):
        for block in range(2):
            shapes += [(planes, inplanes, 3, 3), (planes,), (planes,),
                       (planes, planes, 3, 3), (planes,), (planes,)]
            if block == 0 and (stride != 1 or inplanes != planes):
                shapes += [(planes, inplanes, 1, 1), (planes,), (planes,)]
            inplanes = planes
    shapes += [(1000, 512), (1000,)]
    return shapes


def resnet50_shapes() -> list[tuple[int, ...]]:
    """Parameter tensors of an ImageNet ResNet-50 in definition order (161 tensors)."""
    shapes: list[tuple[int, ...]] = [(64, 3, 7, 7), (64,), (64,)]
    inplanes = 64
    for planes, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for block in range(blocks):
            shapes += [(planes, inplanes, 1, 1), (planes,), (planes,),
                       (planes, planes, 3, 3), (planes,), (planes,),
                       (planes * 4, planes, 1, 1), (planes * 4,), (planes * 4,)]
            if block == 0:
                shapes += [(planes * 4, inplanes, 1, 1), (planes * 4,), (planes * 4,)]
            inplanes = planes * 4
    shapes += [(1000, 2048), (1000,)]
    return shapes


def transformer_shapes(layers: int = 48, hidden: int = 1600, vocab: int = 50257,
                       positions: int = 1024) -> list[tuple[int, ...]]:
    """Decoder-only transformer: token + position tables, per layer two LayerNorms,
    fused qkv, output projection and a 4x MLP, final LayerNorm."""
    shapes: list[tuple[int, ...]] = [(vocab, hidden), (positions, hidden)]
    for _ in range(layers):
        shapes += [(hidden,), (hidden,),
                   (hidden, 3 * hidden), (3 * hidden,),
                   (hidden, hidden), (hidden,),
                   (hidden,), (hidden,),
                   (hidden, 4 * hidden), (4 * hidden,),
                   (4 * hidden, hidden), (hidden,)]
    shapes += [(hidden,), (hidden,)]
    return shapes


def _numel(shape: tuple[int, ...]) -> int:
    n = 1
    for x in shape:
        n *= x
    return n


@dataclass(frozen=True)
class Workload:
    cfg: int                 # 1..5, index into the benchmark's configs (1-based)
    name: str
    kind: str                # "gauss" | "layers" | "heavy"
    d: int
    bucket: int
    s: int
    K: int
    sizes: tuple[int, ...] = field(default=(), repr=False)   # tensor sizes for kind == "layers"
    log10_sigma: tuple[float, float] = (-5.0, -1.0)

    def value_seed(self, worker: int) -> int:
        return 1000 * self.cfg + worker

    def quant_seed(self, worker: int) -> int:
        return worker


def _layers(cfg, name, shapes, bucket, s, K, rng) -> Workload:
    sizes = tuple(_numel(x) for x in shapes)
    return Workload(cfg, name, "layers", sum(sizes), bucket, s, K, sizes, rng)


def workload(cfg: int) -> Workload:
    if cfg == 1:
        return Workload(1, "gauss-1M", "gauss", 1 << 20, 8192, 3, 1)
    if cfg == 2:
        w = _layers(2, "resnet18-shaped", resnet18_shapes(), 8192, 4, 1, (-5.0, -1.0))
        assert w.d == 11_689_512 and len(w.sizes) == 62
        return w
    if cfg == 3:
        w = _layers(3, "resnet50-shaped", resnet50_shapes(), 8192, 3, 8, (-5.0, -1.0))
        assert w.d == 25_557_032 and len(w.sizes) == 161
        return w
    if cfg == 4:
        return Workload(4, "heavy-tail-2^27", "heavy", 1 << 27, 16384, 7, 4)
    if cfg == 5:
        w = _layers(5, "transformer-1.5B-shaped", transformer_shapes(), 512, 3, 4, (-6.0, -2.0))
        assert w.d == 1_557_611_200
        return w
    raise ValueError("workloads are numbered 1..5")


def sync_stride(w: Workload) -> int:
    """The decoder-index stride the benchmark (and the full-size parity tests) use for a workload: the tile decoder
    parses a 2048-coordinate tile of K messages with 64 lanes, a piece each, so K * 2048 / stride = 64, kept within
    128..256 (a finer index costs more bytes than it saves time); one message alone decodes a lane per piece."""
    if w.K == 1:
        return 256
    return max(128, min(256, 32 * w.K))


def scaled(w: Workload, d_target: int) -> Workload:
    """Same structure at a smaller size (for CPU-sized tests): tensor sizes shrunk
    proportionally, at least one element each; flat workloads just shortened."""
    if w.kind != "layers":
        return Workload(w.cfg, w.name + "-small", w.kind, d_target, w.bucket, w.s, w.K)
    f = d_target / w.d
    sizes = tuple(max(1, int(round(n * f))) for n in w.sizes)
    return Workload(w.cfg, w.name + "-small", w.kind, sum(sizes), w.bucket, w.s, w.K, sizes, w.log10_sigma)


def generate(w: Workload, worker: int, device: str | torch.device = "cpu") -> torch.Tensor:
    """The fp32 gradient vector of `worker` for workload `w` on `device`."""
    device = torch.device(device)
    g = torch.Generator(device=device)
    g.manual_seed(w.value_seed(worker))
    out = torch.empty(w.d, dtype=torch.float32, device=device)
    chunk = 1 << 24
    if w.kind == "gauss":
        for lo in range(0, w.d, chunk):
            n = min(chunk, w.d - lo)
            out[lo:lo + n] = torch.randn(n, generator=g, device=device) * 0.01
    elif w.kind == "layers":
        gs = torch.Generator(device="cpu")
        gs.manual_seed(w.value_seed(worker) + 500_000)
        lo_e, hi_e = w.log10_sigma
        sig = 10.0 ** (lo_e + (hi_e - lo_e) * torch.rand(len(w.sizes), generator=gs, dtype=torch.float64))
        off = 0
        for n, sg in zip(w.sizes, sig.tolist()):
            for lo in range(0, n, chunk):
                m = min(chunk, n - lo)
                out[off + lo: off + lo + m] = torch.randn(m, generator=g, device=device) * sg
            off += n
    elif w.kind == "heavy":
        for lo in range(0, w.d, chunk):
            n = min(chunk, w.d - lo)
            z = torch.randn(4, n, generator=g, device=device)
            t = z[0] / torch.sqrt((z[1] * z[1] + z[2] * z[2] + z[3] * z[3]) / 3.0)   # Student-t, 3 d.o.f.
            big = torch.rand(n, generator=g, device=device) < 0.01
            out[lo:lo + n] = 1e-3 * t * torch.where(big, 100.0, 1.0)
    else:
        raise ValueError(w.kind)
    return out


def level_table(kind: str, s: int, p: float = 0.5) -> list[float]:
    """A level sequence l_0 = 0 < l_1 < ... < l_s < l_{s+1} = 1 to hand to the level-table entry points, as fp32
    values: "exp" (0, p^s, ..., p^2, p, 1) (p = 1/2: the nonuniform levels of the paper's main scheme),
    "uniform" (0, 1/(s+1), ..., s/(s+1), 1) (the uniform grid of QSGD).  An input like any other: the method's
    arithmetic starts where a table is used."""
    if kind == "exp":
        vals = [0.0] + [p ** (s + 1 - j) for j in range(1, s + 2)]
    elif kind == "uniform":
        vals = [j / (s + 1) for j in range(s + 2)]
    else:
        raise ValueError(kind)
    out = [float(torch.tensor(x, dtype=torch.float64).to(torch.float32)) for x in vals]
    out[0], out[-1] = 0.0, 1.0
    assert all(b > a for a, b in zip(out, out[1:])), "levels collapse in fp32"
    return out
