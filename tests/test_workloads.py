"""The synthetic workload generators: sizes, determinism, value scale."""
import torch

import workloads


def test_workload_sizes():
    assert workloads.workload(1).d == 1 << 20
    assert workloads.workload(2).d == 11_689_512 and len(workloads.workload(2).sizes) == 62
    assert workloads.workload(3).d == 25_557_032 and len(workloads.workload(3).sizes) == 161
    assert workloads.workload(4).d == 1 << 27
    assert workloads.workload(5).d == 1_557_611_200
    for c, (n, s, K) in {1: (8192, 3, 1), 2: (8192, 4, 1), 3: (8192, 3, 8), 4: (16384, 7, 4), 5: (512, 3, 4)}.items():
        w = workloads.workload(c)
        assert (w.bucket, w.s, w.K) == (n, s, K)


def test_generate_is_deterministic_and_scaled():
    w = workloads.scaled(workloads.workload(3), 60_000)
    a = workloads.generate(w, 0)
    b = workloads.generate(w, 0)
    c = workloads.generate(w, 1)
    assert a.dtype == torch.float32 and a.numel() == w.d
    assert torch.equal(a, b) and not torch.equal(a, c)
    g = workloads.generate(workloads.scaled(workloads.workload(1), 100_000), 0)
    assert 0.009 < g.std().item() < 0.011
    h = workloads.generate(workloads.scaled(workloads.workload(4), 200_000), 0)
    assert torch.isfinite(h).all() and h.abs().max() > 0.05      # inflated heavy tail present
