"""GPU parity of the parameter update (Alg. 1 aggregate, momentum rule of Sec. 4.2) and of the normalized-variance
diagnostic (App. J) through the C ABI against the CPU oracle.  Bars: updated parameters within 1e-6 of the fp64
result relative to the magnitudes that enter each sum; moment sums and the diagnostic within 1e-9 (fp64 on both
sides, different summation order); a step of Alg. 1 is checked with the oracle fed the same gradients, seeds and
the norms the GPU stored in its messages (norms have their own bar)."""
import numpy as np
import pytest
import torch

import oracle
from test_gpu_parity import make_vector

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def g():
    import gpu_util
    return gpu_util


def _sgd():
    from paper_1908_06077_amd import sgd
    return sgd


@pytest.mark.parametrize("d", [1, 5, 1000, 100_003, 1_048_576])
@pytest.mark.parametrize("alpha,mu,l", [(0.1, 0.9, 0.0), (0.05, 0.5, 1.0), (1.0, 0.25, 0.5), (0.3, 0.0, 1.0)])
def test_momentum_step(g, d, alpha, mu, l):
    rng = np.random.default_rng(d + int(1000 * mu))
    w = (rng.standard_normal(d) * 10.0 ** rng.uniform(-3, 2, d)).astype(np.float32)
    yl = (w + rng.standard_normal(d).astype(np.float32) * 0.1).astype(np.float32)
    grad = make_vector("mixed", d, 64, rng)
    for shift in (0, 1):                               # shift 1: pointers off the 16-byte grid, scalar route
        tw, tyl, tg = (torch.from_numpy(np.concatenate([np.zeros(shift, np.float32), a])).to(g.DEV)[shift:]
                       for a in (w, yl, grad))
        g.nuq.nuq_momentum_step(tw, tyl, tg, alpha, mu, l)
        want_w, want_yl = oracle.momentum_step(w, yl, grad, alpha, mu, l)
        a32, m32, l32 = (float(np.float32(x)) for x in (alpha, mu, l))
        mag_yl = np.abs(w) + l32 * a32 * np.abs(grad)
        mag_w = np.abs(w) + a32 * np.abs(grad) + m32 * (mag_yl + np.abs(yl))
        assert np.all(np.abs(tyl.cpu().numpy() - want_yl) <= 1e-6 * mag_yl + 1e-45)
        assert np.all(np.abs(tw.cpu().numpy() - want_w) <= 1e-6 * mag_w + 1e-45)
        np.testing.assert_array_equal(tg.cpu().numpy(), grad)


def test_momentum_step_rejects_bad_arguments(g):
    t = torch.zeros(8, dtype=torch.float32, device=g.DEV)
    for alpha, mu, l in ((0.1, 1.0, 0.0), (0.1, -0.1, 0.0), (float("nan"), 0.5, 0.0), (0.1, 0.5, float("inf"))):
        with pytest.raises(g.nuq.NuqError):
            g.nuq.nuq_momentum_step(t, t.clone(), t.clone(), alpha, mu, l)
    g.nuq.nuq_momentum_step(t[:0], t[:0], t[:0], 0.1, 0.5, 0.0)       # d = 0: nothing to do


@pytest.mark.parametrize("d,M", [(1, 4), (3, 7), (4097, 5), (300_001, 6), (600_000, 3)])
def test_moments_and_normalized_variance(g, d, M):
    rng = np.random.default_rng(d * 31 + M)
    mean = rng.standard_normal(d) * 10.0 ** rng.uniform(-2, 1, d)
    draws = (mean + rng.standard_normal((M, d)) * 0.3 * np.abs(mean)).astype(np.float32)
    for shift in (0, 1):
        acc = _sgd().NormalizedVariance(d, g.DEV)
        for m in range(M):
            row = torch.from_numpy(np.concatenate([np.zeros(shift, np.float32), draws[m]])).to(g.DEV)[shift:]
            acc.add(row)
        x = draws.astype(np.float64)
        np.testing.assert_allclose(acc.total.cpu().numpy(), x.sum(axis=0), rtol=1e-13, atol=1e-300)
        np.testing.assert_allclose(acc.total_sq.cpu().numpy(), (x * x).sum(axis=0), rtol=1e-13, atol=1e-300)
        got = acc.value()
        assert got == pytest.approx(oracle.normalized_variance(draws), rel=1e-9)
        assert acc.value() == got                        # fixed summation order: same bits again


def test_normalized_variance_rejects_bad_arguments(g):
    nuq = g.nuq
    a = torch.zeros(16, dtype=torch.float64, device=g.DEV)
    out2 = torch.zeros(2, dtype=torch.float64, device=g.DEV)
    ws = torch.empty(nuq.VARIANCE_WORKSPACE_BYTES, dtype=torch.uint8, device=g.DEV)
    with pytest.raises(nuq.NuqError):
        nuq.nuq_normalized_variance(a, a, 0, ws, out2)                       # no draws
    with pytest.raises(nuq.NuqError):
        nuq.nuq_normalized_variance(a, a, 3, ws[:1024], out2)                # workspace too small


def _messages_np(g, opt):
    return [(m.norms.cpu().numpy(), g.u64(m.bit_off), g.u32(m.words)) for m in opt.buffers.messages]


def _sum_of_magnitudes(msgs, d, n, s):
    mag = np.zeros(d)
    for norms, bo, words in msgs:
        mag += np.abs(oracle.dequantize(oracle.decode_levels(bo, words, d, n, s), n, s, norms))
    return mag


def _clear_words(opt):
    """The buffers are reused from step to step; cleared here so that the message check can also see that
    nothing is written past a message's end."""
    for m in opt.buffers.messages:
        m.words.zero_()


def _check_messages(g, grads_np, opt, t):
    """Each message is what the oracle codes from the same gradient, seed and the stored norms (bit-exact)."""
    for k, m in enumerate(opt.buffers.messages):
        g.check_norms(grads_np[k], opt.bucket, m.norms.cpu().numpy())
        g.check_message_against_oracle(grads_np[k], opt.bucket, opt.s, oracle.step_seed(opt.seed, t, opt.K, k),
                                       opt.sync_stride, m)


@pytest.mark.parametrize("d,n,s,K,S", [(50_003, 512, 3, 4, 256), (100_000, 8192, 3, 8, 256), (9_999, 1001, 5, 2, 0)])
def test_alg1_plain_step(g, d, n, s, K, S):
    rng = np.random.default_rng(d + K)
    alpha = 0.35
    w0 = rng.standard_normal(d).astype(np.float32)
    w = torch.from_numpy(w0).to(g.DEV)
    opt = _sgd().DataParallelSGD(w, K, alpha, n, s, sync_stride=S, seed=4242)
    prior = w0.astype(np.float64)
    slack = np.zeros(d)
    for t in range(3):
        grads_np = [make_vector("mixed" if k % 2 else "gauss", d, n, rng) for k in range(K)]
        _clear_words(opt)
        opt.step([torch.from_numpy(x).to(g.DEV) for x in grads_np])
        assert g.nuq.nuq_last_error_flags() == 0
        _check_messages(g, grads_np, opt, t)
        msgs = _messages_np(g, opt)
        scale32 = float(np.float32(-alpha / K))
        want = oracle.decode_average([m[0] for m in msgs], [m[1] for m in msgs], [m[2] for m in msgs], d, n, s,
                                     scale32, prior=prior)
        # Each side carries its own fp32 parameters from step to step, so a step's error bound (1e-6 of the
        # magnitudes entering its sum) adds to what the earlier steps left: where a step cancels, the
        # difference stays at the size of the cancelled terms.
        slack += 1e-6 * (abs(scale32) * _sum_of_magnitudes(msgs, d, n, s) + np.abs(prior))
        assert np.all(np.abs(w.cpu().numpy() - want) <= slack + 1e-45)
        if t == 0:
            g.check_average(msgs, d, n, s, -alpha / K, w.cpu().numpy(), prior=prior)     # per-bucket bar as well
        prior = want.astype(np.float32).astype(np.float64)      # the oracle's own fp32 parameters for the next step
    assert opt.t == 3


@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("l,d,n", [(0.0, 70_001, 2048), (1.0, 70_001, 2048), (1.0, 9_999, 1001), (0.5, 40_000, 512)])
def test_alg1_momentum_steps(g, l, d, n, fused):
    s, K, S, alpha, mu = 3, 3, 256 if n > 256 else 0, 0.2, 0.9
    rng = np.random.default_rng(17)
    w0 = rng.standard_normal(d).astype(np.float32)
    w = torch.from_numpy(w0).to(g.DEV)
    opt = _sgd().DataParallelSGD(w, K, alpha, n, s, sync_stride=S, mu=mu, l=l, seed=99, fused=fused)
    avg_gpu = torch.empty(d, dtype=torch.float32, device=g.DEV)
    ow, oyl = w0.copy(), w0.copy()
    slack_w, slack_yl = np.zeros(d), np.zeros(d)
    for t in range(3):
        grads_np = [make_vector("gauss", d, n, rng) for k in range(K)]
        _clear_words(opt)
        opt.step([torch.from_numpy(x).to(g.DEV) for x in grads_np])
        assert g.nuq.nuq_last_error_flags() == 0
        _check_messages(g, grads_np, opt, t)
        msgs = _messages_np(g, opt)
        avg = oracle.decode_average([m[0] for m in msgs], [m[1] for m in msgs], [m[2] for m in msgs], d, n, s,
                                    float(np.float32(1.0 / K)))
        g.nuq.nuq_decode_accumulate(opt.buffers.messages, d, n, s, S, 1.0 / K, False, avg_gpu)
        g.check_average(msgs, d, n, s, 1.0 / K, avg_gpu.cpu().numpy())
        if not fused:
            assert torch.equal(opt.avg, avg_gpu)
        w64, yl64 = oracle.momentum_step(ow, oyl, avg.astype(np.float32), alpha, mu, l)
        # the GPU's fp32 average may differ from the oracle's by one rounding (bar above); each side carries its own
        # fp32 state, so the bounds of the steps add up (see test_alg1_plain_step)
        mag_yl = np.abs(ow) + l * alpha * np.abs(avg)
        mag_w = np.abs(ow) + alpha * np.abs(avg) + mu * (mag_yl + np.abs(oyl))
        slack_w, slack_yl = (slack_w + 2e-6 * mag_w + mu * (slack_w + slack_yl),
                             slack_w + 2e-6 * mag_yl)          # y^l is built from w_t: it inherits w_t's bound
        assert np.all(np.abs(w.cpu().numpy() - w64) <= slack_w + 1e-45)
        assert np.all(np.abs(opt.yl.cpu().numpy() - yl64) <= slack_yl + 1e-45)
        ow, oyl = w64.astype(np.float32), yl64.astype(np.float32)


@pytest.mark.parametrize("d,n,S,shift", [(100_000, 8192, 256, 0), (70_001, 2048, 256, 0), (9_999, 1001, 0, 0),
                                         (50_003, 512, 128, 1), (3_000, 7, 0, 0), (1, 8192, 256, 0)])
def test_decode_momentum_step_equals_the_two_calls(g, d, n, S, shift):
    # one launch (decoder applies the rule) against decode + momentum kernel: the same bits in w and y^l
    nuq = g.nuq
    s, K, alpha, mu, l = 3, 4, 0.3, 0.8, 1.0
    rng = np.random.default_rng(d + n)
    vs = [torch.from_numpy(make_vector("mixed", d, n, rng)).to(g.DEV) for _ in range(K)]
    buf = _sgd().MessageBuffers(K, d, n, s, S, g.DEV)
    nuq.nuq_quantize_encode_batch(vs, n, s, list(range(K)), S, buf.messages, buf.workspace)
    w0 = torch.from_numpy(np.concatenate([np.zeros(shift, np.float32), rng.standard_normal(d).astype(np.float32)]))
    y0 = torch.from_numpy(np.concatenate([np.zeros(shift, np.float32), rng.standard_normal(d).astype(np.float32)]))
    w1, y1 = w0.to(g.DEV)[shift:], y0.to(g.DEV)[shift:]          # shift 1: off the 16-byte grid
    w2, y2 = w0.to(g.DEV)[shift:], y0.to(g.DEV)[shift:]
    avg = torch.empty(d, dtype=torch.float32, device=g.DEV)
    nuq.nuq_decode_accumulate(buf.messages, d, n, s, S, 1.0 / K, False, avg)
    nuq.nuq_momentum_step(w1, y1, avg, alpha, mu, l)
    nuq.nuq_decode_momentum_step(buf.messages, d, n, s, S, 1.0 / K, alpha, mu, l, w2, y2)
    assert nuq.nuq_last_error_flags() == 0
    assert torch.equal(w1, w2) and torch.equal(y1, y2)
    assert not torch.equal(w1, w0.to(g.DEV)[shift:]) or d == 0


def _random_update_cases(count, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(count):
        n = int(round(2.0 ** rng.uniform(0, 15)))
        if rng.random() < 0.4:
            n = int(2 ** rng.integers(6, 16))
        d = int(rng.integers(1, 12 * n + 2)) if rng.random() < 0.5 else int(rng.integers(1, 150_000))
        S = int(rng.choice([0, 64, 128, 256, 512, 1024]))
        K = int(rng.choice([1, 2, 3, 4, 5, 8]))
        cases.append((d, n, S, K, int(rng.integers(0, 2))))
    return cases


@pytest.mark.parametrize("d,n,S,K,shift", _random_update_cases(24, 99))
def test_update_modes_on_random_shapes(g, d, n, S, K, shift):
    """Every tile geometry of the decoder (small and large buckets, 2048- and 4096-coordinate tiles, one message):
    adding onto the output equals writing the sum and adding it afterwards; the momentum rule inside the decoder
    equals decode + momentum kernel.  Bit for bit: the same fp32 operations in the same order."""
    nuq = g.nuq
    s, alpha, mu, l = 3, 0.3, 0.8, 0.5
    rng = np.random.default_rng([d, n, S, K])
    vs = [torch.from_numpy(make_vector("mixed", d, n, rng)).to(g.DEV) for _ in range(K)]
    buf = _sgd().MessageBuffers(K, d, n, s, S, g.DEV)
    nuq.nuq_quantize_encode_batch(vs, n, s, list(range(K)), S, buf.messages, buf.workspace)
    w0 = torch.from_numpy(rng.standard_normal(d + 1).astype(np.float32)).to(g.DEV)
    y0 = torch.from_numpy(rng.standard_normal(d + 1).astype(np.float32)).to(g.DEV)
    cut = lambda x: x.clone()[shift:shift + d]
    total = cut(w0)
    nuq.nuq_decode_accumulate(buf.messages, d, n, s, S, -alpha / K, False, total)          # fp32(scale * sum)
    added = cut(w0)
    nuq.nuq_decode_accumulate(buf.messages, d, n, s, S, -alpha / K, True, added)
    assert torch.equal(added, total + cut(w0))
    avg = cut(w0)
    nuq.nuq_decode_accumulate(buf.messages, d, n, s, S, 1.0 / K, False, avg)
    w1, y1, w2, y2 = cut(w0), cut(y0), cut(w0), cut(y0)
    nuq.nuq_momentum_step(w1, y1, avg, alpha, mu, l)
    nuq.nuq_decode_momentum_step(buf.messages, d, n, s, S, 1.0 / K, alpha, mu, l, w2, y2)
    assert nuq.nuq_last_error_flags() == 0
    assert torch.equal(w1, w2) and torch.equal(y1, y2)


def test_step_with_momentum_replayed_from_a_hip_graph(g):
    """Encode of K workers, the momentum rule inside the decoder and a single-message decode captured into one HIP
    graph; every replay (with eager work and synchronizations in between) must leave the bits the same calls leave
    when made eagerly."""
    nuq = g.nuq
    d, n, s, S, K, alpha, mu, l = 150_000, 8192, 3, 256, 3, 0.2, 0.7, 1.0
    rng = np.random.default_rng(21)
    vs = [torch.from_numpy(make_vector("gauss", d, n, rng)).to(g.DEV) for _ in range(K)]
    seeds = [5 + k for k in range(K)]
    w0 = torch.from_numpy(rng.standard_normal(d).astype(np.float32)).to(g.DEV)

    def make():
        buf = _sgd().MessageBuffers(K, d, n, s, S, g.DEV)
        return buf, w0.clone(), w0.clone(), torch.empty(d, dtype=torch.float32, device=g.DEV)

    def step(buf, w, y, single):
        nuq.nuq_quantize_encode_batch(vs, n, s, seeds, S, buf.messages, buf.workspace)
        nuq.nuq_decode_momentum_step(buf.messages, d, n, s, S, 1.0 / K, alpha, mu, l, w, y)
        nuq.nuq_decode_accumulate(buf.messages[:1], d, n, s, S, 1.0, False, single)

    eb, ew, ey, es = make()
    gb, gw, gy, gs = make()
    step(eb, ew.clone(), ey.clone(), es)                     # warm-up outside the capture (first-call set-up)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(gb, gw, gy, gs)
    torch.cuda.current_stream().wait_stream(side)
    gw.copy_(w0)                                             # (capture does not run the kernels; start both from w0)
    gy.copy_(w0)
    for rep in range(3):
        gs.fill_(7.0)
        for m in gb.messages:
            m.words.zero_()
            m.bit_off.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        step(eb, ew, ey, es)
        torch.cuda.synchronize()
        assert torch.equal(gw, ew) and torch.equal(gy, ey) and torch.equal(gs, es), rep
        for a, b in zip(gb.messages, eb.messages):
            nw = (int(b.bit_off[-1].item()) + 31) // 32
            assert torch.equal(a.bit_off, b.bit_off) and torch.equal(a.words[:nw], b.words[:nw])
    assert nuq.nuq_last_error_flags() == 0
    assert not torch.equal(gw, w0)


def test_updates_at_benchmark_size(g):
    """Config 3 at full size, launched as bench.py --update launches it: one step of the plain rule and one of the
    momentum rule inside the decoder, compared on sampled runs of buckets that the oracle computes one by one."""
    import workloads
    nuq = g.nuq
    wl = workloads.workload(3)
    n, s, K, d, S = wl.bucket, wl.s, wl.K, wl.d, 256
    B = nuq.nuq_num_buckets(d, n)
    alpha, mu, l = 0.1, 0.9, 1.0
    vs = [workloads.generate(wl, k, g.DEV) for k in range(K)]
    gen = torch.Generator(device=g.DEV).manual_seed(5)
    w0 = torch.randn(d, device=g.DEV, generator=gen) * 0.05
    rng = np.random.default_rng(33)
    runs = sorted({0, B - 3} | {int(x) for x in rng.integers(0, B - 3, size=10)})
    for kind in ("plain", "momentum"):
        w = w0.clone()
        opt = _sgd().DataParallelSGD(w, K, alpha, n, s, sync_stride=S, mu=mu if kind == "momentum" else 0.0, l=l,
                                     seed=1234)
        seeds = [oracle.step_seed(1234, 0, K, k) for k in range(K)]
        opt.step(vs)
        assert nuq.nuq_last_error_flags() == 0
        for b_lo in runs:
            c_lo, c_hi = b_lo * n, min(d, (b_lo + 3) * n)
            if kind == "plain":
                g.check_bucket_run(vs, opt.buffers.messages, w, n, s, seeds, S, -alpha / K, b_lo, b_lo + 3, prior=w0)
                continue
            parts = g.check_bucket_run(vs, opt.buffers.messages, None, n, s, seeds, S, 1.0 / K, b_lo, b_lo + 3)
            avg = oracle.decode_average([p[0] for p in parts], [p[1] for p in parts], [p[2] for p in parts],
                                        c_hi - c_lo, n, s, float(np.float32(1.0 / K))).astype(np.float32)
            ow = w0[c_lo:c_hi].cpu().numpy()
            w64, yl64 = oracle.momentum_step(ow, ow, avg, alpha, mu, l)
            # 2e-6: the GPU's fp32 average may sit one rounding from the oracle's
            mag_yl = np.abs(ow) + l * alpha * np.abs(avg)
            mag_w = np.abs(ow) + alpha * np.abs(avg) + mu * (mag_yl + np.abs(ow))
            assert np.all(np.abs(w[c_lo:c_hi].cpu().numpy() - w64) <= 2e-6 * mag_w + 1e-45)
            assert np.all(np.abs(opt.yl[c_lo:c_hi].cpu().numpy() - yl64) <= 2e-6 * mag_yl + 1e-45)
        del opt, w
    torch.cuda.empty_cache()


def _least_squares(d, T, K, seed):
    rng = np.random.default_rng(seed)
    hdiag = rng.uniform(0.5, 2.0, d).astype(np.float32)
    wstar = rng.standard_normal(d).astype(np.float32)
    noise = (0.01 * rng.standard_normal((T, K, d))).astype(np.float32)
    return hdiag, wstar, noise


@pytest.mark.parametrize("mu,l", [(0.0, 0.0), (0.5, 1.0)])
def test_alg1_short_trajectory_matches_oracle_loop(g, mu, l):
    # Both sides run their own loop from the same start; the gradient is elementwise fp32 arithmetic (one rounding
    # per operation on both sides).  At this size the two fp32 norms agree and no draw sits close enough to its
    # threshold for the last-bit differences of w to flip it, so the trajectories stay within accumulated rounding.
    d, n, s, K, T, alpha = 2048, 256, 3, 4, 8, 0.2
    hdiag, wstar, noise = _least_squares(d, T, K, 5)
    want = oracle.data_parallel_sgd(np.zeros(d, np.float32), lambda w, t, k: hdiag * (w - wstar) + noise[t, k],
                                    K, T, alpha, n, s, 256, seed0=31, mu=mu, l=l)
    w = torch.zeros(d, dtype=torch.float32, device=g.DEV)
    th, tstar, tnoise = (torch.from_numpy(a).to(g.DEV) for a in (hdiag, wstar, noise))
    opt = _sgd().DataParallelSGD(w, K, alpha, n, s, sync_stride=256, mu=mu, l=l, seed=31)
    for t in range(T):
        opt.step([th * (w - tstar) + tnoise[t, k] for k in range(K)])
    assert g.nuq.nuq_last_error_flags() == 0
    np.testing.assert_allclose(w.cpu().numpy(), want, rtol=0, atol=2e-5 * float(np.abs(wstar).max()))


def test_alg1_converges_on_least_squares(g):
    d, n, s, K, T, alpha = 65_536, 8192, 3, 4, 300, 0.2
    hdiag, wstar, noise = _least_squares(d, 1, K, 6)
    th, tstar, tnoise = (torch.from_numpy(a).to(g.DEV) for a in (hdiag, wstar, noise[0]))
    loss = lambda x: 0.5 * float((th.double() * (x.double() - tstar.double()) ** 2).sum())
    w = torch.zeros(d, dtype=torch.float32, device=g.DEV)
    wf = torch.zeros_like(w)
    opt = _sgd().DataParallelSGD(w, K, alpha, n, s, seed=8)
    start = loss(w)
    gen = torch.Generator(device=g.DEV).manual_seed(3)
    for t in range(T):
        eps = [0.01 * torch.randn(d, device=g.DEV, generator=gen) for _ in range(K)]
        opt.step([th * (w - tstar) + e for e in eps])
        wf -= alpha * torch.stack([th * (wf - tstar) + e for e in eps]).mean(dim=0)
    assert g.nuq.nuq_last_error_flags() == 0
    assert loss(w) < 1e-3 * start
    assert loss(wf) < loss(w) < 200 * loss(wf)


def test_normalized_variance_of_quantized_estimates(g):
    # M draws of Q(v) through encode + decode; the diagnostic must equal the oracle's over its own draws (same seeds,
    # stored norms: identical draws) and sit near the exact value of Def. 1's two-point law.
    d, n, s, M = 16_384, 8192, 3, 64
    rng = np.random.default_rng(12)
    v = make_vector("gauss", d, n, rng)
    tv = torch.from_numpy(v).to(g.DEV)
    est = _sgd().QuantizedEstimate(d, n, s, g.DEV)
    acc = _sgd().NormalizedVariance(d, g.DEV)
    out = torch.empty(d, dtype=torch.float32, device=g.DEV)
    for m in range(M):
        acc.add(est(tv, 500 + m, out))
    norms = est.buffers.messages[0].norms.cpu().numpy()
    g.check_norms(v, n, norms)
    draws = np.stack([oracle.dequantize(oracle.quantize(v, n, s, 500 + m, norms), n, s, norms) for m in range(M)])
    got = acc.value()
    assert got == pytest.approx(oracle.normalized_variance(draws.astype(np.float32)), rel=1e-6)
    lev = np.array([float(x) for x in oracle.levels(s)])
    r = np.abs(v.astype(np.float64)) / np.repeat(norms.astype(np.float64), n)[:d]
    j = np.clip(np.searchsorted(lev, r, side="right") - 1, 0, s)
    var = (np.repeat(norms.astype(np.float64), n)[:d] ** 2 * (lev[j + 1] - r) * (r - lev[j])).sum()
    exact = var / (var + float((v.astype(np.float64) ** 2).sum()))
    assert got * M / (M - 1) == pytest.approx(exact, rel=0.03)
