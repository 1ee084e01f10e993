"""Alg. 1 as a torch optimizer over a real module (paper_1908_06077_amd.optim.NUQSGD) against the oracle's loop
(oracle.data_parallel_sgd) on a tiny MLP with synthetic data, and the diagnostic of App. J on its gradients.

Both sides run their own trajectory from the same initial parameters.  The gradients are computed by autograd on
each side's own parameters (GPU here, CPU for the oracle): they agree to fp32 rounding, and at this size no draw
sits so close to its threshold that such a difference flips it, so the trajectories stay within accumulated
rounding (the bar below); a flipped draw would move a coordinate by a whole level step, far outside it."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu

DEV = torch.device("cuda:0")


def make_model():
    torch.manual_seed(7)
    return torch.nn.Sequential(torch.nn.Linear(12, 24), torch.nn.Tanh(), torch.nn.Linear(24, 24), torch.nn.Tanh(),
                               torch.nn.Linear(24, 3))


def make_data(K, T, batch=32):
    g = torch.Generator().manual_seed(11)
    x = torch.randn(T, K, batch, 12, generator=g)
    y = torch.tanh(x[..., :3] * 2.0 - x[..., 3:6]) + 0.05 * torch.randn(T, K, batch, 3, generator=g)
    return x, y


def flat(params):
    return torch.cat([p.detach().reshape(-1) for p in params])


def oracle_trajectory(K, T, lr, bucket, s, S, seed, mu, l, x, y):
    model = make_model()
    params = list(model.parameters())
    sizes = [p.numel() for p in params]

    def grad_fn(w, t, k):
        with torch.no_grad():
            for p, chunk in zip(params, torch.from_numpy(np.array(w, dtype=np.float32)).split(sizes)):
                p.copy_(chunk.view_as(p))
        model.zero_grad()
        torch.nn.functional.mse_loss(model(x[t, k]), y[t, k]).backward()
        return flat([p.grad for p in params]).numpy()
    w0 = flat(params).numpy()
    return oracle.data_parallel_sgd(w0, grad_fn, K, T, lr, bucket, s, S, seed0=seed, mu=mu, l=l)


@pytest.mark.parametrize("mu,l", [(0.0, 0.0), (0.9, 0.0), (0.5, 1.0)])
def test_optimizer_over_a_module_follows_the_oracle_loop(mu, l):
    import paper_1908_06077_amd as nuq
    from paper_1908_06077_amd.optim import NUQSGD
    K, T, lr, bucket, s, S, seed = 4, 6, 0.05, 256, 3, 64, 17
    x, y = make_data(K, T)
    want = oracle_trajectory(K, T, lr, bucket, s, S, seed, mu, l, x, y)

    model = make_model().to(DEV)
    w0 = flat(model.parameters()).cpu().numpy()
    opt = NUQSGD(model.parameters(), K=K, lr=lr, bucket=bucket, s=s, sync_stride=S, momentum=mu, nesterov_l=l, seed=seed)
    assert opt.d == want.size and all(p.data_ptr() >= opt.flat_w.data_ptr() for p in model.parameters())
    xd, yd = x.to(DEV), y.to(DEV)
    losses = []
    for t in range(T):
        for k in range(K):
            with opt.worker(k):
                loss = torch.nn.functional.mse_loss(model(xd[t, k]), yd[t, k])
                loss.backward()
            losses.append(float(loss.detach()))
        opt.step()
    assert nuq.nuq_last_error_flags() == 0
    got = flat(model.parameters()).cpu().numpy()
    assert np.array_equal(got, opt.flat_w.cpu().numpy())               # the module's parameters are the flat vector
    moved = np.abs(want - w0).max()
    assert moved > 1e-3                                                 # the steps did something
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-5 * max(1.0, float(np.abs(want).max())))
    assert np.mean(losses[-K:]) < np.mean(losses[:K])                  # and the loss went down


def test_gradient_variance_diagnostic_on_module_gradients():
    """App. J: the normalized variance of Q(g) for the module's gradient, against the oracle's formula over the
    oracle's own draws with the same seeds (fed the library's norms), and against the exact value of Def. 1's
    two-point law."""
    import paper_1908_06077_amd as nuq
    from paper_1908_06077_amd.optim import NUQSGD
    K, bucket, s, M = 2, 256, 3, 64
    x, y = make_data(K, 1)
    model = make_model().to(DEV)
    opt = NUQSGD(model.parameters(), K=K, lr=0.1, bucket=bucket, s=s, sync_stride=64)
    for k in range(K):
        with opt.worker(k):
            torch.nn.functional.mse_loss(model(x[0, k].to(DEV)), y[0, k].to(DEV)).backward()
    got = opt.gradient_variance(k=1, draws=M, seed=900)
    assert nuq.nuq_last_error_flags() == 0
    g = opt.flat_g[1].cpu().numpy()
    assert np.abs(g).max() > 0
    norms = opt._estimate.buffers.messages[0].norms.cpu().numpy()
    want_norms = oracle.bucket_norms(g, bucket)
    assert np.all(np.abs(norms - want_norms) <= 1e-6 * want_norms)
    draws = np.stack([oracle.dequantize(oracle.quantize(g, bucket, s, 900 + m, norms), bucket, s, norms)
                      for m in range(M)])
    assert got == pytest.approx(oracle.normalized_variance(draws.astype(np.float32)), rel=1e-6)
    lev = np.array([float(v) for v in oracle.levels(s)])
    nrm = np.repeat(norms.astype(np.float64), bucket)[: g.size]
    r = np.abs(g.astype(np.float64)) / nrm
    j = np.clip(np.searchsorted(lev, r, side="right") - 1, 0, s)
    var = (nrm ** 2 * (lev[j + 1] - r) * (r - lev[j])).sum()
    exact = var / (var + float((g.astype(np.float64) ** 2).sum()))
    assert got * M / (M - 1) == pytest.approx(exact, rel=0.1)
