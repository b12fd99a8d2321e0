"""bmgd_eval_loss against the fp64 oracle's loss, for the three models, and its use along a run: the global loss
of a mini-batch run with a small learning rate goes down from iteration to iteration."""
import numpy as np
import pytest

import workloads as wl
from gpu_util import rel_l2

pytestmark = pytest.mark.gpu


def _ctx_with_theta(w, theta):
    import paper_2312_08728_amd as B
    ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T, model=w.model, n_classes=w.C)
    ctx.set_theta(theta)
    return ctx


@pytest.mark.parametrize("model,p,rows", [(wl.LINEAR, 10, 1), (wl.LINEAR, 100, 5000), (wl.LOGISTIC, 200, 7777),
                                          (wl.LOGISTIC, 4096, 300), (wl.LINEAR, 37, 70_001)])
def test_glm_loss_matches_oracle(model, p, rows):
    import torch
    from oracle import bmgd as O
    base = wl.CONFIGS["cfg3" if model == wl.LOGISTIC else "cfg2"]
    w = base.scaled(name="case", model=model, N=rows, p=p, N0=max(rows, 2), n=max(min(rows, 100), 1), T=1, R=1, x_cov="identity")
    X, y = wl.dataset(w)
    theta = (np.random.default_rng(1).standard_normal(p) / np.sqrt(p)).astype(np.float32)
    want = O.loss(model, X.astype(np.float64), y.astype(np.float64), theta.astype(np.float64))
    ctx = _ctx_with_theta(w, theta)
    got = ctx.eval_loss(torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda(), rows)
    ctx.close()
    assert abs(got - want) <= 2e-5 * abs(want)


def test_softmax_loss_matches_oracle():
    import torch
    from oracle import bmgd as O
    w = wl.CONFIGS["cfg5"].scaled(name="case", N=3000, p=200, C=130, N0=1500, n=256, T=1, R=1)
    X, y = wl.dataset(w)
    W = (np.random.default_rng(2).standard_normal((w.p, w.C)) * 0.05).astype(np.float32)
    want = O.loss(w.model, O.to_f64(X), y, W.astype(np.float64))
    ctx = _ctx_with_theta(w, W)
    got = ctx.eval_loss(torch.from_numpy(X.view(np.int16)).cuda(), torch.from_numpy(y).cuda(), 3000)
    ctx.close()
    assert abs(got - want) <= 2e-3 * abs(want)                 # logits from the bf16 copy of W


def test_global_loss_goes_down_over_iterations():
    import torch
    import paper_2312_08728_amd as B
    w = wl.CONFIGS["cfg3"].scaled(name="case", N=40_000, p=50, N0=10_000, n=500, T=2, R=4, alpha=0.05)
    X, y = wl.dataset(w)
    xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T, model=w.model)
    s = torch.cuda.Stream()
    losses = [ctx.eval_loss(xd, yd, w.N)]
    for r in range(w.R):
        for k in range(4):
            ctx.run_device_buffer(xd[k * w.N0:(k + 1) * w.N0], yd[k * w.N0:(k + 1) * w.N0], w.N0, s)
        losses.append(ctx.eval_loss(xd, yd, w.N, s))
    ctx.close()
    assert abs(losses[0] - np.log(2.0)) < 1e-6                  # theta = 0: every row costs log 2
    assert all(b < a for a, b in zip(losses, losses[1:])), losses
