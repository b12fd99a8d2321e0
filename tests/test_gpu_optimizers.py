"""Buffered momentum / NAG / Adam (Section 4.3) on the GPU against the fp64 oracle: every chain mode of the GLM paths
(row form with redundant and sliced reduction, moment form, step per launch) and the softmax path.  State is carried
across passes, launches and buffers."""
import numpy as np
import pytest

import workloads as wl
from gpu_util import rel_l2

pytestmark = pytest.mark.gpu

KINDS = [1, 2, 3]           # BMGD_OPT_MOMENTUM, BMGD_OPT_NAG, BMGD_OPT_ADAM


def _run_both(w, X, y, kind, chain, rate, n_workgroups=0, buffers=3, reset_after=None):
    import torch
    import paper_2312_08728_amd as B
    from oracle import bmgd as O
    ref = O.BMGD(w.model, w.p, w.n, rate, w.T, C=w.C)
    ref.set_optimizer(kind, momentum=0.8, beta1=0.9, beta2=0.99, eps=1e-6)
    ctx = B.Context(w.p, w.N0, w.n, rate, w.T, model=w.model, n_classes=w.C, chain=chain, n_workgroups=n_workgroups,
                    optimizer=kind, momentum=0.8, beta1=0.9, beta2=0.99, eps=1e-6)
    Xv = X.view(np.int16) if X.dtype == np.uint16 else X
    xd, yd = torch.from_numpy(Xv).cuda(), torch.from_numpy(y).cuda()
    s = torch.cuda.Stream()
    for k in range(buffers):
        lo, hi = k * w.N0, (k + 1) * w.N0
        ref.run_buffer(X[lo:hi], y[lo:hi])
        ctx.run_device_buffer(xd[lo:hi], yd[lo:hi], w.N0, s)
        if reset_after == k:
            ref.set_optimizer(kind, momentum=0.8, beta1=0.9, beta2=0.99, eps=1e-6)
            ctx.reset_optimizer()
    got = ctx.get_theta()
    st = ctx.stats()
    ctx.close()
    return got.reshape(ref.theta.shape), ref.theta, st


# (model, p, n, chain, workgroups): row form with one workgroup, redundant reduction, sliced reduction (narrow and wide
# rows), step per launch; moment form for two thread layouts
CASES = [(wl.LOGISTIC, 40, 250, 1, 1), (wl.LOGISTIC, 40, 250, 1, 8), (wl.LOGISTIC, 200, 512, 1, 64),
         (wl.LINEAR, 1024, 500, 1, 0), (wl.LINEAR, 2304, 500, 1, 0), (wl.LOGISTIC, 4096, 700, 1, 40),
         (wl.LOGISTIC, 40, 250, 2, 16), (wl.LINEAR, 40, 250, 3, 0), (wl.LINEAR, 100, 300, 3, 0)]


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("model,p,n,chain,G", CASES)
def test_glm_optimizers(kind, model, p, n, chain, G):
    base = wl.CONFIGS["cfg3" if model == wl.LOGISTIC else "cfg2"]
    w = base.scaled(name="case", model=model, N=6000, p=p, N0=2000, n=n, T=5, R=1, x_cov="identity")
    X, y = wl.dataset(w)
    if kind == 3:
        rate = 0.01                                     # Adam moves every coordinate by about the rate per update
    else:
        rate = (0.1 / (p + 10)) if model == wl.LINEAR else 0.05
    got, want, st = _run_both(w, X, y, kind, chain, rate, n_workgroups=G, reset_after=1 if p == 40 and chain == 1 else None)
    assert st.steps == 3 * 5 * (-(-2000 // n))
    assert rel_l2(got, want) <= 1e-4, (st.n_workgroups, st.chain)


@pytest.mark.parametrize("kind", KINDS)
def test_softmax_optimizers(kind):
    w = wl.CONFIGS["cfg5"].scaled(name="case", N=2000, p=128, C=40, N0=1000, n=256, T=2, R=1)
    X, y = wl.dataset(w)
    got, want, _ = _run_both(w, X, y, kind, 0, 0.002 if kind == 3 else 0.02, buffers=2)
    # bf16 operands as in the plain softmax path; Adam's normalised steps turn the bf16 rounding of the gradient
    # into a relative error of the same order in every coordinate
    assert rel_l2(got, want) <= (5e-3 if kind == 3 else 2e-3)


def test_invalid_optimizer_settings():
    import paper_2312_08728_amd as B
    for kw in (dict(optimizer=7), dict(optimizer=1, momentum=1.0), dict(optimizer=3, beta1=1.0), dict(optimizer=3, eps=-1.0)):
        cfg = B.bmgd_default_config()
        cfg.p, cfg.buffer_n, cfg.batch_n, cfg.lr, cfg.passes = 8, 100, 10, 0.1, 1
        for k, v in kw.items():
            setattr(cfg, k, v)
        rc, h = B.bmgd_create_ex(cfg)
        assert rc == B.BMGD_EINVAL and h is None, kw
