"""Running average of estimates on the device (buffered weight averaging, Section 4.4) against the oracle's."""
import numpy as np
import pytest

import workloads as wl
from gpu_util import rel_l2

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("model,p,n,chain", [(wl.LINEAR, 40, 250, 3), (wl.LINEAR, 40, 250, 1), (wl.LOGISTIC, 200, 512, 1),
                                             (wl.LINEAR, 2048, 600, 1), (wl.LOGISTIC, 40, 250, 2)])
def test_glm_average_every_two_buffers(model, p, n, chain):
    import torch
    import paper_2312_08728_amd as B
    from oracle import bmgd as O
    base = wl.CONFIGS["cfg3" if model == wl.LOGISTIC else "cfg2"]
    w = base.scaled(name="case", model=model, N=12_000, p=p, N0=2000, n=n, T=2, R=1, x_cov="identity",
                    alpha=(0.5 / (p + 10)) if model == wl.LINEAR else 0.2)
    X, y = wl.dataset(w)
    ref = O.BMGD(w.model, w.p, w.n, w.alpha, w.T)
    ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T, model=w.model, chain=chain)
    with pytest.raises(B.BmgdError) as e:
        ctx.get_swa()
    assert e.value.code == B.BMGD_ESTATE
    xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    s = torch.cuda.Stream()
    for k in range(6):
        ref.run_buffer(X[k * 2000:(k + 1) * 2000], y[k * 2000:(k + 1) * 2000])
        ctx.run_device_buffer(xd[k * 2000:(k + 1) * 2000], yd[k * 2000:(k + 1) * 2000], 2000, s)
        if k % 2 == 1:
            ref.swa_update()
            ctx.swa_update(s)                       # asynchronous: the next run is enqueued right behind it
    avg, count = ctx.get_swa()
    theta = ctx.get_theta()
    assert count == 3
    assert rel_l2(avg, ref.swa) <= 1e-4 and rel_l2(theta, ref.theta) <= 1e-4
    assert rel_l2(avg, theta) > 1e-3                # the average is not just the last estimate
    # a new average after a reset: one snapshot equals the estimate, bit for bit
    ctx.swa_reset()
    ctx.swa_update(s)
    avg, count = ctx.get_swa()
    assert count == 1 and np.array_equal(avg, theta)
    ctx.close()


def test_softmax_average():
    import torch
    import paper_2312_08728_amd as B
    from oracle import bmgd as O
    w = wl.CONFIGS["cfg5"].scaled(name="case", N=3000, p=128, C=40, N0=1000, n=256, T=1, R=1)
    X, y = wl.dataset(w)
    ref = O.BMGD(w.model, w.p, w.n, w.alpha, w.T, C=w.C)
    ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T, model=w.model, n_classes=w.C)
    xd, yd = torch.from_numpy(X.view(np.int16)).cuda(), torch.from_numpy(y).cuda()
    s = torch.cuda.Stream()
    for k in range(3):
        ref.run_buffer(X[k * 1000:(k + 1) * 1000], y[k * 1000:(k + 1) * 1000])
        ctx.run_device_buffer(xd[k * 1000:(k + 1) * 1000], yd[k * 1000:(k + 1) * 1000], 1000, s)
        ref.swa_update()
        ctx.swa_update(s)
    avg, count = ctx.get_swa()
    ctx.close()
    assert count == 3 and avg.shape == (128, 40)
    assert rel_l2(avg, ref.swa) <= 2e-3
