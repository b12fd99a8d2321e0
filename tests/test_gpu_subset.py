"""bmgd_set_row_subset: a run restricted to chosen rows of its buffer (undersampling of the negative instances of
each buffer, Section 4.2) equals the oracle run on those rows in that order."""
import numpy as np
import pytest

import workloads as wl
from gpu_util import rel_l2

pytestmark = pytest.mark.gpu


def _balanced_subset(y, rng):
    """All positives of the buffer and as many negatives drawn without replacement, in row order."""
    pos = np.flatnonzero(y > 0.5)
    neg = np.flatnonzero(y <= 0.5)
    keep = rng.choice(neg, size=min(len(pos), len(neg)), replace=False)
    return np.sort(np.concatenate([pos, keep])).astype(np.int32)


@pytest.mark.parametrize("chain,resident", [(1, True), (2, True), (1, False)])
def test_undersampled_logistic_regression(chain, resident):
    import torch
    import paper_2312_08728_amd as B
    from oracle import bmgd as O
    w = wl.CONFIGS["cfg3"].scaled(name="case", N=24_000, p=40, N0=8000, n=256, T=2, R=2, alpha=0.2)
    X, y = wl.dataset(w)
    # make positives rare: keep the label only where a second coin agrees
    rng = np.random.default_rng(1)
    y = (y * (rng.random(y.shape) < 0.08)).astype(np.float32)
    ref = O.BMGD(w.model, w.p, w.n, w.alpha, w.T)
    ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T, model=w.model, chain=chain)
    xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    xp, yp = torch.from_numpy(X).pin_memory(), torch.from_numpy(y).pin_memory()
    cs, ks = torch.cuda.Stream(), torch.cuda.Stream()
    keep_alive, total = [], 0
    for r in range(2):
        for k in range(3):
            lo, hi = k * 8000, (k + 1) * 8000
            sel = _balanced_subset(y[lo:hi], rng)
            total += len(sel)
            ref.run_buffer(X[lo:hi][sel], y[lo:hi][sel])
            sd = torch.from_numpy(sel).cuda()
            keep_alive.append(sd)
            ctx.set_row_subset(sd, len(sel))
            if resident:
                ctx.run_device_buffer(xd[lo:hi], yd[lo:hi], 8000, ks)
            else:
                ctx.load_buffer_async(xp[lo:hi], yp[lo:hi], 8000, cs)
                ctx.run_buffer(ks)
    got = ctx.get_theta()
    st = ctx.stats()
    ctx.close()
    assert st.sample_gradients == 2 * total and total < 0.25 * 2 * 24_000
    assert rel_l2(got, ref.theta) <= 1e-4


def test_subset_in_the_moment_form_with_repeats_and_one_shot():
    import torch
    import paper_2312_08728_amd as B
    from oracle import bmgd as O
    w = wl.CONFIGS["cfg2"].scaled(name="case", N=6000, p=24, N0=3000, n=200, T=3, R=1, alpha=0.02)
    X, y = wl.dataset(w)
    rng = np.random.default_rng(2)
    sel = rng.integers(0, 3000, size=1500).astype(np.int32)          # with repeats, unsorted
    ref = O.BMGD(w.model, w.p, w.n, w.alpha, w.T)
    ref.run_buffer(X[:3000][sel], y[:3000][sel])
    ref.run_buffer(X[3000:], y[3000:])                               # the subset held for one run only
    ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T, chain=3)
    xd, yd, sd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda(), torch.from_numpy(sel).cuda()
    s = torch.cuda.Stream()
    ctx.set_row_subset(sd, 1500)
    ctx.run_device_buffer(xd[:3000], yd[:3000], 3000, s)
    ctx.run_device_buffer(xd[3000:], yd[3000:], 3000, s)
    got = ctx.get_theta()
    st = ctx.stats()
    assert st.steps == 3 * 8 + 3 * 15 and st.chain == 3
    assert rel_l2(got, ref.theta) <= 1e-4
    # errors: too many entries for the buffer; an index outside the buffer is caught on the device
    ctx.set_row_subset(sd, 1500)
    with pytest.raises(B.BmgdError) as e:
        ctx.run_device_buffer(xd[:1000], yd[:1000], 1000, s)
    assert e.value.code == B.BMGD_EINVAL
    ctx.set_row_subset(sd, 0)                                        # cancelled
    bad = sel.copy(); bad[7] = 3000
    bd = torch.from_numpy(bad).cuda()
    ctx.set_row_subset(bd, 1500)
    ctx.run_device_buffer(xd[:3000], yd[:3000], 3000, s)
    with pytest.raises(B.BmgdError) as e:
        ctx.get_theta()
    assert e.value.code == B.BMGD_EINVAL
    # theta is not valid after that run: further runs are refused until it has been set again, then all is as before
    with pytest.raises(B.BmgdError) as e:
        ctx.run_device_buffer(xd[:3000], yd[:3000], 3000, s)
    assert e.value.code == B.BMGD_ESTATE
    ctx.set_theta(np.zeros(w.p, dtype=np.float32))
    ctx.run_device_buffer(xd[:3000], yd[:3000], 3000, s)
    ctx.sync()
    assert B.bmgd_set_row_subset(ctx.h, None, 5) == B.BMGD_EINVAL
    assert B.bmgd_set_row_subset(ctx.h, sd, 3001) == B.BMGD_EINVAL
    ctx.close()
