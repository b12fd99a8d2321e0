"""cache_moments: with fixed partitions (Section 3.1.1) the moment matrices of every buffer index are formed once; later
iterations are the chain of eq. (3.1) alone.  Same estimate, bit for bit, as without the cache, and the oracle's."""
import numpy as np
import pytest

import workloads as wl
from gpu_util import rel_l2

pytestmark = pytest.mark.gpu


def _data(N=9000, p=24, N0=3000, n=200, T=2):
    w = wl.CONFIGS["cfg2"].scaled(name="case", N=N, p=p, N0=N0, n=n, T=T, R=4, alpha=0.02)
    X, y = wl.dataset(w)
    return w, X, y


@pytest.mark.parametrize("optimizer", [0, 3])
def test_cached_iterations_equal_uncached_ones_and_the_oracle(optimizer):
    import torch
    import paper_2312_08728_amd as B
    from oracle import bmgd as O
    w, X, y = _data()
    xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    s = torch.cuda.Stream()
    out = {}
    for cached in (False, True):
        ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T, reshuffle=1, n_buffers=3, chain=3, cache_moments=cached, optimizer=optimizer)
        for r in range(4):
            for k in range(3):
                if cached and r >= 2:
                    ctx.run_cached_buffer(s)                        # no rows at all
                else:
                    ctx.run_device_buffer(xd[k * 3000:(k + 1) * 3000], yd[k * 3000:(k + 1) * 3000], 3000, s)
        out[cached] = (ctx.get_theta(), ctx.stats())
        ctx.close()
    assert np.array_equal(out[False][0], out[True][0])
    assert out[False][1].prep_launches == 12 and out[True][1].prep_launches == 3
    assert out[True][1].steps == out[False][1].steps == 4 * 3 * 2 * 15
    ref = O.BMGD(w.model, w.p, w.n, w.alpha, w.T, reshuffle=O.FIXED, K_fixed=3)
    if optimizer:
        ref.set_optimizer(O.ADAM)
    for r in range(4):
        for k in range(3):
            ref.run_buffer(X[k * 3000:(k + 1) * 3000], y[k * 3000:(k + 1) * 3000])
    assert rel_l2(out[True][0], ref.theta) <= (5e-4 if optimizer else 1e-4)


def test_cache_through_the_loader_ragged_buffer_clear_and_errors():
    import torch
    import paper_2312_08728_amd as B
    w, X, y = _data(N=7000)                      # buffers of 3000, 3000, 1000 rows
    xp, yp = torch.from_numpy(X).pin_memory(), torch.from_numpy(y).pin_memory()
    cs, ks = torch.cuda.Stream(), torch.cuda.Stream()
    res = {}
    for cached in (False, True):
        ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T, reshuffle=1, n_buffers=3, cache_moments=cached)
        if cached:
            with pytest.raises(B.BmgdError) as e:
                ctx.run_cached_buffer(ks)                            # nothing cached yet
            assert e.value.code == B.BMGD_ESTATE
        for r in range(3):
            for k in range(3):
                lo, hi = k * 3000, min((k + 1) * 3000, 7000)
                ctx.load_buffer_async(xp[lo:hi], yp[lo:hi], hi - lo, cs)
                ctx.run_buffer(ks)
        if cached:
            ctx.clear_moment_cache()
            with pytest.raises(B.BmgdError):
                ctx.run_cached_buffer(ks)
        for k in range(3):                                           # refilled after the clear
            lo, hi = k * 3000, min((k + 1) * 3000, 7000)
            ctx.load_buffer_async(xp[lo:hi], yp[lo:hi], hi - lo, cs)
            ctx.run_buffer(ks)
        res[cached] = (ctx.get_theta(), ctx.stats().prep_launches)
        ctx.close()
    assert np.array_equal(res[False][0], res[True][0])
    assert res == res and res[False][1] == 12 and res[True][1] == 6
    # configurations the cache does not apply to
    for kw in (dict(reshuffle=0, n_buffers=3), dict(reshuffle=1, n_buffers=0), dict(reshuffle=1, n_buffers=3, chain=1),
               dict(reshuffle=1, n_buffers=3, model=wl.LOGISTIC)):
        with pytest.raises(B.BmgdError) as e:
            B.Context(w.p, w.N0, w.n, w.alpha, w.T, cache_moments=True, **kw)
        assert e.value.code == B.BMGD_EINVAL
    ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T)
    with pytest.raises(B.BmgdError) as e:
        ctx.run_cached_buffer(ks)
    assert e.value.code == B.BMGD_ESTATE
    ctx.close()
