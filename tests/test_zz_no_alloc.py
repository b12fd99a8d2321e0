"""bmgd_eval_loss_static (the entry point that allocates nothing: partial sums in a static device array, result left
on the device) against bmgd_eval_loss, through the C ABI, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


def _case(model, p, rows, seed):
    base = wl.CONFIGS["cfg3" if model == wl.LOGISTIC else "cfg2"]
    w = base.scaled(name="case", model=model, N=rows, p=p, N0=max(rows, 2), n=max(min(rows, 100), 1), T=1, R=1,
                    x_cov="identity", seed=seed)
    X, y = wl.dataset(w)
    theta = (np.random.default_rng(seed).standard_normal(p) / np.sqrt(p)).astype(np.float32)
    return w, X, y, theta


def test_static_scratch_entry_point_equals_eval_loss_on_two_calls_in_a_row():
    import torch
    import paper_2312_08728_amd as B
    from oracle import bmgd as O
    out = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda")
    s = torch.cuda.Stream()
    # the second call is smaller in rows and in p, so partial sums left by the first lie beyond what it may read
    for i, (model, p, rows, seed) in enumerate(((wl.LINEAR, 300, 70_001, 5), (wl.LOGISTIC, 37, 333, 6), (wl.LINEAR, 4096, 9, 7))):
        w, X, y, theta = _case(model, p, rows, seed)
        xd, yd, td = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda(), torch.from_numpy(theta).cuda()
        ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T, model=w.model)
        try:
            ctx.set_theta(theta)
            want = ctx.eval_loss(xd, yd, rows)
        finally:
            ctx.close()
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        rc = B.bmgd_eval_loss_static(model, xd, yd, td, rows, p, s, out)
        assert rc == B.BMGD_OK, B.bmgd_last_error(None)
        s.synchronize()
        if i > 0:           # (the first use of a new stream makes the runtime itself set up a queue)
            assert torch.cuda.mem_get_info()[0] == free_before       # no device memory was taken
        got = float(out.cpu()[0])
        assert got == want, (model, p, rows, got, want)               # same sums in the same order
        ref = O.loss(model, X.astype(np.float64), y.astype(np.float64), theta.astype(np.float64))
        assert abs(got - ref) <= 2e-5 * abs(ref)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import torch
    import paper_2312_08728_amd as B
    x, y, t = torch.zeros(8, 4, device="cuda"), torch.zeros(8, device="cuda"), torch.zeros(4, device="cuda")
    out = torch.zeros(1, dtype=torch.float64, device="cuda")
    assert B.bmgd_eval_loss_static(B.BMGD_SOFTMAX, x, y, t, 8, 4, None, out) == B.BMGD_EINVAL
    assert "static array" in B.bmgd_last_error(None)
    assert B.bmgd_eval_loss_static(B.BMGD_LINEAR, x, y, t, 8, 4097, None, out) == B.BMGD_EINVAL
    assert B.bmgd_eval_loss_static(B.BMGD_LINEAR, x, y, t, 1 << 30, 4, None, out) == B.BMGD_EINVAL
    assert B.bmgd_eval_loss_static(B.BMGD_LINEAR, x, y, t, 0, 4, None, out) == B.BMGD_EINVAL
    assert B.bmgd_eval_loss_static(B.BMGD_LINEAR, x, None, t, 8, 4, None, out) == B.BMGD_EINVAL
    assert B.bmgd_eval_loss_static(B.BMGD_LINEAR, x, y, t, 8, 4, None, out) == B.BMGD_OK
    torch.cuda.synchronize()
    assert float(out.cpu()[0]) == 0.0
