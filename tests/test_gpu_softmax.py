"""Parity of the MFMA softmax path (bf16 predictors, bf16 copy of W for the logits, bf16 residual, fp32 master
weights and accumulation) with the fp64 oracle: relative L2 error of the final W <= 2e-3."""
import numpy as np
import pytest

import workloads as wl
from gpu_util import gpu_run, oracle_run, rel_l2

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _case(N, p, C, N0, n, T=2, R=1, alpha=0.05):
    return wl.CONFIGS["cfg5"].scaled(name="case", N=N, p=p, C=C, N0=N0, n=n, T=T, R=R, alpha=alpha)


SHAPES = [
    # N, p, C, N0, n
    (900, 64, 10, 500, 128),          # one class tile, ragged batches, second buffer shorter
    (1200, 200, 130, 600, 100),       # p not a multiple of the K tile, two class tiles, n below one row tile
    (3000, 96, 2, 1500, 256),         # two classes
    (5000, 512, 1000, 2500, 1024),    # class count of the target workload, split-K logits
    (2100, 1024, 300, 2100, 700),     # single buffer, n not a multiple of 32
]


@pytest.mark.parametrize("N,p,C,N0,n", SHAPES)
def test_softmax_shapes(N, p, C, N0, n):
    w = _case(N, p, C, N0, n)
    X, y = wl.dataset(w)
    want = oracle_run(w, X, y)
    got, st = gpu_run(w, X, y)
    assert got.shape == (p, C) and st.steps == w.steps
    assert np.isfinite(got).all()
    assert rel_l2(got, want) <= TOL
    # every class is parameterised and each update removes and adds the same x-weighted mass: the class-sum of W stays 0
    assert np.abs(got.sum(axis=1)).max() <= 1e-3 * np.abs(got).max() * np.sqrt(C)


def test_softmax_resident_equals_loader_and_initial_value():
    w = _case(2000, 128, 40, 1000, 256, T=2, R=2)
    X, y = wl.dataset(w)
    w0 = (np.random.default_rng(0).standard_normal((w.p, w.C)) * 0.05).astype(np.float32)
    want = oracle_run(w, X, y, theta0=w0)
    a, _ = gpu_run(w, X, y, theta0=w0)
    b, _ = gpu_run(w, X, y, theta0=w0, resident=True)
    assert np.array_equal(a, b)
    assert rel_l2(a, want) <= TOL


def test_softmax_argument_checks():
    import paper_2312_08728_amd as B
    for kw in (dict(p=100), dict(n_classes=1), dict(n_classes=5000), dict(x_dtype=0)):
        cfg = B.bmgd_default_config()
        cfg.p, cfg.buffer_n, cfg.batch_n, cfg.lr, cfg.passes = 64, 1000, 100, 0.1, 1
        cfg.model, cfg.n_classes, cfg.x_dtype = B.BMGD_SOFTMAX, 10, B.BMGD_BF16
        for k, v in kw.items():
            setattr(cfg, k, v)
        rc, h = B.bmgd_create_ex(cfg)
        assert rc == B.BMGD_EINVAL and h is None, kw


def test_softmax_learning_rate_per_update():
    import torch
    import paper_2312_08728_amd as B
    from oracle import bmgd as O
    w = _case(2000, 128, 40, 1000, 256, T=2, R=1)
    X, y = wl.dataset(w)
    table = [0.08 / (1 + 0.3 * u) for u in range(10)]            # 16 updates in the run: the last value persists
    ref = O.BMGD(w.model, w.p, w.n, 9.0, w.T, C=w.C)
    ref.set_lr_schedule(np.asarray(table, dtype=np.float32))
    ctx = B.Context(w.p, w.N0, w.n, 9.0, w.T, model=w.model, n_classes=w.C, x_dtype=B.BMGD_BF16)
    ctx.set_lr_schedule(table)
    xd, yd = torch.from_numpy(X.view(np.int16)).cuda(), torch.from_numpy(y).cuda()
    s = torch.cuda.Stream()
    for k in range(2):
        ref.run_buffer(X[k * 1000:(k + 1) * 1000], y[k * 1000:(k + 1) * 1000])
        ctx.run_device_buffer(xd[k * 1000:(k + 1) * 1000], yd[k * 1000:(k + 1) * 1000], 1000, s)
    got = ctx.get_theta().reshape(w.p, w.C)
    ctx.close()
    assert rel_l2(got, ref.theta) <= TOL


@pytest.mark.parametrize("optimizer", [0, 3])
def test_graph_replays_equal_single_launches(optimizer):
    """The captured pass (BMGD_CHAIN_GRAPH, the default) against the same launches issued one by one
    (BMGD_CHAIN_LAUNCH): bit-identical W after every buffer, over several replays of each graph, with blocking calls,
    a change of the learning rate, a per-update schedule and other device work between the replays; a buffer with
    fewer rows (other graphs) in the rotation; plain steps and Adam (whose update count comes from device memory)."""
    import torch
    import paper_2312_08728_amd as B
    w = _case(2300, 128, 40, 1000, 128, T=2)                      # buffers of 1000, 1000 and 300 rows
    X, y = wl.dataset(w)
    xd, yd = torch.from_numpy(X.view(np.int16)).cuda(), torch.from_numpy(y).cuda()
    s = torch.cuda.Stream()
    scratch = torch.zeros(1 << 20, device="cuda")
    ctxs = [B.Context(w.p, w.N0, w.n, w.alpha, w.T, model=w.model, n_classes=w.C, chain=chain, optimizer=optimizer)
            for chain in (B.BMGD_CHAIN_GRAPH, B.BMGD_CHAIN_LAUNCH)]
    try:
        assert [c.stats().chain for c in ctxs] == [B.BMGD_CHAIN_GRAPH, B.BMGD_CHAIN_LAUNCH]
        for r in range(4):                                           # every graph is replayed on iterations 1..3
            if r == 2:
                for c in ctxs:
                    c.set_lr(0.02)
            if r == 3:
                for c in ctxs:
                    c.set_lr_schedule(np.linspace(0.03, 0.001, 37).astype(np.float32))
            for k in range(w.K):
                lo, hi = wl.buffer_rows(w, k)
                for c in ctxs:
                    c.run_device_buffer(xd[lo:hi], yd[lo:hi], hi - lo, s)
                with torch.cuda.stream(s):
                    scratch.add_(1.0)                                # the program's own work between replays
                a, b = ctxs[0].get_theta(), ctxs[1].get_theta()      # (blocks)
                assert np.isfinite(a).all() and np.array_equal(a, b), (r, k)
        assert ctxs[0].stats().steps == ctxs[1].stats().steps == 4 * 2 * (8 + 8 + 3)
    finally:
        for c in ctxs:
            c.close()
