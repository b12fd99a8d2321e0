"""Helpers shared by the GPU parity tests: drive libbmgd through its C ABI and the oracle on the same bytes."""
from __future__ import annotations

import numpy as np

import workloads as wl
from oracle import bmgd as O


def rel_l2(a, b) -> float:
    a, b = np.asarray(a, dtype=np.float64).ravel(), np.asarray(b, dtype=np.float64).ravel()
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def gpu_run(w: wl.Workload, X: np.ndarray, y: np.ndarray, R=None, resident=False, theta0=None, **opts):
    """Run workload w on the GPU: R iterations over the K contiguous buffers of (X, y).

    resident=False goes through bmgd_load_buffer_async (pinned host memory, a copy stream and a compute
    stream); resident=True puts the data in device memory first and uses bmgd_run_device_buffer.
    Returns (theta, stats).
    """
    import torch
    import paper_2312_08728_amd as B

    R = w.R if R is None else R
    N = X.shape[0]
    K = -(-N // w.N0)
    ctx = B.Context(w.p, min(w.N0, N), min(w.n, min(w.N0, N)), w.alpha, w.T, model=w.model, n_classes=w.C,
                    seed=w.seed, n_buffers=K, **opts)
    try:
        if theta0 is not None:
            ctx.set_theta(theta0)
        xt = torch.from_numpy(X.view(np.int16) if X.dtype == np.uint16 else X)
        yt = torch.from_numpy(y)
        if resident:
            xd, yd = xt.cuda(), yt.cuda()
            s = torch.cuda.Stream()
            for _ in range(R):
                for k in range(K):
                    lo, hi = k * w.N0, min((k + 1) * w.N0, N)
                    ctx.run_device_buffer(xd[lo:hi], yd[lo:hi], hi - lo, s)
        else:
            xp, yp = xt.pin_memory(), yt.pin_memory()
            cs, ks = torch.cuda.Stream(), torch.cuda.Stream()
            for _ in range(R):
                for k in range(K):
                    lo, hi = k * w.N0, min((k + 1) * w.N0, N)
                    ctx.load_buffer_async(xp[lo:hi], yp[lo:hi], hi - lo, cs)
                    ctx.run_buffer(ks)
        theta = ctx.get_theta()
        st = ctx.stats()
        return theta, st
    finally:
        ctx.close()


def oracle_run(w: wl.Workload, X: np.ndarray, y: np.ndarray, R=None, theta0=None, reshuffle=O.PER_PASS):
    R = w.R if R is None else R
    return O.run(w.model, X, y, w.N0, w.n, w.alpha, w.T, R, C=w.C, seed=w.seed, theta0=theta0, reshuffle=reshuffle)
