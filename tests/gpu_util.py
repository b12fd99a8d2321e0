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


def coord_err(a, b) -> float:
    """Largest error of a single coordinate, relative to the largest coordinate of the reference."""
    a, b = np.asarray(a, dtype=np.float64).ravel(), np.asarray(b, dtype=np.float64).ravel()
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300))


def parity_after_every_buffer(w: wl.Workload, n_runs: int, report=None, **opts):
    """The first n_runs buffer runs of workload w (buffers k = 0 .. K-1, then again from 0: iterations r = 1, 2, ...)
    on the GPU through the pinned-host loader and in the oracle, on the same stored bytes, comparing theta after
    EVERY buffer.  Buffers are drawn one at a time into two pinned staging areas that take turns (like the two
    device slots), so a data set larger than host memory allows is never held whole; the copy of buffer i + 1 is
    enqueued before theta after buffer i is fetched.  Returns a list of (rel-L2, largest coordinate error) per run
    and the GPU statistics.
    """
    import torch
    import paper_2312_08728_amd as B

    xdt = torch.int16 if w.x_dtype == "bf16" else torch.float32
    ydt = torch.int32 if w.model == wl.SOFTMAX else torch.float32
    keep_all = w.N * w.p * w.x_itemsize <= (10 << 30)      # up to 10 GB: every buffer is drawn once and kept
    n_stage = w.K if keep_all else 2
    stage = [(torch.empty((w.N0, w.p), dtype=xdt).pin_memory(), torch.empty(w.N0, dtype=ydt).pin_memory())
             for _ in range(min(n_stage, n_runs))]
    drawn = {}

    def draw(i):
        """Buffer of run i in its staging area, as (pinned x, pinned y, numpy x, numpy y, rows)."""
        k = i % w.K
        xs, ys = stage[(k if keep_all else i) % len(stage)]
        lo, hi = wl.buffer_rows(w, k)
        xn = xs.numpy()[:hi - lo]
        xn = xn.view(np.uint16) if w.x_dtype == "bf16" else xn
        yn = ys.numpy()[:hi - lo]
        if not (keep_all and k in drawn):
            wl.rows(w, lo, hi, out_x=xn, out_y=yn)
            drawn[k] = True
        return xs, ys, xn, yn, hi - lo

    st = O.BMGD(w.model, w.p, w.n, w.alpha, w.T, C=w.C, seed=w.seed)
    ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T, model=w.model, n_classes=w.C, seed=w.seed, n_buffers=w.K, **opts)
    errs = []
    try:
        cs, ks = torch.cuda.Stream(), torch.cuda.Stream()
        cur = draw(0)
        ctx.load_buffer_async(cur[0], cur[1], cur[4], cs)
        for i in range(n_runs):
            ctx.run_buffer(ks)
            want = st.run_buffer(cur[2], cur[3]).copy()    # the oracle works while the device does
            nxt = None
            if i + 1 < n_runs:
                nxt = draw(i + 1)                          # its staging area was last copied from before an earlier get_theta
                ctx.load_buffer_async(nxt[0], nxt[1], nxt[4], cs)
            got = ctx.get_theta()
            e = (rel_l2(got, want), coord_err(got, want))
            errs.append(e)
            if report is not None:
                report(i, e)
            cur = nxt
        return errs, ctx.stats()
    finally:
        ctx.close()
