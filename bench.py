"""Throughput of the BMGD computation step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2]

One *step* is one buffer taken through the whole hot path: the device-side partitions for its T passes
and the chain of T * M sequential mini-batch updates (eq. (2.1)).  Buffers are resident in HBM when the
timed region starts (bmgd_run_device_buffer); the pinned-host loader is measured separately and reported
under "h2d".  Prints ONE JSON line.

Metric: sample-gradients per second = rows visited by mini-batch updates per second (R * T * N of
Algorithm 1 per whole run), plus the achieved algorithmic HBM rate of the fused gradient kernel.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth

# HBM traffic of one launch of the chain kernel on the primary workload, from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE (see profiles/), scaled by the copy calibration; valid only for the source of the kernel it was measured on
# (the line reports null once that file has changed: measure again and update the entry).
TRAFFIC = {"cfg2": {"sources": ('gram_kernels.hip', 'gram_layout.h', 'gram_products.hip'), "kernel_sha256": "c5a25ec6a3db67ff4eaedb207055baec6f4cc6cbd01c8f94818cb9a656a95779", "bytes_per_launch": 217072615}, "cfg3": {"sources": ('glm_narrow_kernel.hip', 'glm_exchange.h', 'glm_device.h'), "kernel_sha256": "45fef1bf3ccf41c027138800dba42d12c1e5535d30ae6f2492f523b280ed68fe", "bytes_per_launch": 2473478069}, "cfg4": {"sources": ('glm_split_kernel.hip', 'glm_exchange.h', 'glm_device.h'), "kernel_sha256": "8d8c2fd79cd5ea4e1c2d85d65948ba501b3f0dcb49b443ac8ecd2b5b9677dfeb", "bytes_per_launch": 9428150173}}


def _kernel_sha(sources) -> str:
    h = hashlib.sha256()
    for f in sources:
        with open(os.path.join(ROOT, "paper_2312_08728_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def _algorithmic_bytes_per_sample_gradient(w) -> int:
    # one read of the row (p values) + its response + its index in the partition
    return w.p * w.x_itemsize + 4 + 4


def _device_buffers(w, nbuf, from_host=None):
    """nbuf buffers of the workload in HBM: from the seeded host generator, or drawn on the device."""
    import torch
    import workloads as wl
    bufs = []
    if from_host is not None:
        X, y = from_host
        for k in range(nbuf):
            lo, hi = wl.buffer_rows(w, k % w.K)
            bufs.append((torch.from_numpy(X[lo:hi]).cuda(), torch.from_numpy(y[lo:hi]).cuda(), hi - lo))
        return bufs
    g = torch.Generator(device="cuda")
    g.manual_seed(w.seed)
    if w.model == wl.SOFTMAX:
        Wt = torch.randn(w.p, w.C, device="cuda", generator=g) / w.p ** 0.5
        for k in range(nbuf):
            X = torch.randn(w.N0, w.p, device="cuda", generator=g).to(torch.bfloat16)
            gumbel = -torch.log(-torch.log(torch.rand(w.N0, w.C, device="cuda", generator=g)))
            y = torch.argmax(X.float() @ Wt + gumbel, dim=1).to(torch.int32)
            del gumbel
            bufs.append((X.view(torch.int16), y, w.N0))
        return bufs
    theta = torch.randn(w.p, device="cuda", generator=g) / w.p ** 0.5
    for k in range(nbuf):
        X = torch.randn(w.N0, w.p, device="cuda", generator=g)
        eta = X @ theta
        if w.model == wl.LOGISTIC:
            y = (torch.rand(w.N0, device="cuda", generator=g) < torch.sigmoid(eta)).float()
        else:
            y = eta + w.noise_sigma * torch.randn(w.N0, device="cuda", generator=g)
        bufs.append((X, y, w.N0))
    return bufs


def _time_resident(w, bufs, steps, warmup, chain=0):
    """Run `steps` buffers (cycling over bufs) after `warmup`; returns (seconds, stats delta, theta)."""
    import torch
    import paper_2312_08728_amd as B
    ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T, model=w.model, n_classes=w.C, seed=w.seed, n_buffers=w.K, chain=chain)
    try:
        _, s = _streams()
        for i in range(warmup):
            X, y, rows = bufs[i % len(bufs)]
            ctx.run_device_buffer(X, y, rows, s)
        ctx.sync()
        if warmup:
            # timed run starts from the same state a fresh run would: theta = 0, buffer counter 0
            ctx.set_theta([0.0] * ctx.theta_len)
            ctx.set_position(0)
        st0 = ctx.stats()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            X, y, rows = bufs[i % len(bufs)]
            ctx.run_device_buffer(X, y, rows, s)
        ctx.sync()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        st1 = ctx.stats()
        theta = ctx.get_theta()
        delta = {
            "sample_gradients": st1.sample_gradients - st0.sample_gradients,
            "minibatch_steps": st1.steps - st0.steps,
            "chain_ms": st1.chain_ms - st0.chain_ms,
            "chain_launches": st1.chain_launches - st0.chain_launches,
            "compute_ms": st1.compute_ms - st0.compute_ms,
            "prep_ms": st1.prep_ms - st0.prep_ms,
            "prep_launches": st1.prep_launches - st0.prep_launches,
            "chain": st1.chain,
            "n_workgroups": st1.n_workgroups, "threads_per_group": st1.threads_per_group,
        }
        return dt, delta, theta
    finally:
        ctx.close()


def _stream_read_ceiling():
    """What plain streaming kernels reach on this device: a sum over 1 GiB of fp32 (reads only) and a copy of 1 GiB
    (reads + writes), library kernels, best of five each, timed with events on the current stream.  Yardsticks beside
    the published peak, not targets."""
    import torch
    x = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
    y = torch.empty_like(x)

    def best_ms(fn):
        fn()
        torch.cuda.synchronize()
        best = 1e9
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            e1.synchronize()
            best = min(best, e0.elapsed_time(e1))
        return best

    out = {"sum_1GiB_read_GBs": round((1 << 30) / (best_ms(lambda: x.sum()) * 1e-3) / 1e9, 1),
           "copy_1GiB_read_plus_write_GBs": round(2 * (1 << 30) / (best_ms(lambda: y.copy_(x)) * 1e-3) / 1e9, 1)}
    del x, y
    torch.cuda.empty_cache()
    return out


def _roofline(w, delta, traffic=None):
    import workloads as wl
    per_launch_s = delta["chain_ms"] / 1e3 / max(delta["chain_launches"], 1)
    if w.model == wl.SOFTMAX:
        # two dense contractions per mini-batch update: 2 * (2 n p C) flops
        flops = 4.0 * w.p * w.C * delta["sample_gradients"]
        achieved = flops / (delta["chain_ms"] / 1e3) / 1e12
        return {"bound": "mfma", "achieved": round(achieved, 2), "peak": 2500.0, "unit": "TFLOP/s",
                "frac": round(achieved / 2500.0, 5), "traffic": None,
                "kernel": "gemm_nt_kernel (logits, gradient+update) + softmax_residual_kernel"}
    bytes_per_launch = _algorithmic_bytes_per_sample_gradient(w) * delta["sample_gradients"] / max(delta["chain_launches"], 1)
    if delta.get("chain") in (3, 5):
        # Least squares in the form of eq. (3.1): the rows are read by the kernel that forms the moment matrices
        # of the mini-batches, the updates are applied by the one-workgroup chain kernel.  One launch of each per
        # buffer, and the two kernels of consecutive buffers overlap: the rate is the buffer's algorithmic bytes over
        # the average duration of the longer (dominant) of the two.
        prep_s = delta["prep_ms"] / 1e3 / max(delta["prep_launches"], 1)
        dominant_s = max(per_launch_s, prep_s)
        achieved = bytes_per_launch / dominant_s / 1e9
        steps_per_launch = delta["minibatch_steps"] / max(delta["chain_launches"], 1)
        q = w.p + 1
        return {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 5), "traffic": traffic,
                "kernel": "gram_chain_kernel" if per_launch_s >= prep_s
                          else ("gram_mfma_kernel + affine_pair_kernel" if delta.get("chain") == 5 else "gram_mfma_kernel"),
                "avg_launch_ms": round(dominant_s * 1e3, 4),
                "algorithmic_bytes_per_launch": int(bytes_per_launch),
                "moments_kernel": {"avg_launch_ms": round(prep_s * 1e3, 4),
                                   "reads_GBs": round(bytes_per_launch / prep_s / 1e9, 1),
                                   "fp32_mfma_TFLOPs": round(delta["sample_gradients"] / max(delta["prep_launches"], 1)
                                                             * q * q / prep_s / 1e12, 2)},
                "chain_kernel": {"avg_launch_ms": round(per_launch_s * 1e3, 4),
                                 "us_per_minibatch_update": round(per_launch_s * 1e6 / steps_per_launch, 4),
                                 "moment_bytes_GBs": round(steps_per_launch * (w.p + 1) * w.p * 4 / per_launch_s / 1e9, 1),
                                 "note": "steps multiplied in pairs behind the moments kernel; the chain runs over the pairs"
                                         if delta.get("chain") == 5 else "one workgroup; bound by a single compute unit's load path"}}
    achieved = bytes_per_launch / per_launch_s / 1e9
    return {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 5), "traffic": traffic,
            # the three persistent kernels differ in their workgroup size: 11 wavefronts (rows wider than 1024 floats:
            # eight row wavefronts and an exchange wavefront alone on its SIMD), 12 (narrower rows whose share of a step fits
            # the registers: eight row wavefronts and four exchange wavefronts), else the general kernel
            "kernel": {704: "glm_split_kernel", 768: "glm_narrow_kernel"}.get(delta["threads_per_group"], "glm_chain_kernel"),
            "avg_launch_ms": round(per_launch_s * 1e3, 4),
            "algorithmic_bytes_per_launch": int(bytes_per_launch)}


_STREAMS = []


def _streams():
    """One copy stream and one compute stream for the whole process.  HIP spreads streams over a few hardware
    queues (four by default) and work on two streams that share a queue is serialised, a copy included: with the
    default stream and the library's own chain stream these two fill the four, so every phase reuses them."""
    import torch
    if not _STREAMS:
        _STREAMS.extend([torch.cuda.Stream(), torch.cuda.Stream()])
    return _STREAMS[0], _STREAMS[1]


def _loader_context(w, host):
    """A context for the loader runs, after one untimed sweep over the buffers: the first copy out of newly pinned
    memory takes several milliseconds longer than every later one."""
    import paper_2312_08728_amd as B
    ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T, model=w.model, n_classes=w.C, seed=w.seed, n_buffers=w.K)
    cs, ks = _streams()
    for xs, ys, _, _, rows in host:
        ctx.load_buffer_async(xs, ys, rows, cs)
        ctx.run_buffer(ks)
    ctx.sync()
    return ctx, ctx.stats()


def _time_pipelined(w, host, steps):
    """Same buffers through the pinned-host loader on its own stream; returns overlap figures.  copy_ms is the sum of
    the buffers' own copy intervals, copy_span_ms the time from the start of the first copy to the end of the last
    (it includes the copy stream's idle gaps between buffers: two event records, a wait and two copy commands each)."""
    import torch
    ctx, s0 = _loader_context(w, host)
    try:
        cs, ks = _streams()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(cs)
        for i in range(steps):
            xs, ys, _, _, rows = host[i % len(host)]
            ctx.load_buffer_async(xs, ys, rows, cs)
            ctx.run_buffer(ks)
        e1.record(cs)
        ctx.sync()
        dt = time.perf_counter() - t0
        st = ctx.stats()
        return {"seconds": dt, "copy_ms": st.copy_ms - s0.copy_ms, "wait_ms": st.wait_ms - s0.wait_ms,
                "copy_span_ms": e0.elapsed_time(e1),
                "compute_ms": st.compute_ms - s0.compute_ms, "h2d_bytes": st.h2d_bytes - s0.h2d_bytes}
    finally:
        ctx.close()


def _time_adaptive(w, host, steps, max_passes=64):
    """The loader again, with the number of passes per buffer left to the library: passes go on until the next
    buffer has arrived (Section 2.1), at least the workload's own T."""
    ctx, s0 = _loader_context(w, host)
    try:
        cs, ks = _streams()
        used = []
        t0 = time.perf_counter()
        ctx.load_buffer_async(host[0][0], host[0][1], host[0][4], cs)
        for i in range(steps):
            if i + 1 < steps:
                xs, ys, _, _, rows = host[(i + 1) % len(host)]
                used.append(ctx.run_buffer_adaptive(ks, xs, ys, rows, cs, w.T, max_passes))
            else:
                used.append(ctx.run_buffer_adaptive(ks, None, None, 0, None, w.T, max_passes))
        ctx.sync()
        dt = time.perf_counter() - t0
        st = ctx.stats()
        return {"seconds": dt, "copy_ms": st.copy_ms - s0.copy_ms, "wait_ms": st.wait_ms - s0.wait_ms,
                "compute_ms": st.compute_ms - s0.compute_ms,
                "sample_gradients": st.sample_gradients - s0.sample_gradients, "passes": used}
    finally:
        ctx.close()


def _time_two_level(w, X, y, steps, max_passes=64):
    """Both transfers of Section 2.1 at once: a reader thread brings buffers from files into a pinned ring, the
    loader copies them to the device, and passes over the buffer in hand go on until the next one has arrived."""
    import tempfile
    import paper_2312_08728_amd as B
    with tempfile.TemporaryDirectory() as d:
        fx, fy = os.path.join(d, "x.bin"), os.path.join(d, "y.bin")
        X.tofile(fx)
        y.tofile(fy)
        ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T, model=w.model, n_classes=w.C, seed=w.seed, n_buffers=w.K)
        rd = B.Reader(fx, fy, w.p, w.N, w.N0, x_dtype=B.BMGD_BF16 if w.x_dtype == "bf16" else B.BMGD_F32, ring_slots=3,
                      loop=True)
        try:
            cs, ks = _streams()
            for _ in range(w.K):                       # untimed: first use of the ring's pinned memory
                rd.load_into(ctx, cs)
                ctx.run_buffer(ks)
            ctx.sync()
            s0, (b0, r0) = ctx.stats(), rd.stats()
            used = []
            t0 = time.perf_counter()
            rd.load_into(ctx, cs)
            for i in range(steps):
                if i + 1 < steps:
                    used.append(ctx.run_buffer_adaptive_reader(ks, rd, cs, w.T, max_passes)[0])
                else:
                    used.append(ctx.run_buffer_adaptive(ks, None, None, 0, None, w.T, max_passes))
            ctx.sync()
            dt = time.perf_counter() - t0
            st, (b1, r1) = ctx.stats(), rd.stats()
            return {"buffers": steps, "ms": round(dt * 1e3, 3), "passes_per_buffer": used,
                    "sample_gradients_per_s": round((st.sample_gradients - s0.sample_gradients) / dt, 1),
                    "file_read_GBs": round((b1 - b0) / max(r1 - r0, 1e-9) / 1e9, 2),
                    "frac_h2d_hidden": round(1.0 - (st.wait_ms - s0.wait_ms) / max(st.copy_ms - s0.copy_ms, 1e-9), 4),
                    "note": "files in the temporary directory (page cache), ring of 3 pinned buffers"}
        finally:
            rd.close()
            ctx.close()


def _host_buffers(w, nbuf):
    """The first nbuf buffers of the workload from the seeded generator, each in pinned host memory:
    [(x tensor, y tensor, numpy view of x as stored, numpy view of y, rows)]."""
    import numpy as np
    import torch
    import workloads as wl
    xdt = torch.int16 if w.x_dtype == "bf16" else torch.float32
    ydt = torch.int32 if w.model == wl.SOFTMAX else torch.float32
    out = []
    for k in range(nbuf):
        lo, hi = wl.buffer_rows(w, k)
        xs = torch.empty((hi - lo, w.p), dtype=xdt, pin_memory=True)
        ys = torch.empty(hi - lo, dtype=ydt, pin_memory=True)
        xn = xs.numpy().view(np.uint16) if w.x_dtype == "bf16" else xs.numpy()
        wl.rows(w, lo, hi, out_x=xn, out_y=ys.numpy())
        out.append((xs, ys, xn, ys.numpy(), hi - lo))
    return out


def _cpu_baseline(w, host, budget_s=20.0, max_runs=None):
    """The fp64 oracle, as it stands, on the same stored inputs, over the buffer sequence the timed run uses
    (buffer i of the run = host[i % len(host)]); stops after the buffer during which budget_s of CPU time ran out.
    Returns (the record, theta after the last buffer it completed, number of buffers it completed)."""
    from oracle import bmgd as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([int(t.get("num_threads", 1)) for t in threadpool_info()] or [1])
    except Exception:
        threads = 1
    st = O.BMGD(w.model, w.p, w.n, w.alpha, w.T, C=w.C, seed=w.seed)
    total = w.R * w.K if max_runs is None else max_runs
    t0 = time.perf_counter()
    done_sg = 0
    runs = 0
    while runs < total:
        _, _, xn, yn, rows = host[runs % len(host)]
        st.run_buffer(xn, yn)
        done_sg += w.T * rows
        runs += 1
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    sample = (f"whole {w.name} run ({runs} buffers)" if runs == w.R * w.K
              else f"first {runs} of {w.R * w.K} buffer runs of {w.name} ({runs * w.T * w.M} mini-batch updates; time-bounded)")
    return {"value": round(done_sg / dt, 1), "unit": "sample-gradients/s", "cores": threads, "kind": "oracle",
            "sample": sample, "seconds": round(dt, 3)}, st.theta, runs


def _gpu_prefix(w, bufs, runs, chain):
    """theta after the first `runs` buffers of the timed sequence, from a fresh context (theta = 0, buffer counter 0)."""
    import paper_2312_08728_amd as B
    ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T, model=w.model, n_classes=w.C, seed=w.seed, n_buffers=w.K, chain=chain)
    try:
        _, s = _streams()
        for i in range(runs):
            X, y, rows = bufs[i % len(bufs)]
            ctx.run_device_buffer(X, y, rows, s)
        return ctx.get_theta()
    finally:
        ctx.close()


def _h2d_block(w, host, comp_ms_per_buffer, nb, two_level=None):
    """The pinned-host loader on its own stream against the same buffers: what part of the copy time the computation
    hides at the workload's own T, how well the two overlap, and how the picture changes when the passes go on until
    the next buffer has arrived (Section 2.1)."""
    nbuf = len(host)
    piped = _time_pipelined(w, host, nb)
    copy_ms = piped["copy_ms"]
    comp_alone = comp_ms_per_buffer * nb
    hidden = 1.0 - piped["wait_ms"] / max(copy_ms, 1e-9)
    piped_ms = piped["seconds"] * 1e3
    # the copies alone take their span (own intervals plus the copy stream's gaps between buffers) when the link is
    # the bound; when the computation is, their own intervals
    h2d_alone = piped["copy_span_ms"] if comp_alone <= copy_ms else copy_ms
    overlap_eff = (h2d_alone + comp_alone - piped_ms) / max(min(h2d_alone, comp_alone), 1e-9)
    # the pipeline's own limit for nb buffers: the first copy (link-bound case) or the last computation (compute-bound
    # case) has nothing to overlap with
    shorter, longer = (comp_alone, copy_ms) if comp_alone <= copy_ms else (copy_ms, comp_alone)
    eff_ceiling = (shorter - shorter / nb) / max(shorter, 1e-9)
    out = {"buffers": nb, "distinct_buffers": nbuf, "h2d_gbs": round(piped["h2d_bytes"] / max(copy_ms, 1e-9) / 1e6, 2),
           "copy_ms": round(copy_ms, 3), "copy_span_ms": round(piped["copy_span_ms"], 3), "compute_ms_alone": round(comp_alone, 3),
           "pipelined_ms": round(piped_ms, 3),
           "pipelined_sample_gradients_per_s": round(nb * w.T * w.N0 / (piped_ms * 1e-3), 1),
           "bound": "compute" if comp_alone > copy_ms else "host-to-device link",
           "frac_h2d_hidden": round(hidden, 4),
           # no more of the copy time can be hidden than the device spent computing in that run
           "ceiling_at_this_T": round(min(1.0, piped["compute_ms"] / max(copy_ms, 1e-9)), 4),
           "overlap_efficiency": round(overlap_eff, 4),
           "overlap_efficiency_ceiling_for_this_many_buffers": round(eff_ceiling, 4)}
    # passes needed for the computation on one buffer to last as long as the copy of the next
    pass_ms = comp_ms_per_buffer / w.T
    copy_per_buffer = copy_ms / nb
    t_star = max(w.T, int(copy_per_buffer / max(pass_ms, 1e-9) * 1.15) + 1)
    out["passes_to_cover_one_copy"] = t_star
    sweep = []
    for T in sorted({w.T, 2 * w.T, max(w.T, t_star // 4), max(w.T, t_star // 2), t_star}):
        wt = w.scaled(T=T)
        pt = _time_pipelined(wt, host, nb)
        sweep.append({"T": T, "frac_h2d_hidden": round(1.0 - pt["wait_ms"] / max(pt["copy_ms"], 1e-9), 4),
                      "sample_gradients_per_s": round(nb * T * wt.N0 / pt["seconds"], 1)})
    out["passes_sweep"] = sweep
    ad = _time_adaptive(w, host, nb, max_passes=max(64, 2 * t_star))
    out["adaptive_passes"] = {
        "passes_per_buffer": ad["passes"], "ms": round(ad["seconds"] * 1e3, 3),
        "sample_gradients_per_s": round(ad["sample_gradients"] / ad["seconds"], 1),
        "frac_h2d_hidden": round(1.0 - ad["wait_ms"] / max(ad["copy_ms"], 1e-9), 4),
        # the first buffer's copy has no computation to hide behind: the fraction over the buffers that follow it
        "frac_h2d_hidden_after_first_buffer": round(1.0 - max(ad["wait_ms"] - ad["copy_ms"] / nb, 0.0)
                                                    / max(ad["copy_ms"] * (nb - 1) / nb, 1e-9), 4),
        "device_busy_frac": round(ad["compute_ms"] / (ad["seconds"] * 1e3), 4)}
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="buffers to time (default: one whole run, R*K)")
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg4")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the short side measurements of the other workloads")
    ap.add_argument("--chain", type=int, default=0, help="BMGD_CHAIN_* for the primary workload (0 = automatic)")
    ap.add_argument("--no-h2d", action="store_true")
    ap.add_argument("--device-data", action="store_true",
                    help="draw the workload's buffers on the device (same shapes and distributions) instead of copying the "
                         "seeded host dataset: for profiling the large workloads; implies no oracle comparison and no h2d")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain elementwise copy of 1 GiB (5 launches): the known-size kernel that "
                         "hardware-counter readings of HBM traffic are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on exactly one GPU (the method's step chain is sequential and no "
              "collectives are built); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import paper_2312_08728_amd as B
    import torch
    import workloads as wl
    if not torch.cuda.is_available():
        print("bench.py: no GPU available", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")     # 1 GiB read, 1 GiB written per launch
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read_per_launch": src.numel() * 4,
                                               "bytes_written_per_launch": dst.numel() * 4, "launches": 5}}))
        return 0

    w = wl.CONFIGS[args.workload]
    steps = args.steps if args.steps is not None else w.R * w.K
    # Data sets of up to 10 GB are drawn whole; of a larger one (cfg4: 32.8 GB) the first two buffers, which the run
    # then takes in turn: every buffer has the configuration's full size, and the rows are independent draws anyway.
    nbuf_data = w.K if w.N * w.p * w.x_itemsize <= (10 << 30) else 2
    host = None
    if args.device_data:
        args.no_cpu_baseline = args.no_h2d = True
        bufs = _device_buffers(w, min(w.K, 2))
    else:
        host = _host_buffers(w, nbuf_data)
        bufs = [(xs.cuda(), ys.cuda(), rows) for xs, ys, _, _, rows in host]
    dt, delta, theta = _time_resident(w, bufs, steps, args.warmup, args.chain)

    tr = TRAFFIC.get(w.name, {})
    traffic = tr.get("bytes_per_launch") if tr.get("kernel_sha256") == _kernel_sha(tr.get("sources", ())) else None
    result = {
        "metric": "sample-gradients/sec (BMGD computation step, buffers resident in HBM)",
        "value": round(delta["sample_gradients"] / dt, 1),
        "unit": "sample-gradients/s",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": round(dt * 1e3 / steps, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.x_dtype == "bf16" else "f32",
        "data": "synthetic, drawn on the device" if args.device_data else "synthetic",
        "config": {"workload": f"{w.name}: {wl.MODEL_NAMES[w.model]} regression N={w.N} p={w.p} buffer={w.N0} "
                               f"batch={w.n} passes={w.T} lr={w.alpha} (a step = one buffer = {w.T * w.M} mini-batch updates)",
                   "buffers": (f"the {len(bufs)} buffers of the data set, in order" if len(bufs) == w.K else
                               f"the first {len(bufs)} of the data set's {w.K} buffers (full size), taken in turn"),
                   "minibatch_updates_timed": delta["minibatch_steps"],
                   "us_per_minibatch_update": round(dt * 1e6 / max(delta["minibatch_steps"], 1), 3),
                   "workgroups": delta["n_workgroups"], "threads_per_group": delta["threads_per_group"]},
        "roofline": _roofline(w, delta, traffic),
    }
    if result["roofline"]["bound"] == "hbm":
        result["roofline"]["measured_streaming_kernels"] = _stream_read_ceiling()

    if not args.no_cpu_baseline:
        base, theta_cpu, runs = _cpu_baseline(w, host)
        result["cpu_baseline"] = base
        # the same buffers in the same order on the device, from theta = 0, against the oracle's estimate at that point
        got = _gpu_prefix(w, bufs, runs, args.chain).astype(np.float64).ravel()
        want = theta_cpu.ravel()
        result["parity_rel_l2_vs_oracle"] = float(f"{np.linalg.norm(got - want) / np.linalg.norm(want):.3e}")
        result["parity_largest_coordinate_error"] = float(f"{np.max(np.abs(got - want)) / np.max(np.abs(want)):.3e}")
        result["parity_sample"] = f"theta after the first {runs} buffer runs ({runs * w.T * w.M} mini-batch updates), both from theta = 0"
    del bufs
    torch.cuda.empty_cache()

    if not args.no_h2d:
        result["h2d"] = _h2d_block(w, host, delta["compute_ms"] / steps, 16)
    del host

    if not args.no_others:
        others = {}
        side = [("cfg1", 5, 0, 5), ("cfg2", 10, 0, 20), ("cfg2", 10, 1, 10), ("cfg2", 10, 3, 20), ("cfg3", 2, 0, 4), ("cfg4", 2, 0, 4),
                ("cfg4_full_batch", 1, 0, 1), ("cfg5", 1, 0, 1)]
        for name, nbuf, chain, nsteps in side:
            if name == w.name and chain == args.chain:
                continue                            # that is the headline
            note = None
            if name == "cfg4_full_batch":
                # the fused gradient kernel at its real tile shape on one batch = the whole buffer (the method's own
                # full-batch special case): its streaming rate with the per-step exchange amortised away
                wo = wl.CONFIGS["cfg4"].scaled(name=name, n=wl.CONFIGS["cfg4"].N0)
                note = "kernel-only probe: one mini-batch = the whole buffer, so there is no chain of updates; not a run configuration"
            else:
                wo = wl.CONFIGS[name]
            try:
                ob = _device_buffers(wo, nbuf)
                odt, od, _ = _time_resident(wo, ob, nsteps, 1, chain)
                if chain == 1:
                    name += "_row_form"          # the same workload with the updates taken row by row (eq. (2.1))
                if chain == 3:
                    name += "_chain_of_all_steps"   # the moment form without the pair products the automatic choice makes (eq. (3.2))
                rf = _roofline(wo, od)
                others[name] = {"value": round(od["sample_gradients"] / odt, 1), "ms_per_step": round(odt * 1e3 / nsteps, 4),
                                "us_per_minibatch_update": round(odt * 1e6 / od["minibatch_steps"], 3),
                                "roofline_bound": rf["bound"], "roofline_frac": rf["frac"], "roofline_kernel": rf["kernel"],
                                "achieved": rf["achieved"], "achieved_unit": rf["unit"],
                                "data": "synthetic, drawn on the device"}
                if od["n_workgroups"] > 0:
                    others[name]["workgroups"] = od["n_workgroups"]
                if note:
                    others[name]["note"] = note
                if wo.name == "cfg3" and not args.no_h2d:
                    # the host-resident configuration through the loader at its own T (inputs drawn on the device and
                    # copied back into pinned memory: they are not under test here)
                    hb = []
                    for Xd, yd, rows in ob:
                        xs = torch.empty(Xd.shape, dtype=Xd.dtype, pin_memory=True).copy_(Xd)
                        ys = torch.empty(yd.shape, dtype=yd.dtype, pin_memory=True).copy_(yd)
                        hb.append((xs, ys, None, None, rows))
                    del ob
                    ob = None
                    torch.cuda.empty_cache()
                    hd = _h2d_block(wo, hb, od["compute_ms"] / nsteps, 12)
                    others[name]["h2d"] = hd
                    del hb
                del ob
                torch.cuda.empty_cache()
            except Exception as e:  # a side measurement must not lose the main line
                others[name] = {"error": str(e)[:200]}
        if not args.no_h2d:
            try:
                # both transfers of Section 2.1 at once, on cfg2 (its 400 MB data set goes to files in the page cache)
                wo = wl.CONFIGS["cfg2"]
                Xo, yo = wl.dataset(wo)
                others["cfg2_reader_and_adaptive_passes"] = _time_two_level(wo, Xo, yo, 20)
                del Xo, yo
            except Exception as e:
                others["cfg2_reader_and_adaptive_passes"] = {"error": str(e)[:200]}
        # cfg2 under fixed partitions (Section 3.1.1) with the moment matrices of every buffer cached: after the first
        # iteration a buffer costs its chain of updates only, and no row is read or copied.  With BMGD_CHAIN_PRODUCT the
        # product of a buffer's steps is kept as well (same rate, same passes): a buffer then costs one small matrix-vector
        # product.
        for key, chain_mode, note in (("cfg2_fixed_partitions_cached_moments", 0, "iterations after the first: chain of eq. (3.1) only"),
                                      ("cfg2_fixed_partitions_cached_products", 5,
                                       "iterations after the first: the kept product of a buffer's steps (eq. (3.2)) applied once")):
            try:
                wo = wl.CONFIGS["cfg2"]
                ob = _device_buffers(wo, wo.K)
                ctx = B.Context(wo.p, wo.N0, wo.n, wo.alpha, wo.T, seed=wo.seed, reshuffle=B.BMGD_RESHUFFLE_FIXED, n_buffers=wo.K,
                                cache_moments=True, chain=chain_mode)
                _, s = _streams()
                for Xb, yb, rows in ob:
                    ctx.run_device_buffer(Xb, yb, rows, s)
                ctx.sync()
                st0 = ctx.stats()
                t0 = time.perf_counter()
                for _ in range(4 * wo.K):
                    ctx.run_cached_buffer(s)
                ctx.sync()
                odt = time.perf_counter() - t0
                st1 = ctx.stats()
                ctx.close()
                others[key] = {
                    "value": round((st1.sample_gradients - st0.sample_gradients) / odt, 1), "ms_per_step": round(odt * 1e3 / (4 * wo.K), 4),
                    "us_per_minibatch_update": round(odt * 1e6 / (st1.steps - st0.steps), 3),
                    "note": note, "data": "synthetic, drawn on the device"}
                del ob
                torch.cuda.empty_cache()
            except Exception as e:
                others[key] = {"error": str(e)[:200]}
        result["other_workloads"] = others

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
