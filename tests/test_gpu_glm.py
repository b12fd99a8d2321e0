"""Parity of the HIP chain (least squares, logistic) with the fp64 oracle: final theta after whole runs,
relative L2 error <= 1e-4 (fp32 arithmetic against fp64; the iteration is contractive, so per-step
rounding of order 1e-7 does not accumulate beyond that)."""
import numpy as np
import pytest

import workloads as wl
from gpu_util import gpu_run, oracle_run, rel_l2

pytestmark = pytest.mark.gpu
TOL = 1e-4


def _case(model, N, p, N0, n, T, R, alpha, **kw):
    base = wl.CONFIGS["cfg3" if model == wl.LOGISTIC else "cfg2"]
    return base.scaled(name="case", model=model, N=N, p=p, N0=N0, n=n, T=T, R=R, alpha=alpha, **kw)


def test_cfg1_full_run():
    w = wl.CONFIGS["cfg1"]
    X, y = wl.dataset(w)
    want = oracle_run(w, X, y)
    for chain in (0, 1):                                # 0: automatic (the chain of eq. (3.1) here: 40 steps per launch), 1: row form
        got, st = gpu_run(w, X, y, chain=chain)
        assert st.chain == (3 if chain == 0 else 1)
        assert st.steps == w.steps and st.sample_gradients == w.sample_gradients
        assert st.h2d_bytes == w.R * (X.nbytes + y.nbytes)
        assert rel_l2(got, want) <= TOL


def test_the_four_calls_with_defaults():
    """bmgd_create(p, buffer_n, batch_n, lr, passes) with every default (least squares, fp32, seed 0, a new partition
    per pass, theta = 0, automatic chain, default stream), then only bmgd_load_buffer_async, bmgd_run_buffer and
    bmgd_get_theta, called as plain C entry points, against the oracle."""
    import torch
    import paper_2312_08728_amd as B
    from oracle import bmgd as O
    for p, N0, n, lr, T in ((12, 3000, 250, 0.05, 2), (300, 5000, 999, 0.002, 3)):
        w = _case(wl.LINEAR, 3 * N0 - 77, p, N0, n, T, 1, lr, x_cov="identity")
        X, y = wl.dataset(w)
        xp, yp = torch.from_numpy(X).pin_memory(), torch.from_numpy(y).pin_memory()
        h = B.bmgd_create(p, N0, n, lr, T)
        assert h, B.bmgd_last_error(None)
        try:
            st = O.BMGD(O.LINEAR, p, n, lr, T)
            out = np.empty(p, dtype=np.float32)
            for k in range(w.K):
                lo, hi = wl.buffer_rows(w, k)
                assert B.bmgd_load_buffer_async(h, xp[lo:hi], yp[lo:hi], hi - lo) == B.BMGD_OK
                assert B.bmgd_run_buffer(h) == B.BMGD_OK
                assert B.bmgd_get_theta(h, out, p) == B.BMGD_OK
                assert rel_l2(out, st.run_buffer(X[lo:hi], y[lo:hi])) <= TOL, (p, k)
        finally:
            B.bmgd_destroy(h)


# p chosen to hit every vector width / lanes-per-row / chunks-per-lane combination, with ragged batches
SHAPES = [
    # model, p, N0, n
    (wl.LINEAR, 1, 300, 64), (wl.LINEAR, 3, 1000, 96), (wl.LINEAR, 10, 2000, 100), (wl.LINEAR, 37, 3000, 500),
    (wl.LOGISTIC, 64, 5000, 1000), (wl.LINEAR, 100, 10_000, 1000), (wl.LOGISTIC, 130, 6000, 1024),
    (wl.LOGISTIC, 200, 30_000, 4096), (wl.LINEAR, 257, 3000, 700), (wl.LINEAR, 500, 10_000, 1000),
    (wl.LOGISTIC, 1000, 5000, 2048), (wl.LINEAR, 1022, 3000, 1024), (wl.LINEAR, 2048, 5000, 2048),
    (wl.LOGISTIC, 4096, 9000, 4096),
]


@pytest.mark.parametrize("model,p,N0,n", SHAPES)
def test_shapes_two_buffers(model, p, N0, n):
    N = 2 * N0 - 123                                    # second buffer is shorter than the first
    w = _case(model, N, p, N0, n, T=2, R=2, alpha=0.5 / (p + 10) if model == wl.LINEAR else 0.1,
              x_cov="identity")
    X, y = wl.dataset(w)
    want = oracle_run(w, X, y)
    got, st = gpu_run(w, X, y, chain=1)
    assert st.steps == w.steps
    assert rel_l2(got, want) <= TOL, (st.n_workgroups, st.threads_per_group)


# least squares in the form of eq. (3.1): every lanes-per-row / planes-per-thread choice of the chain, every tile
# count of the moment kernel in both of its splits over workgroups (many short batches: the wider split),
# p not a multiple of 4, ragged batches, batches shorter than p, a single batch, both partition modes
MOMENT_SHAPES = [(1, 300, 64), (3, 1000, 96), (10, 2000, 100), (20, 1500, 300), (37, 3000, 500), (50, 2500, 128),
                 (64, 5000, 1000), (65, 2000, 130), (75, 3000, 750), (85, 2600, 512), (95, 2400, 600), (96, 2400, 200),
                 (100, 10_000, 1000), (108, 2200, 1100), (116, 3000, 256), (127, 3000, 40), (128, 4000, 4000),
                 (20, 5200, 20), (37, 5200, 20), (50, 5200, 20), (75, 5200, 20), (85, 5200, 20), (100, 5200, 20),
                 (116, 5200, 20), (128, 5200, 20)]


@pytest.mark.parametrize("p,N0,n", MOMENT_SHAPES)
@pytest.mark.parametrize("reshuffle", [0, 1])
def test_moment_form_shapes(p, N0, n, reshuffle):
    from oracle import bmgd as O
    N = 2 * N0 - 123
    w = _case(wl.LINEAR, N, p, N0, n, T=5, R=2, alpha=0.5 / (p + 10), x_cov="identity")
    X, y = wl.dataset(w)
    want = oracle_run(w, X, y, reshuffle=O.FIXED if reshuffle else O.PER_PASS)
    got, st = gpu_run(w, X, y, chain=3, reshuffle=reshuffle)
    assert st.steps == w.steps and st.chain == 3
    assert rel_l2(got, want) <= TOL


@pytest.mark.parametrize("G", [1, 2, 7, 64, 256])
@pytest.mark.parametrize("chain", [1, 2])
def test_workgroup_counts_and_chain_modes(G, chain):
    w = _case(wl.LOGISTIC, 12_000, 200, 6000, 1000, T=2, R=1, alpha=0.1)
    X, y = wl.dataset(w)
    want = oracle_run(w, X, y)
    got, st = gpu_run(w, X, y, n_workgroups=G, chain=chain)
    assert st.n_workgroups == G and st.chain == chain
    assert rel_l2(got, want) <= TOL


def _wide_threads(n_workgroups, chain):
    """Threads per workgroup for rows of more than 1024 floats: eight or more workgroups in the persistent chain run the
    kernel with eight row wavefronts and an exchange wavefront, everything else the 512-thread kernels."""
    return 704 if chain == 1 and n_workgroups >= 8 else 512


def test_wide_rows_grids_and_chain_modes():
    """p = 4096, 2048 and 1540: a single workgroup, a few workgroups (sliced reduction), eight and more workgroups (the
    kernel with an exchange wavefront and the two-level exchange) up to the full grid, and the step-per-launch mode."""
    for p, alpha in ((4096, 1e-4), (2048, 2e-4), (1540, 2e-4)):
        w = _case(wl.LINEAR, 6000, p, 3000, 1024, T=1, R=1, alpha=alpha, x_cov="identity")
        X, y = wl.dataset(w)
        want = oracle_run(w, X, y)
        for G, chain in ((1, 1), (3, 1), (8, 1), (48, 1), (256, 1), (64, 2)):
            got, st = gpu_run(w, X, y, n_workgroups=G, chain=chain)
            assert st.n_workgroups == G and st.threads_per_group == _wide_threads(G, chain)
            assert rel_l2(got, want) <= TOL, (p, G, chain)


@pytest.mark.parametrize("model,p,n,G", [(wl.LINEAR, 4096, 1000, 5), (wl.LOGISTIC, 4096, 700, 24), (wl.LINEAR, 2052, 900, 40),
                                         (wl.LOGISTIC, 1028, 512, 0), (wl.LINEAR, 3000, 333, 2), (wl.LINEAR, 4096, 100, 16),
                                         (wl.LOGISTIC, 2048, 2500, 256), (wl.LINEAR, 4092, 1111, 30)])
def test_wide_rows_rows_in_flight_across_steps(model, p, n, G):
    """Wide rows over several workgroups, both kernels (fewer than eight workgroups: two rows per wavefront in flight;
    eight or more: rows split over the wavefronts of a workgroup, groups of rows in flight, exchange wavefront).
    Steps that end on every slot of the ring, one group per step, workgroups without a row in a step, a ragged
    last batch, several passes and buffers, columns that do not fill the last chunk, a requested workgroup count that
    is not a multiple of eight (rounded down)."""
    w = _case(model, 5000, p, 2500, n, T=2, R=2, alpha=(0.2 / p) if model == wl.LINEAR else 0.05, x_cov="identity")
    X, y = wl.dataset(w)
    want = oracle_run(w, X, y)
    got, st = gpu_run(w, X, y, n_workgroups=G, chain=1)
    assert st.threads_per_group == _wide_threads(st.n_workgroups, 1) and st.n_workgroups > 1
    assert G < 8 or st.n_workgroups % 8 == 0
    assert rel_l2(got, want) <= TOL, (p, n, st.n_workgroups)
    again, _ = gpu_run(w, X, y, n_workgroups=G, chain=1, resident=True)
    assert np.array_equal(got, again)


def test_wide_rows_one_step_per_launch_and_one_row_per_wavefront():
    """The smallest launches of the wide-row kernel: a single mini-batch per buffer and pass (the refill two groups ahead
    then always points past the launch), and batches smaller than the number of row slots."""
    for p, N0, n, T, G in ((4096, 1500, 1500, 1, 8), (2048, 600, 600, 2, 16), (4096, 40, 40, 1, 2), (1028, 100, 7, 3, 4)):
        w = _case(wl.LINEAR, 2 * N0, p, N0, n, T=T, R=2, alpha=0.2 / p, x_cov="identity")
        X, y = wl.dataset(w)
        want = oracle_run(w, X, y)
        got, st = gpu_run(w, X, y, n_workgroups=G, chain=1)
        assert st.threads_per_group == _wide_threads(G, 1) and st.n_workgroups == G
        assert rel_l2(got, want) <= TOL, (p, N0, n, T, G)


def test_edge_cases():
    for N, N0, n in [(1, 1, 1), (5, 5, 8), (64, 64, 64), (65, 64, 64), (1000, 1000, 1000), (999, 500, 1)]:
        w = _case(wl.LINEAR, N, 6, N0, min(n, N0), T=3, R=2, alpha=0.05, x_cov="identity")
        X, y = wl.dataset(w)
        want = oracle_run(w, X, y)
        for chain in (1, 3):
            got, _ = gpu_run(w, X, y, chain=chain)
            assert rel_l2(got, want) <= TOL, (N, N0, n, chain)


def test_resident_path_equals_loader_path_bitwise_and_is_reproducible():
    w = _case(wl.LOGISTIC, 20_000, 200, 8000, 1000, T=2, R=2, alpha=0.1)
    X, y = wl.dataset(w)
    a, _ = gpu_run(w, X, y)
    b, _ = gpu_run(w, X, y)
    c, _ = gpu_run(w, X, y, resident=True)
    assert np.array_equal(a, b) and np.array_equal(a, c)


def test_fixed_partition_mode():
    from oracle import bmgd as O
    w = _case(wl.LINEAR, 3000, 20, 1000, 100, T=3, R=3, alpha=0.02)
    X, y = wl.dataset(w)
    want = oracle_run(w, X, y, reshuffle=O.FIXED)
    for chain in (1, 3):
        got, _ = gpu_run(w, X, y, reshuffle=1, chain=chain)
        assert rel_l2(got, want) <= TOL


def test_initial_value_and_resume():
    import paper_2312_08728_amd as B
    w = _case(wl.LINEAR, 4000, 30, 1000, 100, T=2, R=1, alpha=0.02)
    X, y = wl.dataset(w)
    th0 = np.linspace(-1, 1, w.p).astype(np.float32)
    want = oracle_run(w, X, y, theta0=th0)
    got, _ = gpu_run(w, X, y, theta0=th0)
    assert rel_l2(got, want) <= TOL
    # stop after two buffers, carry (theta, buffer counter) into a new context, finish there
    import torch
    s = torch.cuda.Stream()
    xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    c1 = B.Context(w.p, w.N0, w.n, w.alpha, w.T)
    c1.set_theta(th0)
    for k in range(2):
        c1.run_device_buffer(xd[k * 1000:(k + 1) * 1000], yd[k * 1000:(k + 1) * 1000], 1000, s)
    mid = c1.get_theta()
    c1.close()
    c2 = B.Context(w.p, w.N0, w.n, w.alpha, w.T)
    c2.set_theta(mid)
    c2.set_position(2)
    for k in range(2, 4):
        c2.run_device_buffer(xd[k * 1000:(k + 1) * 1000], yd[k * 1000:(k + 1) * 1000], 1000, s)
    fin = c2.get_theta()
    c2.close()
    assert np.array_equal(fin, got)


def test_schedules_of_learning_rate_and_passes():
    """alpha_r and T_r changing with the iteration r (Theorem 4; stage-wise T of Section 4)."""
    import torch
    import paper_2312_08728_amd as B
    from oracle import bmgd as O
    w = _case(wl.LOGISTIC, 6000, 40, 2000, 250, T=3, R=3, alpha=0.2)
    X, y = wl.dataset(w)
    alphas, passes = [0.2, 0.2 / 2 ** 0.5, 0.2 / 3 ** 0.5], [3, 2, 1]
    ref = O.BMGD(w.model, w.p, w.n, alphas[0], passes[0])
    ctx = B.Context(w.p, w.N0, w.n, alphas[0], passes[0], model=w.model)
    xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    s = torch.cuda.Stream()
    for r in range(3):
        ref.alpha, ref.T = alphas[r], passes[r]
        ctx.set_lr(alphas[r])
        ctx.set_passes(passes[r])
        for k in range(3):
            ref.run_buffer(X[k * 2000:(k + 1) * 2000], y[k * 2000:(k + 1) * 2000])
            ctx.run_device_buffer(xd[k * 2000:(k + 1) * 2000], yd[k * 2000:(k + 1) * 2000], 2000, s)
    got = ctx.get_theta()
    st = ctx.stats()
    ctx.close()
    assert st.steps == 3 * 8 * (3 + 2 + 1)
    assert rel_l2(got, ref.theta) <= TOL
    assert B.bmgd_set_lr(None, 0.1) == B.BMGD_EINVAL


@pytest.mark.parametrize("model,p,n,chain", [(wl.LOGISTIC, 40, 250, 1), (wl.LOGISTIC, 200, 512, 1), (wl.LINEAR, 1024, 500, 1),
                                             (wl.LINEAR, 2304, 600, 1), (wl.LINEAR, 40, 250, 3), (wl.LINEAR, 100, 300, 3), (wl.LOGISTIC, 40, 250, 2)])
def test_learning_rate_per_update(model, p, n, chain):
    """A cosine table of learning rates over the updates of the whole run (Section 4.4), shorter than the run so that
    its last value has to persist, crossing passes, launches (T = 5 > 4 passes per launch) and buffers; then cleared."""
    import torch
    import paper_2312_08728_amd as B
    from oracle import bmgd as O
    w = _case(model, 6000, p, 2000, n, T=5, R=1, alpha=0.5 / (p + 10) if model == wl.LINEAR else 0.2, x_cov="identity")
    X, y = wl.dataset(w)
    updates = 3 * 5 * (-(-2000 // n))
    base = w.alpha
    table = [base * (0.1 + 0.9 * 0.5 * (1 + np.cos(np.pi * u / (updates - 20)))) for u in range(updates - 20)]
    ref = O.BMGD(w.model, w.p, w.n, 7.0, w.T)                   # 7.0: never used while the table is set
    ref.set_lr_schedule(np.asarray(table, dtype=np.float32))    # the library holds the table in fp32
    ctx = B.Context(w.p, w.N0, w.n, 7.0, w.T, model=w.model, chain=chain)
    ctx.set_lr_schedule(table)
    xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    s = torch.cuda.Stream()
    for k in range(3):
        ref.run_buffer(X[k * 2000:(k + 1) * 2000], y[k * 2000:(k + 1) * 2000])
        ctx.run_device_buffer(xd[k * 2000:(k + 1) * 2000], yd[k * 2000:(k + 1) * 2000], 2000, s)
    got = ctx.get_theta()
    assert ctx.stats().steps == updates
    assert rel_l2(got, ref.theta) <= TOL
    # cleared: the constant rate applies again
    ref.set_lr_schedule(None); ref.alpha = base
    ctx.set_lr_schedule(None); ctx.set_lr(base)
    ref.run_buffer(X[:2000], y[:2000])
    ctx.run_device_buffer(xd[:2000], yd[:2000], 2000, s)
    assert rel_l2(ctx.get_theta(), ref.theta) <= TOL
    assert B.bmgd_set_lr_schedule(ctx.h, np.array([0.1, -1.0], dtype=np.float32), 2) == B.BMGD_EINVAL
    assert B.bmgd_set_lr_schedule(ctx.h, None, 3) == B.BMGD_EINVAL
    ctx.close()


def test_loader_ordering_under_overlap():
    """Many large buffers through the two-slot loader with copies and compute overlapping on two streams must
    give, bit for bit, what the resident path gives: a run that read a slot before its copy finished, or a copy
    that overwrote a slot still being read, would change theta."""
    w = _case(wl.LOGISTIC, 800_000, 200, 200_000, 4096, T=1, R=3, alpha=0.1)
    X, y = wl.dataset(w)
    a, sa = gpu_run(w, X, y)
    b, _ = gpu_run(w, X, y, resident=True)
    assert np.array_equal(a, b)
    assert sa.h2d_bytes == 3 * (X.nbytes + y.nbytes)            # loads do not depend on the number of passes
    assert sa.copy_ms > 0 and sa.compute_ms > 0 and sa.wait_ms >= 0


def test_device_side_wait_is_bounded():
    """With a 1 us limit on device-side waits some workgroup is bound to give up while it waits for the others:
    the kernel must exit by itself, the next blocking call must report it, and the library must stay usable."""
    import torch
    import paper_2312_08728_amd as B
    w = _case(wl.LINEAR, 20_000, 100, 20_000, 250, T=4, R=1, alpha=0.01)
    X, y = wl.dataset(w)
    xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    c = B.Context(w.p, w.N0, w.n, w.alpha, w.T, n_workgroups=64, barrier_timeout_us=1, chain=B.BMGD_CHAIN_PERSISTENT)
    assert B.bmgd_run_device_buffer(c.h, xd, yd, w.N0, None) == B.BMGD_OK
    out = np.zeros(w.p, dtype=np.float32)
    assert B.bmgd_get_theta(c.h, out, w.p) == B.BMGD_EHIP
    assert "barrier_timeout_us" in B.bmgd_last_error(c.h)
    # theta is undefined now: runs are refused until it has been set again, then the context works as before
    assert B.bmgd_run_device_buffer(c.h, xd, yd, w.N0, None) == B.BMGD_ESTATE
    assert "bmgd_set_theta" in B.bmgd_last_error(c.h)
    c.set_theta(np.zeros(w.p, dtype=np.float32))
    c.set_position(0)
    assert B.bmgd_run_device_buffer(c.h, xd, yd, w.N0, None) == B.BMGD_OK      # accepted (and gives up again: same limit)
    assert B.bmgd_sync(c.h) == B.BMGD_EHIP
    c.set_theta(np.zeros(w.p, dtype=np.float32))                               # the failure was reported: plain success
    assert np.array_equal(c.get_theta(), np.zeros(w.p, dtype=np.float32))
    c.close()
    got, _ = gpu_run(w, X, y, n_workgroups=64, chain=1)          # default limit: same shape runs to the end
    assert rel_l2(got, oracle_run(w, X, y)) <= TOL


def test_error_paths():
    import torch
    import paper_2312_08728_amd as B
    c = B.Context(8, 100, 10, 0.1, 1)
    x = torch.zeros(100, 8).pin_memory()
    y = torch.zeros(100).pin_memory()
    assert B.bmgd_run_buffer(c.h, None) == B.BMGD_ESTATE
    assert B.bmgd_load_buffer_async(c.h, x, y, 101, None) == B.BMGD_EINVAL
    assert B.bmgd_load_buffer_async(c.h, x, y, 0, None) == B.BMGD_EINVAL
    assert B.bmgd_load_buffer_async(c.h, None, y, 10, None) == B.BMGD_EINVAL
    assert B.bmgd_load_buffer_async(c.h, x, y, 100, None) == B.BMGD_OK
    assert B.bmgd_load_buffer_async(c.h, x, y, 100, None) == B.BMGD_ESTATE
    assert "already loaded" in B.bmgd_last_error(c.h)
    assert B.bmgd_run_buffer(c.h, None) == B.BMGD_OK
    out = np.zeros(9, dtype=np.float32)
    assert B.bmgd_get_theta(c.h, out, 9) == B.BMGD_EINVAL
    assert B.bmgd_get_theta(c.h, out, 8) == B.BMGD_OK
    assert B.bmgd_set_lr(c.h, 0.0) == B.BMGD_EINVAL and B.bmgd_set_lr(c.h, float('nan')) == B.BMGD_EINVAL
    assert B.bmgd_set_passes(c.h, 0) == B.BMGD_EINVAL
    c.close()


@pytest.mark.parametrize("kw", [dict(model=wl.LINEAR, p=40, chain=0), dict(model=wl.LOGISTIC, p=200, chain=1),
                                dict(model=wl.LINEAR, p=40, chain=3, optimizer=3)])
def test_caller_provided_workspace(kw):
    """Everything the context needs on the device lives in memory the caller allocates (bmgd_workspace_bytes), here a
    torch tensor with guard bytes on both sides that must come back untouched; results equal the library-owned run."""
    import torch
    import paper_2312_08728_amd as B
    model, p, chain = kw["model"], kw["p"], kw["chain"]
    opt = kw.get("optimizer", 0)
    w = _case(model, 4000, p, 2000, 250, T=5, R=1, alpha=0.01, x_cov="identity")
    X, y = wl.dataset(w)
    xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    s = torch.cuda.Stream()

    def run(**extra):
        ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T, model=model, chain=chain, optimizer=opt, **extra)
        for k in range(2):
            ctx.run_device_buffer(xd[k * 2000:(k + 1) * 2000], yd[k * 2000:(k + 1) * 2000], 2000, s)
        th = ctx.get_theta()
        ctx.close()
        return th

    cfg = B.bmgd_default_config()
    cfg.p, cfg.buffer_n, cfg.batch_n, cfg.lr, cfg.passes = w.p, w.N0, w.n, w.alpha, w.T
    cfg.model, cfg.chain, cfg.optimizer = model, chain, opt
    need = B.bmgd_workspace_bytes(cfg)
    assert need > 0 and need % 256 == 0
    guard = 4096
    raw = torch.full((need + 2 * guard + 256,), 0x5A, dtype=torch.uint8, device="cuda")
    off = (-raw.data_ptr() - guard) % 256 + guard                 # 256-byte aligned start behind the front guard
    ws = raw[off:off + need]
    got = run(workspace=ws, workspace_bytes=need)
    torch.cuda.synchronize()
    assert bool((raw[:off] == 0x5A).all()) and bool((raw[off + need:] == 0x5A).all())
    assert np.array_equal(got, run())
    with pytest.raises(B.BmgdError):
        B.Context(w.p, w.N0, w.n, w.alpha, w.T, model=model, chain=chain, optimizer=opt, workspace=ws, workspace_bytes=need - 256)


@pytest.mark.parametrize("chain,resident", [(3, True), (1, True), (2, True), (3, False)])
def test_ten_thousand_runs_without_a_blocking_call(chain, resident):
    """The library folds the events of old runs by itself once some thousand are open; results and counters
    must not depend on when that happens."""
    w = _case(wl.LINEAR, 640, 8, 64, 16, T=1, R=1000, alpha=0.01)
    X, y = wl.dataset(w)
    want = oracle_run(w, X, y)
    got, st = gpu_run(w, X, y, resident=resident, chain=chain)
    assert st.chain == chain
    assert st.buffers_run == 10_000 and st.steps == 40_000
    assert st.chain_launches == 10_000          # one timed launch (or chunk of launches) per run at T = 1
    if chain == 3:
        assert st.prep_launches == 10_000
    assert st.compute_ms > 0 and st.chain_ms > 0
    assert rel_l2(got, want) <= TOL
