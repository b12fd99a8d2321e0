"""The persistent kernel for rows of up to 1024 floats whose share of a step fits the registers (eight row wavefronts
with two alternating groups of rows, four exchange wavefronts): every register shape it is built for, against the oracle."""
import numpy as np
import pytest

import workloads as wl
from gpu_util import gpu_run, oracle_run, rel_l2, coord_err

pytestmark = pytest.mark.gpu

TOL = 1e-4
NARROW_THREADS = 768          # 12 wavefronts: what tells this kernel from the others in the statistics


def _case(model, N, p, N0, n, T, R, alpha):
    base = wl.CONFIGS["cfg3" if model == wl.LOGISTIC else "cfg2"]
    return base.scaled(name="case", N=N, p=p, N0=N0, n=n, T=T, R=R, alpha=alpha, x_cov="identity")


# (model, p, n, G, N0): floats per load V, chunks per lane CPL, rows per lane slot PF, lanes per row L that result
SHAPES = [
    (wl.LOGISTIC, 200, 4096, 256, 10_000),   # V 4, CPL 1, PF 2, L 64: cfg3's shape; a short last mini-batch; 9 steps per launch (odd)
    (wl.LINEAR, 100, 1000, 64, 6_000),       # V 4, CPL 1, PF 1, L 32: two rows side by side in a wavefront
    (wl.LINEAR, 36, 5000, 128, 12_000),      # V 4, CPL 1, PF 2, L 16: four rows side by side
    (wl.LOGISTIC, 1024, 2048, 256, 5_000),   # V 4, CPL 4, PF 1: the widest rows
    (wl.LINEAR, 512, 4096, 256, 9_000),      # V 4, CPL 2, PF 2
    (wl.LINEAR, 250, 3000, 128, 7_000),      # V 2, CPL 2, PF 4
    (wl.LOGISTIC, 70, 8000, 128, 17_000),    # V 2, CPL 1, PF 8: the most rows per lane slot
    (wl.LINEAR, 600, 128, 8, 1_000),         # V 4, CPL 4, PF 2 on the fewest workgroups
    (wl.LOGISTIC, 200, 1400, 24, 5_000),     # V 4, CPL 1, PF 8 on 24 workgroups: 32 floats of rows per lane and group
]


@pytest.mark.parametrize("model,p,n,G,N0", SHAPES)
def test_register_shapes_against_the_oracle(model, p, n, G, N0):
    import paper_2312_08728_amd as B
    w = _case(model, 2 * N0 - 77, p, N0, n, T=3, R=2, alpha=0.5 / (p + 10) if model == wl.LINEAR else 0.1)
    X, y = wl.dataset(w)
    want = oracle_run(w, X, y)
    got, st = gpu_run(w, X, y, n_workgroups=G, chain=B.BMGD_CHAIN_PERSISTENT)
    assert st.threads_per_group == NARROW_THREADS and st.n_workgroups == G, (st.threads_per_group, st.n_workgroups)
    assert st.steps == w.steps
    assert rel_l2(got, want) <= TOL and coord_err(got, want) <= 10 * TOL


@pytest.mark.parametrize("optimizer", [1, 2, 3])
def test_update_rules_with_state(optimizer):
    """Momentum, NAG and Adam keep their state per coordinate in global memory; the first exchange wavefront of the
    workgroup that owns a slice updates it."""
    import paper_2312_08728_amd as B
    from oracle import bmgd as O
    w = _case(wl.LOGISTIC, 12_000, 200, 6_000, 2048, T=2, R=2, alpha=0.01 if optimizer == 3 else 0.05)
    X, y = wl.dataset(w)
    ref = O.BMGD(w.model, w.p, w.n, w.alpha, w.T)
    ref.set_optimizer(optimizer)
    for _ in range(w.R):
        for k in range(2):
            ref.run_buffer(X[k * 6000:(k + 1) * 6000], y[k * 6000:(k + 1) * 6000])
    got, st = gpu_run(w, X, y, n_workgroups=64, chain=B.BMGD_CHAIN_PERSISTENT, optimizer=optimizer)
    assert st.threads_per_group == NARROW_THREADS
    assert rel_l2(got, ref.theta) <= TOL


def test_is_reproducible_and_equals_the_loader_path():
    import paper_2312_08728_amd as B
    w = _case(wl.LOGISTIC, 30_000, 200, 10_000, 4096, T=2, R=2, alpha=0.1)
    X, y = wl.dataset(w)
    a, sa = gpu_run(w, X, y, chain=B.BMGD_CHAIN_PERSISTENT)
    b, _ = gpu_run(w, X, y, chain=B.BMGD_CHAIN_PERSISTENT, resident=True)
    c, _ = gpu_run(w, X, y, chain=B.BMGD_CHAIN_PERSISTENT)
    assert sa.threads_per_group == NARROW_THREADS
    assert np.array_equal(a, b) and np.array_equal(a, c)


def test_other_kernels_keep_their_cases():
    """Few workgroups, sums small enough for every workgroup to add up itself, odd p, a step that does not fit the
    registers: the general kernel (1024 threads)."""
    import paper_2312_08728_amd as B
    for kw, p, n, N0 in ((dict(n_workgroups=4), 200, 1000, 4000),          # fewer than eight workgroups
                         (dict(n_workgroups=16), 100, 1000, 4000),         # 16 * 100 words: one trip, redundant sums
                         (dict(n_workgroups=64), 201, 1000, 4000),         # odd p
                         (dict(n_workgroups=8), 200, 4096, 9000)):         # 64 slots: 64 rows per slot
        w = _case(wl.LINEAR, 2 * N0, p, N0, n, T=2, R=1, alpha=0.5 / (p + 10))
        X, y = wl.dataset(w)
        want = oracle_run(w, X, y)
        got, st = gpu_run(w, X, y, chain=B.BMGD_CHAIN_PERSISTENT, **kw)
        assert st.threads_per_group == 1024, (kw, p, st.threads_per_group)
        assert rel_l2(got, want) <= TOL


def test_more_passes_than_one_launch_holds_and_a_rate_per_update():
    """Five passes are two launches (four passes, then one): tags, versions and the position in the table of learning
    rates carry over from launch to launch."""
    import torch
    import paper_2312_08728_amd as B
    from oracle import bmgd as O
    w = _case(wl.LOGISTIC, 12_000, 200, 6_000, 2048, T=5, R=1, alpha=0.1)
    X, y = wl.dataset(w)
    steps = 2 * 5 * 3
    sched = (0.1 * (0.5 + 0.5 * np.cos(np.pi * np.arange(steps) / steps))).astype(np.float32)
    ref = O.BMGD(w.model, w.p, w.n, w.alpha, w.T)
    ref.set_lr_schedule(sched)
    ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T, model=w.model, n_workgroups=64, chain=B.BMGD_CHAIN_PERSISTENT)
    ctx.set_lr_schedule(sched)
    xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    s = torch.cuda.Stream()
    for k in range(2):
        ref.run_buffer(X[k * 6000:(k + 1) * 6000], y[k * 6000:(k + 1) * 6000])
        ctx.run_device_buffer(xd[k * 6000:(k + 1) * 6000], yd[k * 6000:(k + 1) * 6000], 6000, s)
    got = ctx.get_theta()
    st = ctx.stats()
    ctx.close()
    assert st.threads_per_group == NARROW_THREADS and st.steps == steps and st.chain_launches == 4
    assert rel_l2(got, ref.theta) <= TOL
