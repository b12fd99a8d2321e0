"""Parity at the full size of the five run configurations, in the launch configuration bench.py times (same p,
buffer size, mini-batch size, passes, learning rate, automatic workgroup count).

All five run whole (R * K buffer runs at full buffer size; cfg4 and cfg5 together take about two and a half minutes,
most of it the oracle; BMGD_QUICK=1 cuts them to their first 4 and 2 buffer runs).  The estimate is compared
with the oracle after EVERY buffer, by relative L2 error (the stated metric) and by the largest error of a single
coordinate relative to the largest coordinate.  The short-buffer cases at the end are the quick tier."""
import os

import numpy as np
import pytest

import workloads as wl
from gpu_util import gpu_run, oracle_run, parity_after_every_buffer, rel_l2

pytestmark = pytest.mark.gpu

QUICK = os.environ.get("BMGD_QUICK", "") == "1"
TOL_F32 = 1e-4           # fp32 least squares / logistic paths
TOL_BF16 = 2e-3          # softmax: bf16 operands, fp32 accumulation and master weights


def _report(name):
    def say(i, e):
        print(f"{name}: after buffer run {i + 1}: rel-L2 {e[0]:.3e}, largest coordinate error {e[1]:.3e}", flush=True)
    return say


def test_cfg2_whole_run():
    w = wl.CONFIGS["cfg2"]
    X, y = wl.dataset(w)
    want = oracle_run(w, X, y)
    # automatic (the form of eq. (3.1) with steps multiplied in pairs: 300 steps per launch), the plain chain of eq. (3.1),
    # the row form
    for chain in (0, 3, 1):
        got, st = gpu_run(w, X, y, resident=True, chain=chain)
        assert st.chain == {0: 5, 3: 3, 1: 1}[chain]
        assert st.steps == 15_000 and st.sample_gradients == 15_000_000
        assert rel_l2(got, want) <= TOL_F32
        assert np.linalg.norm(got - wl.true_theta(w)) < 0.15  # and it has learnt the coefficients


def test_cfg2_whole_run_theta_after_every_buffer():
    w = wl.CONFIGS["cfg2"]
    errs, st = parity_after_every_buffer(w, w.R * w.K)
    assert st.steps == 15_000 and len(errs) == 50
    assert max(e[0] for e in errs) <= TOL_F32 and max(e[1] for e in errs) <= TOL_F32


def test_cfg3_whole_run_theta_after_every_buffer():
    """Logistic regression, all R * K = 30 buffers of 1,000,000 rows through the pinned-host loader: 14,700 updates."""
    w = wl.CONFIGS["cfg3"]
    errs, st = parity_after_every_buffer(w, w.R * w.K, report=_report("cfg3"))
    assert st.steps == 14_700 and st.sample_gradients == 60_000_000 and st.n_workgroups == 256
    assert st.h2d_bytes == w.R * w.N * (w.p + 1) * 4
    assert max(e[0] for e in errs) <= TOL_F32 and max(e[1] for e in errs) <= TOL_F32


def test_cfg4_whole_run_theta_after_every_buffer():
    """Least squares with p = 4096: all 16 buffer runs (BMGD_QUICK=1: the first 4), each a full 250,000 x 4,096 buffer
    (4.1 GB slot) through the pinned-host loader, both passes, M = 31 with the ragged last mini-batch of 4,240 rows:
    992 updates."""
    w = wl.CONFIGS["cfg4"]
    runs = 4 if QUICK else w.R * w.K
    errs, st = parity_after_every_buffer(w, runs, report=_report("cfg4"))
    assert st.steps == runs * 62 and st.n_workgroups == 256 and st.threads_per_group == 704
    assert st.h2d_bytes == runs * w.N0 * (w.p + 1) * 4
    assert max(e[0] for e in errs) <= TOL_F32 and max(e[1] for e in errs) <= TOL_F32


def test_cfg5_whole_run_theta_after_every_buffer():
    """Softmax regression, 3,072 features x 1,000 classes: all 20 buffer runs (BMGD_QUICK=1: the first 2), each a full
    buffer of 100,000 bf16 rows, both passes, M = 98 with the ragged last mini-batch of 672 rows: 3,920 updates."""
    w = wl.CONFIGS["cfg5"]
    runs = 2 if QUICK else w.R * w.K
    errs, st = parity_after_every_buffer(w, runs, report=_report("cfg5"))
    assert st.steps == runs * 196
    assert max(e[0] for e in errs) <= TOL_BF16 and max(e[1] for e in errs) <= TOL_BF16


# ---- quick tier: the configurations' p, n, T, alpha and ragged tail on a short buffer -----------------------------
def test_cfg3_two_full_buffers():
    w = wl.CONFIGS["cfg3"].scaled(N=2_000_000, R=1)
    X, y = wl.dataset(w)
    want = oracle_run(w, X, y)
    got, st = gpu_run(w, X, y)                                 # through the pinned-host loader
    assert st.steps == 2 * 2 * 245 and st.n_workgroups == 256
    assert rel_l2(got, want) <= TOL_F32


def test_cfg4_shape_short_buffer():
    base = wl.CONFIGS["cfg4"]
    rows = 3 * base.n + 4240                                   # three full mini-batches + cfg4's own ragged tail
    w = base.scaled(N=rows, N0=rows, R=1)
    X, y = wl.dataset(w)
    want = oracle_run(w, X, y)
    got, st = gpu_run(w, X, y, resident=True)
    assert st.steps == 2 * 4 and st.n_workgroups == 256 and st.threads_per_group == 704
    assert rel_l2(got, want) <= TOL_F32


def test_cfg5_shape_short_buffer():
    base = wl.CONFIGS["cfg5"]
    rows = 4 * base.n + 672                                    # four full mini-batches + cfg5's own ragged tail
    w = base.scaled(N=rows, N0=rows, R=1)
    X, y = wl.dataset(w)
    want = oracle_run(w, X, y)
    got, st = gpu_run(w, X, y, resident=True)
    assert st.steps == 2 * 5 and got.shape == (3072, 1000)
    assert rel_l2(got, want) <= TOL_BF16
