"""Parity at the full shapes of the five run configurations, in the launch configuration bench.py times
(same p, mini-batch size, passes, learning rate, automatic workgroup count).  cfg1 and cfg2 run whole
(R * K buffers); cfg3 runs two full-size buffers; cfg4 and cfg5 keep p, n, T, alpha and the ragged last
mini-batch of the configuration but shorten the buffer so that the fp64 oracle finishes in seconds (the
launch shape depends on p and n only).  The chain is sequential, so the checked output is the final theta."""
import numpy as np
import pytest

import workloads as wl
from gpu_util import gpu_run, oracle_run, rel_l2

pytestmark = pytest.mark.gpu


def test_cfg2_whole_run():
    w = wl.CONFIGS["cfg2"]
    X, y = wl.dataset(w)
    want = oracle_run(w, X, y)
    for chain in (0, 1):                                       # automatic (the form of eq. (3.1)), then the row form
        got, st = gpu_run(w, X, y, resident=True, chain=chain)
        assert st.chain == (3 if chain == 0 else 1)
        assert st.steps == 15_000 and st.sample_gradients == 15_000_000
        assert rel_l2(got, want) <= 1e-4
        assert np.linalg.norm(got - wl.true_theta(w)) < 0.15  # and it has learnt the coefficients


def test_cfg3_two_full_buffers():
    w = wl.CONFIGS["cfg3"].scaled(N=2_000_000, R=1)
    X, y = wl.dataset(w)
    want = oracle_run(w, X, y)
    got, st = gpu_run(w, X, y)                                 # through the pinned-host loader
    assert st.steps == 2 * 2 * 245 and st.n_workgroups == 256
    assert rel_l2(got, want) <= 1e-4


def test_cfg4_shape_short_buffer():
    base = wl.CONFIGS["cfg4"]
    rows = 3 * base.n + 4240                                   # three full mini-batches + cfg4's own ragged tail
    w = base.scaled(N=rows, N0=rows, R=1)
    X, y = wl.dataset(w)
    want = oracle_run(w, X, y)
    got, st = gpu_run(w, X, y, resident=True)
    assert st.steps == 2 * 4 and st.n_workgroups == 256 and st.threads_per_group == 512
    assert rel_l2(got, want) <= 1e-4


def test_cfg5_shape_short_buffer():
    base = wl.CONFIGS["cfg5"]
    rows = 4 * base.n + 672                                    # four full mini-batches + cfg5's own ragged tail
    w = base.scaled(N=rows, N0=rows, R=1)
    X, y = wl.dataset(w)
    want = oracle_run(w, X, y)
    got, st = gpu_run(w, X, y, resident=True)
    assert st.steps == 2 * 5 and got.shape == (3072, 1000)
    assert rel_l2(got, want) <= 2e-3
