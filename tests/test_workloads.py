"""The synthetic inputs have the shapes and distributions the run shapes call for
(Section 4.1's simulation design) and any row block can be regenerated on its own."""
import numpy as np

import workloads as wl


def test_config_table():
    c = wl.CONFIGS
    assert [c[k].M for k in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5")] == [20, 100, 245, 31, 98]
    assert [c[k].K for k in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5")] == [5, 10, 10, 8, 10]
    assert [c[k].steps for k in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5")] == [2000, 15000, 14700, 992, 3920]
    assert [c[k].sample_gradients for k in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5")] == \
        [200_000, 15_000_000, 60_000_000, 8_000_000, 4_000_000]


def test_blocks_regenerate_identically_and_thread_count_does_not_matter():
    w = wl.CONFIGS["cfg2"].scaled(N=30_000)
    X, y = wl.rows(w, 0, 30_000, threads=1)
    X2, y2 = wl.rows(w, 7_000, 19_000, threads=4)
    assert np.array_equal(X[7_000:19_000], X2) and np.array_equal(y[7_000:19_000], y2)
    assert X.dtype == np.float32 and y.dtype == np.float32


def test_ar1_covariance_and_noise_level():
    w = wl.CONFIGS["cfg2"].scaled(N=60_000, p=12)
    X, y = wl.dataset(w)
    S = np.cov(X.astype(np.float64), rowvar=False)
    want = 0.5 ** np.abs(np.subtract.outer(np.arange(12), np.arange(12)))
    assert np.abs(S - want).max() < 0.03
    resid = y - X.astype(np.float64) @ wl.true_theta(w)
    assert abs(resid.std() - 1.0) < 0.02


def test_logistic_labels_follow_the_link():
    w = wl.CONFIGS["cfg3"].scaled(N=50_000, p=8)
    X, y = wl.dataset(w)
    assert set(np.unique(y)) == {0.0, 1.0}
    eta = X.astype(np.float64) @ wl.true_theta(w)
    hi, lo = y[eta > 1.0].mean(), y[eta < -1.0].mean()
    assert hi > 0.75 and lo < 0.25


def test_sparse_truth_and_softmax_shapes():
    th = wl.true_theta(wl.CONFIGS["cfg4"])
    assert th.shape == (4096,) and np.count_nonzero(th) == 64 and np.abs(th).max() <= 1.0
    w = wl.CONFIGS["cfg5"].scaled(N=3_000, p=48, C=10)
    X, y = wl.dataset(w)
    assert X.dtype == np.uint16 and y.dtype == np.int32 and 0 <= y.min() and y.max() < 10
    xf = wl.bf16_bits_to_f32(X)
    assert abs(xf.std() - 1.0) < 0.02
    assert np.array_equal(wl.f32_to_bf16_bits(xf), X)            # stored values are exact bf16
    scores = xf.astype(np.float64) @ wl.true_theta(w)
    assert (np.argmax(scores, axis=1) == y).mean() > 0.2          # labels carry signal (chance = 0.1)
