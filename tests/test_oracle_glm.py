"""Pins for the oracle's logistic and softmax paths (Section 3.2.3: the GLM loss and its
derivative; Section 4.1: the logistic data model)."""
import math

import numpy as np
import pytest
from scipy import optimize, special

from oracle import bmgd, perm as P

LOGI, SOFT = bmgd.LOGISTIC, bmgd.SOFTMAX


def _logistic_data(N, p, seed=0):
    g = np.random.default_rng(seed)
    X = g.standard_normal((N, p))
    th = g.standard_normal(p) / np.sqrt(p)
    y = (g.random(N) < special.expit(X @ th)).astype(np.float32)
    return X.astype(np.float32), y, th


def _softmax_data(N, p, C, seed=0):
    g = np.random.default_rng(seed)
    X = g.standard_normal((N, p))
    W = g.standard_normal((p, C))
    y = np.argmax(X @ W + g.gumbel(size=(N, C)), axis=1).astype(np.int32)
    return X.astype(np.float32), y, W


def test_losses_match_library_routines():
    X, y, _ = _logistic_data(200, 5, seed=1)
    th = np.linspace(-2, 2, 5)
    u = X.astype(np.float64) @ th
    want = -np.mean(y * special.log_expit(u) + (1 - y) * special.log_expit(-u))
    assert abs(bmgd.loss(LOGI, X.astype(np.float64), y.astype(np.float64), th) - want) < 1e-13
    Xs, ys, _ = _softmax_data(150, 4, 6, seed=2)
    W = np.random.default_rng(3).standard_normal((4, 6)) * 3
    lp = special.log_softmax(Xs.astype(np.float64) @ W, axis=1)
    want = -np.mean(lp[np.arange(150), ys])
    assert abs(bmgd.loss(SOFT, Xs.astype(np.float64), ys, W) - want) < 1e-13
    assert np.allclose(bmgd.sigmoid(np.array([-800.0, -3.0, 0.0, 3.0, 800.0])),
                       special.expit(np.array([-800.0, -3.0, 0.0, 3.0, 800.0])), rtol=1e-15, atol=0)
    U = np.random.default_rng(4).standard_normal((7, 9)) * 50
    assert np.allclose(bmgd.softmax_rows(U), special.softmax(U, axis=1), rtol=1e-13, atol=1e-300)


@pytest.mark.parametrize("model", [bmgd.LINEAR, LOGI, SOFT])
def test_gradient_matches_central_differences(model):
    g = np.random.default_rng(7)
    if model == SOFT:
        X, y, _ = _softmax_data(40, 3, 4, seed=5)
        th = g.standard_normal((3, 4))
        y = y
    else:
        X, y, _ = _logistic_data(40, 3, seed=5)
        y = y.astype(np.float64) if model == LOGI else g.standard_normal(40)
        th = g.standard_normal(3)
    Xd = X.astype(np.float64)
    grad = bmgd.minibatch_gradient(model, Xd, y, th)
    num = np.zeros_like(th)
    eps = 1e-6
    it = np.nditer(th, flags=["multi_index"])
    for _ in it:
        e = np.zeros_like(th)
        e[it.multi_index] = eps
        num[it.multi_index] = (bmgd.loss(model, Xd, y, th + e) - bmgd.loss(model, Xd, y, th - e)) / (2 * eps)
    assert np.linalg.norm(grad - num) < 1e-7 * np.linalg.norm(num)


def test_logistic_full_batch_reaches_mle():
    """Full-batch descent must land on the maximum-likelihood estimate found by Newton's method
    (textbook IRLS, written here) and by a library optimiser."""
    N, p = 500, 4
    X, y, _ = _logistic_data(N, p, seed=11)
    Xd, yd = X.astype(np.float64), y.astype(np.float64)
    beta = np.zeros(p)
    for _ in range(50):
        mu = special.expit(Xd @ beta)
        H = (Xd * (mu * (1 - mu))[:, None]).T @ Xd
        beta = beta + np.linalg.solve(H, Xd.T @ (yd - mu))
    res = optimize.minimize(lambda b: -np.sum(yd * special.log_expit(Xd @ b) + (1 - yd) * special.log_expit(-Xd @ b)),
                            np.zeros(p), method="BFGS", options={"gtol": 1e-10})
    assert np.linalg.norm(res.x - beta) < 1e-5
    th = bmgd.run(LOGI, X, y, N0=N, n=N, alpha=2.0, T=200, R=10)
    assert np.linalg.norm(th - beta) < 1e-9
    assert np.linalg.norm(bmgd.minibatch_gradient(LOGI, Xd, yd, th)) < 1e-10


def test_logistic_full_batch_loss_non_increasing():
    N, p = 300, 5
    X, y, _ = _logistic_data(N, p, seed=12)
    Xd, yd = X.astype(np.float64), y.astype(np.float64)
    Lsmooth = 0.25 * np.linalg.eigvalsh(Xd.T @ Xd / N)[-1]
    st = bmgd.BMGD(LOGI, p, n=N, alpha=1.0 / Lsmooth, T=40)
    nll = lambda th: -np.mean(yd * special.log_expit(Xd @ th) + (1 - yd) * special.log_expit(-Xd @ th))
    losses = [nll(st.theta)]
    st.run_buffer(X, y, on_step=lambda s: losses.append(nll(s.theta)))
    assert np.all(np.diff(losses) <= 1e-15) and losses[-1] < losses[0]


def test_minibatch_global_loss_decreases_over_iterations():
    N, p = 2000, 6
    X, y, _ = _logistic_data(N, p, seed=13)
    Xd, yd = X.astype(np.float64), y.astype(np.float64)
    nll = lambda th: -np.mean(yd * special.log_expit(Xd @ th) + (1 - yd) * special.log_expit(-Xd @ th))
    marks = []
    bmgd.run(LOGI, X, y, N0=500, n=50, alpha=0.02, T=2, R=6,
             on_buffer=lambda r, k, st: marks.append(nll(st.theta)) if k == 3 else None)
    assert len(marks) == 6 and np.all(np.diff(marks) < 0)


def test_softmax_invariants():
    N, p, C = 240, 5, 7
    X, y, _ = _softmax_data(N, p, C, seed=21)
    Pm = bmgd.softmax_rows(X.astype(np.float64) @ np.random.default_rng(1).standard_normal((p, C)))
    assert np.allclose(Pm.sum(axis=1), 1.0, atol=1e-14)
    sums = []
    W = bmgd.run(SOFT, X, y, N0=120, n=16, alpha=0.3, T=2, R=2, C=C,
                 on_buffer=lambda r, k, st: sums.append(st.theta.sum(axis=1)))
    # every class gets the same x-weighted mass removed and added: the class-sum of W never moves
    for s in sums:
        assert np.allclose(s, 0.0, atol=1e-13)
    assert np.linalg.norm(W) > 0.1


def test_two_class_softmax_is_logistic_with_twice_the_rate():
    N, p = 200, 4
    X, y, _ = _logistic_data(N, p, seed=22)
    alpha = 0.07
    W = bmgd.run(SOFT, X, y.astype(np.int32), N0=100, n=10, alpha=alpha, T=2, R=2, C=2, seed=3)
    th = bmgd.run(LOGI, X, y, N0=100, n=10, alpha=2 * alpha, T=2, R=2, seed=3)
    assert np.allclose(W[:, 1] - W[:, 0], th, rtol=0, atol=1e-13)


def test_hand_unrolled_logistic_and_softmax():
    """N0 = 4, p = 2, n = 2, T = 2, every update written with scalars and math.exp (eq. (2.1))."""
    X = [[1.0, 2.0], [0.5, -1.0], [-1.5, 0.25], [2.0, 1.0]]
    y = [1, 0, 0, 1]
    alpha = 0.5
    a = b = 0.0
    for t in (1, 2):
        pm = P.perm_scalar(5, 0, t, 4)
        for m in range(2):
            ga = gb = 0.0
            for i in (pm[2 * m], pm[2 * m + 1]):
                u = X[i][0] * a + X[i][1] * b
                r = 1.0 / (1.0 + math.exp(-u)) - y[i]
                ga += r * X[i][0] / 2
                gb += r * X[i][1] / 2
            a, b = a - alpha * ga, b - alpha * gb
    th = bmgd.run(LOGI, np.array(X, dtype=np.float32), np.array(y, dtype=np.float32),
                  N0=4, n=2, alpha=alpha, T=2, R=1, seed=5)
    assert np.allclose(th, [a, b], rtol=0, atol=1e-15)

    cls = [2, 0, 1, 2]
    W = [[0.0] * 3 for _ in range(2)]
    for t in (1, 2):
        pm = P.perm_scalar(5, 0, t, 4)
        for m in range(2):
            G = [[0.0] * 3 for _ in range(2)]
            for i in (pm[2 * m], pm[2 * m + 1]):
                u = [X[i][0] * W[0][c] + X[i][1] * W[1][c] for c in range(3)]
                e = [math.exp(v - max(u)) for v in u]
                pr = [v / sum(e) for v in e]
                for c in range(3):
                    r = pr[c] - (1.0 if cls[i] == c else 0.0)
                    G[0][c] += r * X[i][0] / 2
                    G[1][c] += r * X[i][1] / 2
            W = [[W[j][c] - alpha * G[j][c] for c in range(3)] for j in range(2)]
    got = bmgd.run(SOFT, np.array(X, dtype=np.float32), np.array(cls, dtype=np.int32),
                   N0=4, n=2, alpha=alpha, T=2, R=1, C=3, seed=5)
    assert np.allclose(got, W, rtol=0, atol=1e-15)


def test_bf16_storage_is_widened_exactly():
    import workloads as wl
    v = np.array([1.0, -2.5, 3.140625, 1e-3, 65504.0], dtype=np.float32)
    bits = wl.f32_to_bf16_bits(v)
    assert np.array_equal(bmgd.to_f64(bits), wl.bf16_bits_to_f32(bits).astype(np.float64))
    # round-to-nearest-even on the 16 dropped bits
    assert wl.f32_to_bf16_bits(np.array([1.0 + 2.0 ** -8], dtype=np.float32))[0] == 0x3F80      # tie -> even
    assert wl.f32_to_bf16_bits(np.array([1.0 + 3 * 2.0 ** -8], dtype=np.float32))[0] == 0x3F82  # tie -> even (up)
    assert wl.f32_to_bf16_bits(np.array([1.0 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32))[0] == 0x3F81
