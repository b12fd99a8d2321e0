"""Pins for the oracle on least squares: closed forms of Section 3.1 (eqs. (3.1)-(3.3),
the stable solution, Theorems 1 and 2) and the OLS estimator."""
import numpy as np
import pytest

from oracle import bmgd, perm as P

LIN = bmgd.LINEAR


def _data(N, p, seed=0, rho=0.5, sigma=1.0):
    g = np.random.default_rng(seed)
    z = g.standard_normal((N, p))
    for j in range(1, p):
        z[:, j] = rho * z[:, j - 1] + np.sqrt(1 - rho * rho) * z[:, j]
    th = g.standard_normal(p) / np.sqrt(p)
    y = z @ th + sigma * g.standard_normal(N)
    return z.astype(np.float32), y.astype(np.float32), th


def test_full_batch_error_propagation_and_ols_limit():
    """One buffer holding all N rows with n = N is full-batch gradient descent:
    theta_j - theta_ols = (I - alpha Sxx)^j (theta_0 - theta_ols)  (eq. (3.1) with M = 1)."""
    N, p = 400, 6
    X, y, _ = _data(N, p)
    Xd, yd = X.astype(np.float64), y.astype(np.float64)
    ols = np.linalg.lstsq(Xd, yd, rcond=None)[0]
    Sxx = Xd.T @ Xd / N
    lam1 = np.linalg.eigvalsh(Sxx)[-1]
    alpha = 1.0 / lam1
    assert 0 < alpha < 2 / lam1                                 # Theorem 1's range
    th0 = np.linspace(-1, 1, p)
    for j in [1, 2, 7, 40]:
        th = bmgd.run(LIN, X, y, N0=N, n=N, alpha=alpha, T=j, R=1, theta0=th0)
        want = ols + np.linalg.matrix_power(np.eye(p) - alpha * Sxx, j) @ (th0 - ols)
        assert np.allclose(th, want, rtol=0, atol=1e-12)
    th = bmgd.run(LIN, X, y, N0=N, n=N, alpha=alpha, T=50, R=40, theta0=th0)
    assert np.linalg.norm(th - ols) < 1e-10 * max(1.0, np.linalg.norm(ols))


def _fixed_partition_matrices(X, y, N0, n, alpha, T, seed):
    """Dense Delta, A, B, C, D of eqs. (3.1)-(3.2) for every buffer, with the partition PERM(seed, k, 0, N0)."""
    Xd, yd = X.astype(np.float64), y.astype(np.float64)
    N, p = Xd.shape
    K = N // N0
    Cs, Ds = [], []
    for k in range(K):
        pm = P.perm(seed, k, 0, N0) + k * N0
        A = np.eye(p)
        B = np.zeros(p)
        for s in range(0, N0, n):
            idx = pm[s:s + n]
            Sxx = Xd[idx].T @ Xd[idx] / len(idx)
            Sxy = Xd[idx].T @ yd[idx] / len(idx)
            Delta = np.eye(p) - alpha * Sxx
            A = Delta @ A                    # later mini-batches act on the left
            B = Delta @ B + Sxy              # B = sum_m (prod_{s>m} Delta_s) Sxy_m
        C = np.linalg.matrix_power(A, T)
        D = sum(np.linalg.matrix_power(A, j) for j in range(T)) @ B
        Cs.append(C)
        Ds.append(D)
    return Cs, Ds


def test_fixed_partition_buffer_map():
    """theta_{r,k} = C^(k) theta_{r,k-1} + alpha D^(k)  (eq. (3.2)) after every buffer."""
    N, p, N0, n, alpha, T, R = 240, 5, 60, 12, 0.07, 3, 3
    X, y, _ = _data(N, p, seed=1)
    Cs, Ds = _fixed_partition_matrices(X, y, N0, n, alpha, T, seed=4)
    th0 = np.arange(p, dtype=np.float64) / p
    seen = []
    bmgd.run(LIN, X, y, N0, n, alpha, T, R, seed=4, reshuffle=bmgd.FIXED, theta0=th0,
             on_buffer=lambda r, k, st: seen.append(st.theta.copy()))
    prev = th0
    K = N // N0
    assert len(seen) == R * K
    for i, got in enumerate(seen):
        k = i % K
        want = Cs[k] @ prev + alpha * Ds[k]
        assert np.allclose(got, want, rtol=0, atol=1e-12)
        prev = got


def test_outer_iteration_reaches_stable_solution():
    """End-of-buffer estimates, stacked over k, converge geometrically to alpha (I - C*)^-1 D*
    (eq. (3.3) and Theorem 1(b))."""
    N, p, N0, n, alpha, T = 300, 4, 100, 20, 0.05, 2
    X, y, _ = _data(N, p, seed=2)
    K = N // N0
    Cs, Ds = _fixed_partition_matrices(X, y, N0, n, alpha, T, seed=9)
    Cstar = np.zeros((K * p, K * p))
    Cstar[0:p, (K - 1) * p:K * p] = Cs[0]
    for k in range(1, K):
        Cstar[k * p:(k + 1) * p, (k - 1) * p:k * p] = Cs[k]
    Dstar = np.concatenate(Ds)
    stable = alpha * np.linalg.solve(np.eye(K * p) - Cstar, Dstar)
    # the stable solution satisfies the per-buffer recursion cyclically
    for k in range(K):
        prev = stable[((k - 1) % K) * p:((k - 1) % K + 1) * p]
        assert np.allclose(stable[k * p:(k + 1) * p], Cs[k] @ prev + alpha * Ds[k], atol=1e-12)
    R = 60
    stacked = np.zeros((R, K * p))
    bmgd.run(LIN, X, y, N0, n, alpha, T, R, seed=9, reshuffle=bmgd.FIXED,
             on_buffer=lambda r, k, st: stacked[r, k * p:(k + 1) * p].__setitem__(slice(None), st.theta))
    err = np.linalg.norm(stacked - stable, axis=1)
    assert err[-1] < 1e-9 * np.linalg.norm(stable) + 1e-12
    live = err[:25]
    ratios = live[1:] / live[:-1]
    assert np.all(ratios < 1.0) and ratios[5:].std() < 0.05      # linear rate, settled
    lam = np.linalg.eigvalsh(X.astype(np.float64).T @ X.astype(np.float64) / N)
    assert 0 < alpha < 2 / lam[-1]


def _stable_distance(X, y, N0, n, alpha, T, seed):
    N, p = X.shape
    K = N // N0
    ols = np.linalg.lstsq(X.astype(np.float64), y.astype(np.float64), rcond=None)[0]
    stacked = np.zeros(K * p)
    last = []
    bmgd.run(LIN, X, y, N0, n, alpha, T, R=int(40 / (alpha * T * 0.5)) // (N // n) + 30, seed=seed,
             reshuffle=bmgd.FIXED,
             on_buffer=lambda r, k, st: stacked.__setitem__(slice(k * p, (k + 1) * p), st.theta))
    return np.linalg.norm(stacked - np.tile(ols, K))


def test_distance_to_ols_scales_with_alpha_T():
    """Theorem 2: the stable solution sits within c * alpha * T of the OLS estimator; and the
    same alpha*T with different T gives similar accuracy (Section 4.1's first finding)."""
    X, y, _ = _data(600, 4, seed=3)
    d1 = _stable_distance(X, y, 200, 20, 0.02, 2, seed=1)
    d2 = _stable_distance(X, y, 200, 20, 0.01, 2, seed=1)
    d4 = _stable_distance(X, y, 200, 20, 0.005, 2, seed=1)
    assert 1.6 < d1 / d2 < 2.5 and 1.6 < d2 / d4 < 2.5
    dT1 = _stable_distance(X, y, 200, 20, 0.02, 1, seed=1)
    dT4 = _stable_distance(X, y, 200, 20, 0.005, 4, seed=1)
    assert 0.5 < dT1 / dT4 < 2.0


def test_full_batch_loss_is_non_increasing():
    N, p = 300, 5
    X, y, _ = _data(N, p, seed=5)
    Xd, yd = X.astype(np.float64), y.astype(np.float64)
    lam1 = np.linalg.eigvalsh(Xd.T @ Xd / N)[-1]
    st = bmgd.BMGD(LIN, p, n=N, alpha=1.5 / lam1, T=30)
    losses = [np.mean((Xd @ st.theta - yd) ** 2)]
    st.run_buffer(X, y, on_step=lambda s: losses.append(np.mean((Xd @ s.theta - yd) ** 2)))
    assert len(losses) == 31 and np.all(np.diff(losses) <= 1e-15)


def test_minibatch_run_approaches_truth_at_statistical_rate():
    import workloads as wl
    w = wl.CONFIGS["cfg1"]
    X, y = wl.dataset(w)
    th = bmgd.run(w.model, X, y, w.N0, w.n, w.alpha, w.T, w.R)
    ols = np.linalg.lstsq(X.astype(np.float64), y.astype(np.float64), rcond=None)[0]
    truth = wl.true_theta(w)
    assert np.linalg.norm(ols - truth) < 4 * np.sqrt(w.p / w.N)
    assert np.linalg.norm(th - truth) < 0.15           # noisy SGD plateau at alpha = 0.05, n = 100


def test_hand_unrolled_tiny_run():
    """N0 = 4, p = 2, n = 2, T = 2 written out with scalars (eq. (2.1))."""
    X = np.array([[1.0, 2.0], [0.5, -1.0], [-1.5, 0.25], [2.0, 1.0]], dtype=np.float32)
    y = np.array([1.0, -2.0, 0.5, 3.0], dtype=np.float32)
    alpha = 0.1
    a, b = 0.0, 0.0
    X32, y32, X, y = X, y, X.tolist(), y.tolist()      # plain Python floats below
    for t in (1, 2):
        pm = P.perm_scalar(0, 0, t, 4)
        for m in range(2):
            i, j = pm[2 * m], pm[2 * m + 1]
            ri = X[i][0] * a + X[i][1] * b - y[i]
            rj = X[j][0] * a + X[j][1] * b - y[j]
            ga = (ri * X[i][0] + rj * X[j][0]) / 2
            gb = (ri * X[i][1] + rj * X[j][1]) / 2
            a, b = a - alpha * ga, b - alpha * gb
    th = bmgd.run(LIN, X32, y32, N0=4, n=2, alpha=alpha, T=2, R=1)
    assert np.allclose(th, [a, b], rtol=0, atol=1e-15)


def test_ragged_last_batch_is_averaged_over_its_own_size():
    X = np.array([[1.0], [2.0], [3.0]], dtype=np.float32)
    y = np.array([1.0, 1.0, 1.0], dtype=np.float32)
    pm = P.perm_scalar(0, 0, 1, 3)
    th = 0.0
    x = [1.0, 2.0, 3.0]
    i, j = pm[0], pm[1]
    th -= 0.1 * ((x[i] * th - 1) * x[i] + (x[j] * th - 1) * x[j]) / 2
    k = pm[2]
    th -= 0.1 * ((x[k] * th - 1) * x[k]) / 1
    got = bmgd.run(LIN, X, y, N0=3, n=2, alpha=0.1, T=1, R=1)
    assert abs(got[0] - th) < 1e-15


def test_per_update_learning_rates_hand_unrolled_and_special_cases():
    """A learning rate per mini-batch update (Theorem 4; cosine schedule of Section 4.4): written out with scalars on
    N0 = 4, p = 1, n = 2 over two buffers; the table's last value persists; a constant table is the constant rate;
    and with full batches and rates 1/lambda on an orthogonal design one update lands on the OLS solution."""
    x = [1.0, -2.0, 0.5, 3.0]
    yv = [0.5, 1.0, -1.0, 2.0]
    X = np.array(x, dtype=np.float32).reshape(4, 1)
    y = np.array(yv, dtype=np.float32)
    table = [0.2, 0.1, 0.05]                            # shorter than the 4 updates of the run
    th = 0.0
    u = 0
    for b in (0, 1):
        pm = P.perm_scalar(0, b, 1, 4)
        for m in range(2):
            i, j = pm[2 * m], pm[2 * m + 1]
            g = ((x[i] * th - yv[i]) * x[i] + (x[j] * th - yv[j]) * x[j]) / 2
            th -= table[min(u, 2)] * g
            u += 1
    st = bmgd.BMGD(LIN, 1, 2, 123.0, 1)                 # the constant rate must not be used once a table is set
    st.set_lr_schedule(table)
    st.run_buffer(X, y)
    st.run_buffer(X, y)
    assert abs(st.theta[0] - th) < 1e-15

    Xd, yd, _ = _data(600, 5, seed=3)
    a = bmgd.BMGD(LIN, 5, 100, 0.03, 2)
    b_ = bmgd.BMGD(LIN, 5, 100, 0.5, 2)
    b_.set_lr_schedule([0.03] * 7)
    assert np.array_equal(a.run_buffer(Xd, yd), b_.run_buffer(Xd, yd))
    b_.set_lr_schedule(None)                            # cleared: back to the constant rate
    assert b_.step_size() == 0.5

    # orthogonal columns with squared norms N * lam_j... use one column: a full-batch update with alpha = 1 / Sxx
    # solves the one-dimensional least squares problem exactly
    xc, yc = Xd[:, :1].astype(np.float64), yd.astype(np.float64)
    sxx = float((xc[:, 0] ** 2).mean())
    c = bmgd.BMGD(LIN, 1, 600, 1.0, 1)
    c.set_lr_schedule([1.0 / sxx])
    got = c.run_buffer(Xd[:, :1], yd)
    assert abs(got[0] - float((xc[:, 0] * yc).mean()) / sxx) < 1e-12
