"""Pins for the oracle's buffered NAG / momentum / Adam updates (Section 4.3 combines the buffering idea with these
methods): closed forms on quadratics, limiting cases, invariances, hand-unrolled scalar runs."""
import numpy as np

from oracle import bmgd, perm as P

LIN = bmgd.LINEAR


def _quadratic(N=400, p=4, seed=1):
    g = np.random.default_rng(seed)
    X = g.standard_normal((N, p)).astype(np.float32)
    y = (X @ g.standard_normal(p) + 0.3 * g.standard_normal(N)).astype(np.float32)
    Xd, yd = X.astype(np.float64), y.astype(np.float64)
    return X, y, Xd.T @ Xd / N, Xd.T @ yd / N


def test_momentum_and_nag_follow_the_linear_recurrence_on_a_quadratic():
    """Full batch least squares: g = S theta - b, so (theta, v) evolves by a fixed affine map; compare the oracle
    after k updates with that map applied k times as a dense matrix."""
    X, y, S, b = _quadratic()
    p, alpha, mu, k = 4, 0.05, 0.8, 25
    I = np.eye(p)
    for kind in (bmgd.MOMENTUM, bmgd.NAG):
        # v' = mu v - alpha (S th - b);  th' = th + v' (momentum)  or  th + mu v' - alpha (S th - b) (NAG)
        if kind == bmgd.MOMENTUM:
            A = np.block([[I - alpha * S, mu * I], [-alpha * S, mu * I]])
            c = np.concatenate([alpha * b, alpha * b])
        else:
            A = np.block([[I - (1 + mu) * alpha * S, mu * mu * I], [-alpha * S, mu * I]])
            c = np.concatenate([(1 + mu) * alpha * b, alpha * b])
        z = np.zeros(2 * p)
        for _ in range(k):
            z = A @ z + c
        st = bmgd.BMGD(LIN, p, 400, alpha, k)
        st.set_optimizer(kind, momentum=mu)
        st.run_buffer(X, y)                              # one batch = the whole buffer, k passes
        assert np.allclose(st.theta, z[:p], rtol=0, atol=1e-12)
        assert np.allclose(st.m, z[p:], rtol=0, atol=1e-12)
    # mu = 0 is plain gradient descent for both
    ref = bmgd.BMGD(LIN, p, 100, alpha, 3).run_buffer(X, y)
    for kind in (bmgd.MOMENTUM, bmgd.NAG):
        st = bmgd.BMGD(LIN, p, 100, alpha, 3)
        st.set_optimizer(kind, momentum=0.0)
        assert np.allclose(st.run_buffer(X, y), ref, rtol=0, atol=1e-15)


def test_nag_equals_gradient_at_the_lookahead_point():
    """Nesterov's method in its original form evaluates the gradient at y_k = x_k + mu (x_k - x_{k-1}):
    x_{k+1} = y_k - alpha grad f(y_k).  The stored iterate of the form used here is y_k."""
    X, y, S, b = _quadratic(seed=5)
    p, alpha, mu = 4, 0.04, 0.7
    x_prev = np.zeros(p)
    x = np.zeros(p)
    ys = []
    for _ in range(12):
        yk = x + mu * (x - x_prev)
        ys.append(yk)
        x_prev, x = x, yk - alpha * (S @ yk - b)
    ys.append(x + mu * (x - x_prev))
    st = bmgd.BMGD(LIN, p, 400, alpha, 1)
    st.set_optimizer(bmgd.NAG, momentum=mu)
    for k in range(12):
        assert np.allclose(st.theta, ys[k], rtol=0, atol=1e-12)
        st.run_buffer(X, y)
    assert np.allclose(st.theta, ys[12], rtol=0, atol=1e-12)


def test_adam_hand_unrolled_first_step_and_scale_invariance():
    x = [1.0, -2.0, 0.5, 3.0]
    yv = [0.5, 1.0, -1.0, 2.0]
    X = np.array(x, dtype=np.float32).reshape(4, 1)
    y = np.array(yv, dtype=np.float32)
    alpha, b1, b2, eps = 0.1, 0.9, 0.999, 1e-8
    th = m = s = 0.0
    k = 0
    for t in (1, 2):
        pm = P.perm_scalar(0, 0, t, 4)
        for mb in range(2):
            i, j = pm[2 * mb], pm[2 * mb + 1]
            g = ((x[i] * th - yv[i]) * x[i] + (x[j] * th - yv[j]) * x[j]) / 2
            k += 1
            m = b1 * m + (1 - b1) * g
            s = b2 * s + (1 - b2) * g * g
            th -= alpha * (m / (1 - b1 ** k)) / ((s / (1 - b2 ** k)) ** 0.5 + eps)
    st = bmgd.BMGD(LIN, 1, 2, alpha, 2)
    st.set_optimizer(bmgd.ADAM, beta1=b1, beta2=b2, eps=eps)
    st.run_buffer(X, y)
    assert abs(st.theta[0] - th) < 1e-14 and st.k == 4

    # first update: m_hat = g, s_hat = g^2, so every coordinate moves by alpha * sign(g) (up to eps)
    Xq, yq, S, b = _quadratic()
    st = bmgd.BMGD(LIN, 4, 400, 0.01, 1)
    st.set_optimizer(bmgd.ADAM)
    st.run_buffer(Xq, yq)
    assert np.allclose(st.theta, 0.01 * np.sign(b), rtol=0, atol=1e-8)     # gradient at theta = 0 is -b

    # a batch with every row twice has the same mean gradient: identical paths
    a1 = bmgd.BMGD(LIN, 4, 400, 0.02, 3); a1.set_optimizer(bmgd.ADAM, eps=0.0)
    a2 = bmgd.BMGD(LIN, 4, 800, 0.02, 3); a2.set_optimizer(bmgd.ADAM, eps=0.0)
    a1.run_buffer(Xq, yq)
    a2.run_buffer(np.concatenate([Xq, Xq]), np.concatenate([yq, yq]))
    assert np.allclose(a1.theta, a2.theta, rtol=0, atol=1e-12)
    # with eps = 0 Adam is invariant to a positive rescaling of the loss: gradients c g give the same path
    r = np.random.default_rng(0)
    gs = r.standard_normal((6, 4))
    u = bmgd.BMGD(LIN, 4, 1, 0.03, 1); u.set_optimizer(bmgd.ADAM, eps=0.0)
    v = bmgd.BMGD(LIN, 4, 1, 0.03, 1); v.set_optimizer(bmgd.ADAM, eps=0.0)
    for g in gs:
        u.apply(g)
        v.apply(1000.0 * g)
    assert np.allclose(u.theta, v.theta, rtol=1e-12, atol=0)


def test_state_is_carried_across_buffers_and_passes():
    """Running two buffers through run_buffer equals running their updates one after another by hand with one state."""
    X, y, _, _ = _quadratic(N=300, p=3, seed=2)
    for kind in (bmgd.MOMENTUM, bmgd.NAG, bmgd.ADAM):
        st = bmgd.BMGD(LIN, 3, 50, 0.05, 2)
        st.set_optimizer(kind)
        st.run_buffer(X[:150], y[:150])
        st.run_buffer(X[150:], y[150:])
        ref = bmgd.BMGD(LIN, 3, 50, 0.05, 2)
        ref.set_optimizer(kind)
        for b, (lo, hi) in enumerate(((0, 150), (150, 300))):
            Xb, yb = X[lo:hi].astype(np.float64), y[lo:hi].astype(np.float64)
            for t in (1, 2):
                pm = P.perm(0, b, t, 150)
                for s0 in range(0, 150, 50):
                    idx = pm[s0:s0 + 50]
                    ref.apply(Xb[idx].T @ (Xb[idx] @ ref.theta - yb[idx]) / 50)
        assert np.allclose(st.theta, ref.theta, rtol=0, atol=1e-13)


def test_running_average_of_estimates_is_their_plain_mean():
    """Weight averaging (Section 4.4): after k snapshots the running average equals the arithmetic mean of the k
    estimates, whatever happened between them; a single snapshot is the estimate itself."""
    rng = np.random.default_rng(5)
    X = rng.standard_normal((600, 6))
    y = X @ rng.standard_normal(6) + 0.1 * rng.standard_normal(600)
    st = bmgd.BMGD(bmgd.LINEAR, 6, 50, 0.05, 2)
    snaps = []
    for k in range(6):
        st.run_buffer(X[k * 100:(k + 1) * 100], y[k * 100:(k + 1) * 100])
        if k % 2 == 1:
            st.swa_update()
            snaps.append(st.theta.copy())
            np.testing.assert_allclose(st.swa, np.mean(snaps, axis=0), rtol=0, atol=1e-15)
    assert st.swa_count == 3
    assert np.array_equal(snaps[0], np.mean(snaps[:1], axis=0))
    assert not np.allclose(st.swa, st.theta)
