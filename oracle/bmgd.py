"""CPU oracle for buffered mini-batch gradient descent (TEST INFRASTRUCTURE).

A plain, slow, fp64 implementation of the computation step of the paper's
Algorithm 1 with the update rule of eq. (2.1): for every buffer, T passes;
at the start of each pass a fresh partition into mini-batches; for each
mini-batch, in order,

    theta <- theta - alpha * (1/n_b) * sum_{i in mini-batch} grad l(X_i, Y_i; theta)

and the estimate at the end of a buffer is the start of the next (Section 2.2).
Per-sample gradients:

  * least squares (Section 3.1, eq. (3.1)):   (x'theta - y) x
    -- eq. (3.1) writes the step as (I - alpha Sxx) theta + alpha Sxy, i.e. the
       gradient of one half of the squared residual; that factor is kept here.
  * generalised linear model (Section 3.2.3): (b'(x'theta) - y) x, the displayed
    derivative; logistic regression has b' = sigmoid (Section 4.1).
  * softmax regression: the C-class member of the same family, parameter W of
    shape p x C, all classes parameterised:  x (softmax(x'W) - onehot(y))'.

When a buffer's row count is not a multiple of n the last mini-batch is short
and its gradient is averaged over its own size (the gradient is a mean over the
mini-batch's index set).

This file exists to check the GPU library.  It shares no code with it, is not
imported by it, and only tests, the smoke check and the benchmark's CPU
baseline call it.  The partition comes from ``oracle.perm``.
"""
from __future__ import annotations

import numpy as np

from . import perm as _perm

LINEAR, LOGISTIC, SOFTMAX = 0, 1, 2
PER_PASS, FIXED = 0, 1
SGD, MOMENTUM, NAG, ADAM = 0, 1, 2, 3


def sigmoid(u: np.ndarray) -> np.ndarray:
    """1/(1+exp(-u)) evaluated without overflow on either side."""
    e = np.exp(-np.abs(u))
    return np.where(u >= 0, 1.0 / (1.0 + e), e / (1.0 + e))


def softmax_rows(U: np.ndarray) -> np.ndarray:
    Z = U - U.max(axis=1, keepdims=True)
    E = np.exp(Z)
    return E / E.sum(axis=1, keepdims=True)


def residual(model: int, U: np.ndarray, y: np.ndarray) -> np.ndarray:
    """b'(u) - y for each row of the mini-batch (a matrix P - onehot(y) for softmax)."""
    if model == LINEAR:
        return U - y
    if model == LOGISTIC:
        return sigmoid(U) - y
    if model == SOFTMAX:
        Rm = softmax_rows(U)
        Rm[np.arange(len(y)), y] -= 1.0
        return Rm
    raise ValueError(model)


def minibatch_gradient(model: int, Xb: np.ndarray, yb: np.ndarray, theta: np.ndarray) -> np.ndarray:
    """Mean per-sample gradient over the rows of one mini-batch."""
    U = Xb @ theta
    return Xb.T @ residual(model, U, yb) / Xb.shape[0]


def loss(model: int, X: np.ndarray, y: np.ndarray, theta: np.ndarray) -> float:
    """Mean per-sample loss whose gradient ``minibatch_gradient`` returns."""
    U = X @ theta
    if model == LINEAR:
        return float(0.5 * np.mean((U - y) ** 2))
    if model == LOGISTIC:
        # -(y u - log(1 + e^u)), with log(1+e^u) = max(u,0) + log1p(e^-|u|)
        return float(np.mean(np.maximum(U, 0.0) + np.log1p(np.exp(-np.abs(U))) - y * U))
    if model == SOFTMAX:
        Z = U - U.max(axis=1, keepdims=True)
        lse = np.log(np.exp(Z).sum(axis=1))
        return float(np.mean(lse - Z[np.arange(len(y)), y]))
    raise ValueError(model)


def to_f64(X: np.ndarray) -> np.ndarray:
    """Widen stored predictors (fp32, or bfloat16 bit patterns in uint16) to fp64 exactly."""
    if X.dtype == np.uint16:
        return (X.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return X.astype(np.float64)


class BMGD:
    """State carried across buffers: theta and the count b of buffers processed."""

    def __init__(self, model: int, p: int, n: int, alpha: float, T: int, C: int = 1,
                 seed: int = 0, reshuffle: int = PER_PASS, K_fixed: int = 0,
                 theta0: np.ndarray | None = None):
        self.model, self.p, self.n, self.alpha, self.T = model, p, n, float(alpha), T
        self.C, self.seed, self.reshuffle, self.K_fixed = C, seed, reshuffle, K_fixed
        shape = (p, C) if model == SOFTMAX else (p,)
        self.theta = np.zeros(shape) if theta0 is None else np.array(theta0, dtype=np.float64).reshape(shape)
        self.b = 0
        self.steps = 0
        # Optional learning rate per mini-batch update (Theorem 4 lets alpha change over the run; Section 4.4 uses
        # a cosine schedule): update number u, counted from the moment the schedule is set, uses
        # lr_schedule[min(u, len - 1)]; None = the constant self.alpha.
        self.lr_schedule = None
        self.lr_pos = 0

    def set_lr_schedule(self, alphas) -> None:
        self.lr_schedule = None if alphas is None or len(alphas) == 0 else np.asarray(alphas, dtype=np.float64)
        self.lr_pos = 0

    def set_optimizer(self, kind: int, momentum: float = 0.9, beta1: float = 0.9, beta2: float = 0.999,
                      eps: float = 1e-8) -> None:
        """Buffered variants of other gradient methods (Section 4.3: the buffering idea combined with NAG and Adam):
        the mini-batch gradient g of eq. (2.1) is fed to the chosen update rule instead of theta <- theta - alpha g.
          MOMENTUM  v <- mu v - alpha g;  theta <- theta + v                       (heavy ball)
          NAG       v <- mu v - alpha g;  theta <- theta + mu v - alpha g          (Nesterov, in the form that keeps
                                                                                    the gradient at the stored iterate)
          ADAM      m <- b1 m + (1 - b1) g;  s <- b2 s + (1 - b2) g^2;  k <- k + 1
                    theta <- theta - alpha (m / (1 - b1^k)) / (sqrt(s / (1 - b2^k)) + eps)   (Kingma and Ba, Algorithm 1)
        State starts at zero and is carried across buffers like theta."""
        self.opt, self.mu, self.b1, self.b2, self.eps = kind, float(momentum), float(beta1), float(beta2), float(eps)
        self.m = np.zeros_like(self.theta)
        self.s = np.zeros_like(self.theta)
        self.k = 0

    def apply(self, g: np.ndarray) -> None:
        """One update of theta from the mini-batch gradient g."""
        a = self.step_size()
        opt = getattr(self, "opt", SGD)
        if opt == SGD:
            self.theta = self.theta - a * g
        elif opt == MOMENTUM:
            self.m = self.mu * self.m - a * g
            self.theta = self.theta + self.m
        elif opt == NAG:
            self.m = self.mu * self.m - a * g
            self.theta = self.theta + self.mu * self.m - a * g
        elif opt == ADAM:
            self.k += 1
            self.m = self.b1 * self.m + (1.0 - self.b1) * g
            self.s = self.b2 * self.s + (1.0 - self.b2) * g * g
            mhat = self.m / (1.0 - self.b1 ** self.k)
            shat = self.s / (1.0 - self.b2 ** self.k)
            self.theta = self.theta - a * mhat / (np.sqrt(shat) + self.eps)
        else:
            raise ValueError("unknown optimizer")

    def swa_update(self) -> None:
        """Fold the current estimate into the running average of estimates (Section 4.4, weight averaging every so
        many buffer epochs): after k calls self.swa is the plain mean of the k estimates."""
        self.swa_count = getattr(self, "swa_count", 0) + 1
        if self.swa_count == 1:
            self.swa = self.theta.copy()
        else:
            self.swa = self.swa + (self.theta - self.swa) / self.swa_count

    def step_size(self) -> float:
        """Learning rate of the update about to be made."""
        if self.lr_schedule is None:
            return self.alpha
        return float(self.lr_schedule[min(self.lr_pos, len(self.lr_schedule) - 1)])

    def partition(self, N0: int, t: int) -> np.ndarray:
        """Index permutation used for pass t (1-based) of the buffer about to be processed."""
        if self.reshuffle == FIXED:
            k = self.b % self.K_fixed if self.K_fixed > 0 else self.b
            return _perm.perm(self.seed, k, 0, N0)
        return _perm.perm(self.seed, self.b, t, N0)

    def run_buffer(self, X: np.ndarray, y: np.ndarray, on_step=None) -> np.ndarray:
        """T passes of sequential mini-batch updates over one buffer (stored dtype in, fp64 inside)."""
        N0 = X.shape[0]
        small = X.size <= (1 << 24)
        Xd = to_f64(X) if small else None
        yd = y if self.model == SOFTMAX else y.astype(np.float64)
        for t in range(1, self.T + 1):
            pm = self.partition(N0, t)
            for start in range(0, N0, self.n):
                idx = pm[start:min(start + self.n, N0)]
                Xb = Xd[idx] if small else to_f64(X[idx])
                g = minibatch_gradient(self.model, Xb, yd[idx], self.theta)
                self.apply(g)
                self.steps += 1
                self.lr_pos += 1
                if on_step is not None:
                    on_step(self)
        self.b += 1
        return self.theta


def run(model: int, X: np.ndarray, y: np.ndarray, N0: int, n: int, alpha: float, T: int, R: int,
        C: int = 1, seed: int = 0, reshuffle: int = PER_PASS, theta0=None, on_buffer=None) -> np.ndarray:
    """Whole run: R iterations over K = ceil(N/N0) contiguous buffers of X."""
    N, p = X.shape
    K = -(-N // N0)
    st = BMGD(model, p, n, alpha, T, C=C, seed=seed, reshuffle=reshuffle, K_fixed=K, theta0=theta0)
    for r in range(R):
        for k in range(K):
            lo, hi = k * N0, min((k + 1) * N0, N)
            st.run_buffer(X[lo:hi], y[lo:hi])
            if on_buffer is not None:
                on_buffer(r, k, st)
    return st.theta
