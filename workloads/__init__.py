"""Seeded synthetic inputs for buffered mini-batch gradient descent runs.

This module only *draws data*: design matrices, true coefficients, responses
and labels with the shapes and value distributions of the paper's simulation
design (Section 4.1: Gaussian predictors with a Toeplitz covariance, a
coefficient vector drawn once and then fixed, Gaussian noise for the linear
model and Bernoulli responses for the logistic model).  It holds none of the
method's own arithmetic (no gradient, no update, no mini-batch partition), so
both the CPU oracle's tests and the GPU path's tests may use it to obtain the
same stored bytes.

Every array is generated in fixed-size row chunks, each chunk from its own
counter-based Philox stream keyed by (seed, stream id, chunk index), so any
block of rows can be regenerated on its own and chunks can be filled by
several threads with a result that does not depend on the thread count.
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace

import numpy as np

LINEAR, LOGISTIC, SOFTMAX = 0, 1, 2
MODEL_NAMES = {LINEAR: "linear", LOGISTIC: "logistic", SOFTMAX: "softmax"}

_CHUNK_ROWS = 8192
_STREAM_X, _STREAM_THETA, _STREAM_NOISE, _STREAM_SUPPORT = 1, 2, 3, 4


@dataclass(frozen=True)
class Workload:
    """One run's shape, in the paper's notation (Section 2.2).

    N samples of p features, split into K buffers of N0 rows; each buffer is
    swept T times in mini-batches of n rows with learning rate alpha; the whole
    sample is visited R times.
    """
    name: str
    model: int
    N: int
    p: int
    N0: int
    n: int
    T: int
    R: int
    alpha: float
    C: int = 1                 # classes (softmax only)
    x_dtype: str = "f32"       # "f32" or "bf16" (storage type of X)
    x_cov: str = "identity"    # "identity" or "ar1:<rho>"
    theta_kind: str = "gauss"  # "ones", "gauss", "sparse:<nnz>"
    noise_sigma: float = 1.0
    seed: int = 0

    @property
    def K(self) -> int:
        return -(-self.N // self.N0)

    @property
    def M(self) -> int:
        return -(-self.N0 // self.n)

    @property
    def steps(self) -> int:
        total = 0
        for k in range(self.K):
            rows = min(self.N0, self.N - k * self.N0)
            total += -(-rows // self.n)
        return self.R * self.T * total

    @property
    def sample_gradients(self) -> int:
        return self.R * self.T * self.N

    @property
    def x_itemsize(self) -> int:
        return 2 if self.x_dtype == "bf16" else 4

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five run shapes this repository is measured and checked on.
CONFIGS = {
    "cfg1": Workload("cfg1", LINEAR, N=10_000, p=10, N0=2_000, n=100, T=2, R=10,
                     alpha=0.05, theta_kind="ones", noise_sigma=1.0),
    "cfg2": Workload("cfg2", LINEAR, N=1_000_000, p=100, N0=100_000, n=1_000, T=3, R=5,
                     alpha=0.01, x_cov="ar1:0.5", theta_kind="gauss", noise_sigma=1.0),
    "cfg3": Workload("cfg3", LOGISTIC, N=10_000_000, p=200, N0=1_000_000, n=4_096, T=2, R=3,
                     alpha=0.1, theta_kind="gauss"),
    "cfg4": Workload("cfg4", LINEAR, N=2_000_000, p=4_096, N0=250_000, n=8_192, T=2, R=2,
                     alpha=0.005, theta_kind="sparse:64", noise_sigma=0.5),
    "cfg5": Workload("cfg5", SOFTMAX, N=1_000_000, p=3_072, N0=100_000, n=1_024, T=2, R=2,
                     alpha=0.05, C=1_000, x_dtype="bf16", theta_kind="gauss"),
}


def _rng(seed: int, stream: int, chunk: int) -> np.random.Generator:
    key = np.array([(seed << 8) | stream, chunk], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to bfloat16 (round-to-nearest-even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns (uint16) to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def true_theta(w: Workload) -> np.ndarray:
    """The coefficient vector (or p x C matrix) the responses are drawn around; fp64."""
    p = w.p
    if w.model == SOFTMAX:
        g = _rng(w.seed, _STREAM_THETA, 0)
        return g.standard_normal((p, w.C)) / math.sqrt(p)
    if w.theta_kind == "ones":
        return np.full(p, 1.0 / math.sqrt(p))
    if w.theta_kind == "gauss":
        return _rng(w.seed, _STREAM_THETA, 0).standard_normal(p) / math.sqrt(p)
    if w.theta_kind.startswith("sparse:"):
        nnz = min(int(w.theta_kind.split(":")[1]), p)
        gs = _rng(w.seed, _STREAM_SUPPORT, 0)
        support = gs.choice(p, size=nnz, replace=False)
        th = np.zeros(p)
        th[support] = _rng(w.seed, _STREAM_THETA, 0).uniform(-1.0, 1.0, size=nnz)
        return th
    raise ValueError(w.theta_kind)


def _x_chunk(w: Workload, chunk: int, rows: int) -> np.ndarray:
    """fp32 predictors for one chunk of rows (before any bf16 rounding)."""
    g = _rng(w.seed, _STREAM_X, chunk)
    z = g.standard_normal((rows, w.p), dtype=np.float32)
    if w.x_cov == "identity":
        return z
    if w.x_cov.startswith("ar1:"):
        # Stationary AR(1) across columns gives cov(x_i, x_j) = rho^|i-j| exactly.
        rho = np.float32(float(w.x_cov.split(":")[1]))
        s = np.float32(math.sqrt(1.0 - float(rho) ** 2))
        for j in range(1, w.p):
            z[:, j] = rho * z[:, j - 1] + s * z[:, j]
        return z
    raise ValueError(w.x_cov)


def _fill_chunk(w: Workload, theta: np.ndarray, chunk: int, r0: int, r1: int, X, y) -> None:
    lo, hi = chunk * _CHUNK_ROWS, min((chunk + 1) * _CHUNK_ROWS, w.N)
    x = _x_chunk(w, chunk, hi - lo)
    if w.x_dtype == "bf16":
        xb = f32_to_bf16_bits(x)
        x = bf16_bits_to_f32(xb)          # responses see the stored (rounded) values
    else:
        xb = x
    a, b = max(lo, r0), min(hi, r1)
    sl = slice(a - lo, b - lo)
    X[a - r0:b - r0] = xb[sl]
    g = _rng(w.seed, _STREAM_NOISE, chunk)
    if w.model == LINEAR:
        eps = g.standard_normal(hi - lo) * w.noise_sigma
        y[a - r0:b - r0] = (x.astype(np.float64) @ theta + eps)[sl].astype(np.float32)
    elif w.model == LOGISTIC:
        u = g.random(hi - lo)
        eta = x.astype(np.float64) @ theta
        prob = np.where(eta >= 0, 1.0 / (1.0 + np.exp(-np.abs(eta))),
                        np.exp(-np.abs(eta)) / (1.0 + np.exp(-np.abs(eta))))
        y[a - r0:b - r0] = (u < prob)[sl].astype(np.float32)
    else:
        # label = argmax_c(x'W* + Gumbel(0,1)); fp32 scores are enough to *draw* labels
        scores = x @ theta.astype(np.float32)
        scores += g.gumbel(size=scores.shape).astype(np.float32)
        y[a - r0:b - r0] = np.argmax(scores, axis=1)[sl].astype(np.int32)


def rows(w: Workload, r0: int, r1: int, out_x=None, out_y=None, threads: int | None = None):
    """Rows [r0, r1) of the sample as stored: (X, y).

    X is fp32 [rows, p], or uint16 bfloat16 bit patterns when ``x_dtype`` is
    "bf16"; y is fp32 [rows] (0/1 for the logistic model) or int32 class ids for
    softmax.  ``out_x`` / ``out_y`` may be preallocated (e.g. pinned) arrays.
    """
    if not (0 <= r0 <= r1 <= w.N):
        raise ValueError("row range outside the sample")
    nrow = r1 - r0
    xdt = np.uint16 if w.x_dtype == "bf16" else np.float32
    ydt = np.int32 if w.model == SOFTMAX else np.float32
    X = out_x if out_x is not None else np.empty((nrow, w.p), dtype=xdt)
    y = out_y if out_y is not None else np.empty(nrow, dtype=ydt)
    if X.shape != (nrow, w.p) or X.dtype != xdt or y.shape != (nrow,) or y.dtype != ydt:
        raise ValueError("output arrays have the wrong shape or dtype")
    if nrow == 0:
        return X, y
    theta = true_theta(w)
    chunks = range(r0 // _CHUNK_ROWS, (r1 - 1) // _CHUNK_ROWS + 1)
    nthreads = threads if threads is not None else min(16, os.cpu_count() or 1)
    if nthreads <= 1 or len(chunks) == 1:
        for c in chunks:
            _fill_chunk(w, theta, c, r0, r1, X, y)
    else:
        with ThreadPoolExecutor(nthreads) as pool:
            list(pool.map(lambda c: _fill_chunk(w, theta, c, r0, r1, X, y), chunks))
    return X, y


def buffer_rows(w: Workload, k: int):
    """Row range of buffer k (0-based): buffers are contiguous blocks of N0 rows."""
    return k * w.N0, min((k + 1) * w.N0, w.N)


def dataset(w: Workload, threads: int | None = None):
    """The whole sample (X, y) in host memory."""
    return rows(w, 0, w.N, threads=threads)
