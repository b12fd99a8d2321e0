"""ctypes binding of libbmgd (see include/bmgd.h).

Argument marshalling only: every step of the computation runs inside the
library's HIP kernels.  The module-level ``bmgd_*`` functions mirror the C
entry points one to one; ``Context`` is a small convenience wrapper around a
``bmgd_ctx*`` that accepts numpy arrays and torch tensors (anything with a data
pointer) and torch streams.  If the shared library has not been built the
import fails loudly -- there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbmgd.so")

BMGD_OK, BMGD_EINVAL, BMGD_ESTATE, BMGD_EHIP, BMGD_ENOMEM = 0, 1, 2, 3, 4
BMGD_LINEAR, BMGD_LOGISTIC, BMGD_SOFTMAX = 0, 1, 2
BMGD_F32, BMGD_BF16 = 0, 1
BMGD_RESHUFFLE_PER_PASS, BMGD_RESHUFFLE_FIXED = 0, 1
BMGD_CHAIN_AUTO, BMGD_CHAIN_PERSISTENT, BMGD_CHAIN_LAUNCH, BMGD_CHAIN_GRAM, BMGD_CHAIN_GRAPH, BMGD_CHAIN_PRODUCT = 0, 1, 2, 3, 4, 5
BMGD_OPT_SGD, BMGD_OPT_MOMENTUM, BMGD_OPT_NAG, BMGD_OPT_ADAM = 0, 1, 2, 3

EXPORTS = [
    "bmgd_default_config", "bmgd_create", "bmgd_create_ex", "bmgd_workspace_bytes",
    "bmgd_run_cached_buffer", "bmgd_clear_moment_cache", "bmgd_set_row_subset", "bmgd_swa_update", "bmgd_get_swa", "bmgd_swa_reset",
    "bmgd_reader_open", "bmgd_reader_acquire", "bmgd_reader_release", "bmgd_load_from_reader", "bmgd_run_buffer_adaptive_reader", "bmgd_reader_stats",
    "bmgd_reader_last_error", "bmgd_reader_close",
    "bmgd_load_buffer_async", "bmgd_run_buffer", "bmgd_run_buffer_adaptive", "bmgd_run_device_buffer", "bmgd_get_theta",
    "bmgd_set_theta", "bmgd_set_lr", "bmgd_set_passes", "bmgd_set_lr_schedule", "bmgd_reset_optimizer", "bmgd_eval_loss", "bmgd_eval_loss_static", "bmgd_set_position", "bmgd_get_perm", "bmgd_sync", "bmgd_get_stats",
    "bmgd_last_error", "bmgd_destroy",
]


class bmgd_config(C.Structure):
    _fields_ = [
        ("p", C.c_int64), ("buffer_n", C.c_int64), ("batch_n", C.c_int64), ("lr", C.c_double),
        ("passes", C.c_int32), ("model", C.c_int32), ("n_classes", C.c_int32), ("x_dtype", C.c_int32),
        ("seed", C.c_uint64), ("reshuffle", C.c_int32), ("n_buffers", C.c_int32), ("chain", C.c_int32),
        ("n_workgroups", C.c_int32), ("barrier_timeout_us", C.c_int64), ("workspace", C.c_void_p),
        ("workspace_bytes", C.c_size_t), ("optimizer", C.c_int32), ("cache_moments", C.c_int32),
        ("momentum", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
    ]


class bmgd_stats(C.Structure):
    _fields_ = [
        ("buffers_run", C.c_int64), ("steps", C.c_int64), ("sample_gradients", C.c_int64),
        ("h2d_bytes", C.c_int64), ("copy_ms", C.c_double), ("compute_ms", C.c_double),
        ("wait_ms", C.c_double), ("n_workgroups", C.c_int32), ("threads_per_group", C.c_int32),
        ("chain", C.c_int32), ("reserved", C.c_int32), ("chain_ms", C.c_double), ("chain_launches", C.c_int64),
        ("prep_ms", C.c_double), ("prep_launches", C.c_int64),
    ]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -m paper_2312_08728_amd.build "
                          f"or __graft_entry__.build()); there is no fallback path")
    # PyTorch bundles its own HIP runtime under the same soname as the system one; a process must use
    # exactly one of them.  Importing torch first makes libbmgd bind to the runtime torch's allocator
    # and streams already use.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i64, i32 = C.c_void_p, C.c_int64, C.c_int
    lib.bmgd_default_config.argtypes, lib.bmgd_default_config.restype = [C.POINTER(bmgd_config)], None
    lib.bmgd_create.argtypes, lib.bmgd_create.restype = [i64, i64, i64, C.c_double, i32], vp
    lib.bmgd_create_ex.argtypes, lib.bmgd_create_ex.restype = [C.POINTER(bmgd_config), C.POINTER(vp)], i32
    lib.bmgd_workspace_bytes.argtypes, lib.bmgd_workspace_bytes.restype = [C.POINTER(bmgd_config)], C.c_size_t
    lib.bmgd_load_buffer_async.argtypes, lib.bmgd_load_buffer_async.restype = [vp, vp, vp, i64, vp], i32
    lib.bmgd_run_buffer.argtypes, lib.bmgd_run_buffer.restype = [vp, vp], i32
    lib.bmgd_run_device_buffer.argtypes, lib.bmgd_run_device_buffer.restype = [vp, vp, vp, i64, vp], i32
    lib.bmgd_run_buffer_adaptive.argtypes = [vp, vp, vp, vp, i64, vp, C.c_int, C.c_int, C.POINTER(C.c_int)]
    lib.bmgd_run_buffer_adaptive.restype = i32
    lib.bmgd_run_cached_buffer.argtypes, lib.bmgd_run_cached_buffer.restype = [vp, vp], i32
    lib.bmgd_clear_moment_cache.argtypes, lib.bmgd_clear_moment_cache.restype = [vp], i32
    lib.bmgd_set_row_subset.argtypes, lib.bmgd_set_row_subset.restype = [vp, vp, i64], i32
    lib.bmgd_swa_update.argtypes, lib.bmgd_swa_update.restype = [vp, vp], i32
    lib.bmgd_get_swa.argtypes, lib.bmgd_get_swa.restype = [vp, vp, i64, C.POINTER(i64)], i32
    lib.bmgd_swa_reset.argtypes, lib.bmgd_swa_reset.restype = [vp], i32
    lib.bmgd_reader_open.argtypes = [C.c_char_p, C.c_char_p, i64, i32, i64, i64, i32, i32, C.POINTER(vp)]
    lib.bmgd_reader_open.restype = i32
    lib.bmgd_reader_acquire.argtypes, lib.bmgd_reader_acquire.restype = [vp, C.POINTER(vp), C.POINTER(vp), C.POINTER(i64)], i32
    lib.bmgd_reader_release.argtypes, lib.bmgd_reader_release.restype = [vp, vp, i32], i32
    lib.bmgd_load_from_reader.argtypes, lib.bmgd_load_from_reader.restype = [vp, vp, vp, C.POINTER(i64)], i32
    lib.bmgd_run_buffer_adaptive_reader.argtypes = [vp, vp, vp, vp, C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(i64)]
    lib.bmgd_run_buffer_adaptive_reader.restype = i32
    lib.bmgd_reader_stats.argtypes, lib.bmgd_reader_stats.restype = [vp, C.POINTER(i64), C.POINTER(C.c_double)], i32
    lib.bmgd_reader_last_error.argtypes, lib.bmgd_reader_last_error.restype = [vp], C.c_char_p
    lib.bmgd_reader_close.argtypes, lib.bmgd_reader_close.restype = [vp], None
    lib.bmgd_get_theta.argtypes, lib.bmgd_get_theta.restype = [vp, vp, i64], i32
    lib.bmgd_set_theta.argtypes, lib.bmgd_set_theta.restype = [vp, vp, i64], i32
    lib.bmgd_set_position.argtypes, lib.bmgd_set_position.restype = [vp, i64], i32
    lib.bmgd_set_lr.argtypes, lib.bmgd_set_lr.restype = [vp, C.c_double], i32
    lib.bmgd_eval_loss.argtypes, lib.bmgd_eval_loss.restype = [vp, vp, vp, C.c_int64, vp, C.POINTER(C.c_double)], i32
    lib.bmgd_eval_loss_static.argtypes = [C.c_int32, vp, vp, vp, C.c_int64, C.c_int64, vp, vp]
    lib.bmgd_eval_loss_static.restype = i32
    lib.bmgd_reset_optimizer.argtypes, lib.bmgd_reset_optimizer.restype = [vp], i32
    lib.bmgd_set_lr_schedule.argtypes, lib.bmgd_set_lr_schedule.restype = [vp, vp, C.c_int64], i32
    lib.bmgd_set_passes.argtypes, lib.bmgd_set_passes.restype = [vp, i32], i32
    lib.bmgd_get_perm.argtypes, lib.bmgd_get_perm.restype = [vp, i64, i32, vp, i64], i32
    lib.bmgd_sync.argtypes, lib.bmgd_sync.restype = [vp], i32
    lib.bmgd_get_stats.argtypes, lib.bmgd_get_stats.restype = [vp, C.POINTER(bmgd_stats)], i32
    lib.bmgd_last_error.argtypes, lib.bmgd_last_error.restype = [vp], C.c_char_p
    lib.bmgd_destroy.argtypes, lib.bmgd_destroy.restype = [vp], None
    return lib


lib = _load()


def _ptr(a) -> int:
    """Address of a numpy array, torch tensor, ctypes buffer or raw int."""
    if a is None:
        return 0
    if isinstance(a, int):
        return a
    if isinstance(a, np.ndarray):
        if not a.flags["C_CONTIGUOUS"]:
            raise ValueError("array must be C-contiguous")
        return a.ctypes.data
    if hasattr(a, "data_ptr"):
        if not a.is_contiguous():
            raise ValueError("tensor must be contiguous")
        return a.data_ptr()
    return C.addressof(a)


def _stream(s) -> int:
    if s is None:
        return 0
    if isinstance(s, int):
        return s
    return int(s.cuda_stream)


# ---- one-to-one mirrors of the C entry points -------------------------------------------------
def bmgd_default_config() -> bmgd_config:
    cfg = bmgd_config()
    lib.bmgd_default_config(C.byref(cfg))
    return cfg


def bmgd_create(p, buffer_n, batch_n, lr, passes):
    return lib.bmgd_create(p, buffer_n, batch_n, lr, passes)


def bmgd_create_ex(cfg: bmgd_config):
    out = C.c_void_p()
    rc = lib.bmgd_create_ex(C.byref(cfg), C.byref(out))
    return rc, out.value


def bmgd_workspace_bytes(cfg: bmgd_config) -> int:
    return lib.bmgd_workspace_bytes(C.byref(cfg))


def bmgd_load_buffer_async(ctx, host_x, host_y, rows, copy_stream=None) -> int:
    return lib.bmgd_load_buffer_async(ctx, _ptr(host_x), _ptr(host_y), rows, _stream(copy_stream))


def bmgd_run_buffer(ctx, compute_stream=None) -> int:
    return lib.bmgd_run_buffer(ctx, _stream(compute_stream))


def bmgd_run_buffer_adaptive(ctx, compute_stream, next_host_x, next_host_y, next_rows, copy_stream, min_passes, max_passes):
    done = C.c_int(0)
    nx = _ptr(next_host_x) if next_host_x is not None else None
    ny = _ptr(next_host_y) if next_host_y is not None else None
    rc = lib.bmgd_run_buffer_adaptive(ctx, _stream(compute_stream), nx, ny, next_rows, _stream(copy_stream), min_passes,
                                      max_passes, C.byref(done))
    return rc, done.value


def bmgd_run_device_buffer(ctx, dev_x, dev_y, rows, compute_stream=None) -> int:
    return lib.bmgd_run_device_buffer(ctx, _ptr(dev_x), _ptr(dev_y), rows, _stream(compute_stream))


def bmgd_get_theta(ctx, host_out, length) -> int:
    return lib.bmgd_get_theta(ctx, _ptr(host_out), length)


def bmgd_set_theta(ctx, host_in, length) -> int:
    return lib.bmgd_set_theta(ctx, _ptr(host_in), length)


def bmgd_set_lr(ctx, lr) -> int:
    return lib.bmgd_set_lr(ctx, lr)


def bmgd_eval_loss(ctx, dev_x, dev_y, rows, stream=None):
    out = C.c_double(0.0)
    rc = lib.bmgd_eval_loss(ctx, _ptr(dev_x), _ptr(dev_y), rows, _stream(stream), C.byref(out))
    return rc, out.value


def bmgd_eval_loss_static(model, dev_x, dev_y, dev_theta, rows, p, stream, dev_out) -> int:
    return lib.bmgd_eval_loss_static(model, _ptr(dev_x), _ptr(dev_y), _ptr(dev_theta), rows, p, _stream(stream), _ptr(dev_out))


def bmgd_reset_optimizer(ctx) -> int:
    return lib.bmgd_reset_optimizer(ctx)


def bmgd_set_lr_schedule(ctx, host_alphas, length) -> int:
    return lib.bmgd_set_lr_schedule(ctx, _ptr(host_alphas), length)


def bmgd_set_passes(ctx, passes) -> int:
    return lib.bmgd_set_passes(ctx, passes)


def bmgd_set_position(ctx, buffer_counter) -> int:
    return lib.bmgd_set_position(ctx, buffer_counter)


def bmgd_get_perm(ctx, buffer_counter, pass_, host_out, length) -> int:
    return lib.bmgd_get_perm(ctx, buffer_counter, pass_, _ptr(host_out), length)


def bmgd_sync(ctx) -> int:
    return lib.bmgd_sync(ctx)


def bmgd_get_stats(ctx):
    st = bmgd_stats()
    rc = lib.bmgd_get_stats(ctx, C.byref(st))
    return rc, st


def bmgd_last_error(ctx=None) -> str:
    msg = lib.bmgd_last_error(ctx)
    return msg.decode() if msg else ""


def bmgd_destroy(ctx) -> None:
    lib.bmgd_destroy(ctx)


# ---- convenience wrapper ------------------------------------------------------------------------
class BmgdError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"bmgd status {code}: {msg}")
        self.code = code


def bmgd_run_cached_buffer(ctx, compute_stream=None) -> int:
    return lib.bmgd_run_cached_buffer(ctx, _stream(compute_stream))


def bmgd_clear_moment_cache(ctx) -> int:
    return lib.bmgd_clear_moment_cache(ctx)


def bmgd_set_row_subset(ctx, dev_idx, count) -> int:
    return lib.bmgd_set_row_subset(ctx, _ptr(dev_idx), count)


def bmgd_swa_update(ctx, compute_stream=None) -> int:
    return lib.bmgd_swa_update(ctx, _stream(compute_stream))


def bmgd_get_swa(ctx, host_out, length):
    count = C.c_int64(0)
    rc = lib.bmgd_get_swa(ctx, _ptr(host_out), length, C.byref(count))
    return rc, count.value


def bmgd_swa_reset(ctx) -> int:
    return lib.bmgd_swa_reset(ctx)


def bmgd_reader_open(x_path, y_path, p, x_dtype, n_rows, buffer_n, ring_slots, loop):
    h = C.c_void_p()
    rc = lib.bmgd_reader_open(os.fsencode(x_path), os.fsencode(y_path), p, x_dtype, n_rows, buffer_n, ring_slots,
                              1 if loop else 0, C.byref(h))
    return rc, (h if rc == BMGD_OK else None)


def bmgd_reader_acquire(reader):
    x, y, rows = C.c_void_p(), C.c_void_p(), C.c_int64()
    rc = lib.bmgd_reader_acquire(reader, C.byref(x), C.byref(y), C.byref(rows))
    return rc, x.value, y.value, rows.value


def bmgd_reader_release(reader, copy_stream=None, after_stream=True) -> int:
    return lib.bmgd_reader_release(reader, _stream(copy_stream), 1 if after_stream else 0)


def bmgd_load_from_reader(ctx, reader, copy_stream=None):
    rows = C.c_int64()
    rc = lib.bmgd_load_from_reader(ctx, reader, _stream(copy_stream), C.byref(rows))
    return rc, rows.value


def bmgd_run_buffer_adaptive_reader(ctx, compute_stream, reader, copy_stream, min_passes, max_passes):
    done, rows = C.c_int(0), C.c_int64(0)
    rc = lib.bmgd_run_buffer_adaptive_reader(ctx, _stream(compute_stream), reader, _stream(copy_stream), min_passes,
                                             max_passes, C.byref(done), C.byref(rows))
    return rc, done.value, rows.value


def bmgd_reader_stats(reader):
    b, t = C.c_int64(), C.c_double()
    rc = lib.bmgd_reader_stats(reader, C.byref(b), C.byref(t))
    return rc, b.value, t.value


def bmgd_reader_last_error(reader=None) -> str:
    msg = lib.bmgd_reader_last_error(reader)
    return msg.decode() if msg else ""


def bmgd_reader_close(reader) -> None:
    lib.bmgd_reader_close(reader)


class Reader:
    """Host thread that reads buffers of a data set from two flat files into a ring of pinned buffers (bmgd_reader_*)."""

    def __init__(self, x_path, y_path, p, n_rows, buffer_n, x_dtype=BMGD_F32, ring_slots=3, loop=False):
        rc, h = bmgd_reader_open(x_path, y_path, p, x_dtype, n_rows, buffer_n, ring_slots, loop)
        if rc != BMGD_OK:
            raise BmgdError(rc, bmgd_reader_last_error(None))
        self.h = h

    def _check(self, rc):
        if rc != BMGD_OK:
            raise BmgdError(rc, bmgd_reader_last_error(self.h))

    def acquire(self):
        """(address of x, address of y, rows) of the next buffer; rows = 0 at the end of the data."""
        rc, x, y, rows = bmgd_reader_acquire(self.h)
        self._check(rc)
        return x, y, rows

    def release(self, copy_stream=None, after_stream=True):
        self._check(bmgd_reader_release(self.h, copy_stream, after_stream))

    def load_into(self, ctx: "Context", copy_stream=None) -> int:
        """Next buffer into ctx's idle slot (bmgd_load_from_reader); returns its rows, 0 at the end of the data."""
        rc, rows = bmgd_load_from_reader(ctx.h, self.h, copy_stream)
        if rc != BMGD_OK:
            raise BmgdError(rc, bmgd_last_error(ctx.h) or bmgd_reader_last_error(self.h))
        return rows

    def stats(self):
        rc, b, t = bmgd_reader_stats(self.h)
        self._check(rc)
        return b, t

    def close(self):
        if getattr(self, "h", None):
            bmgd_reader_close(self.h)
            self.h = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Context:
    """Owns one bmgd_ctx*; raises BmgdError on any non-OK status."""

    def __init__(self, p, buffer_n, batch_n, lr, passes, model=BMGD_LINEAR, n_classes=1, x_dtype=None,
                 seed=0, reshuffle=BMGD_RESHUFFLE_PER_PASS, n_buffers=0, chain=BMGD_CHAIN_AUTO,
                 n_workgroups=0, barrier_timeout_us=0, workspace=None, workspace_bytes=0, optimizer=BMGD_OPT_SGD,
                 momentum=0.9, beta1=0.9, beta2=0.999, eps=1e-8, cache_moments=False):
        cfg = bmgd_default_config()
        cfg.p, cfg.buffer_n, cfg.batch_n, cfg.lr, cfg.passes = p, buffer_n, batch_n, lr, passes
        cfg.model, cfg.n_classes = model, n_classes
        cfg.x_dtype = (BMGD_BF16 if model == BMGD_SOFTMAX else BMGD_F32) if x_dtype is None else x_dtype
        cfg.seed, cfg.reshuffle, cfg.n_buffers = seed, reshuffle, n_buffers
        cfg.chain, cfg.n_workgroups, cfg.barrier_timeout_us = chain, n_workgroups, barrier_timeout_us
        cfg.optimizer, cfg.momentum, cfg.beta1, cfg.beta2, cfg.eps = optimizer, momentum, beta1, beta2, eps
        cfg.cache_moments = 1 if cache_moments else 0
        if workspace is not None:
            cfg.workspace, cfg.workspace_bytes = _ptr(workspace), workspace_bytes
        self.cfg = cfg
        self.theta_len = p * (n_classes if model == BMGD_SOFTMAX else 1)
        self._keep = workspace
        rc, h = bmgd_create_ex(cfg)
        if rc != BMGD_OK:
            raise BmgdError(rc, bmgd_last_error(None))
        self.h = h

    def _check(self, rc):
        if rc != BMGD_OK:
            raise BmgdError(rc, bmgd_last_error(self.h))

    def load_buffer_async(self, host_x, host_y, rows, copy_stream=None):
        self._check(bmgd_load_buffer_async(self.h, host_x, host_y, rows, copy_stream))

    def run_buffer(self, compute_stream=None):
        self._check(bmgd_run_buffer(self.h, compute_stream))

    def run_buffer_adaptive(self, compute_stream, next_host_x, next_host_y, next_rows, copy_stream, min_passes, max_passes) -> int:
        """Passes over the loaded buffer until the next one has arrived; returns the number of passes made."""
        rc, done = bmgd_run_buffer_adaptive(self.h, compute_stream, next_host_x, next_host_y, next_rows, copy_stream,
                                            min_passes, max_passes)
        self._check(rc)
        return done

    def run_cached_buffer(self, compute_stream=None):
        self._check(bmgd_run_cached_buffer(self.h, compute_stream))

    def clear_moment_cache(self):
        self._check(bmgd_clear_moment_cache(self.h))

    def set_row_subset(self, dev_idx, count):
        """Restrict the next run to rows dev_idx[:count] (an int32 device tensor) of its buffer."""
        self._check(bmgd_set_row_subset(self.h, dev_idx, count))

    def swa_update(self, compute_stream=None):
        self._check(bmgd_swa_update(self.h, compute_stream))

    def get_swa(self):
        """(running average of the estimates folded in by swa_update, number of them)."""
        out = np.empty(self.theta_len, dtype=np.float32)
        rc, count = bmgd_get_swa(self.h, out, self.theta_len)
        self._check(rc)
        if self.cfg.model == BMGD_SOFTMAX:
            out = out.reshape(self.cfg.p, self.cfg.n_classes)
        return out, count

    def swa_reset(self):
        self._check(bmgd_swa_reset(self.h))

    def run_buffer_adaptive_reader(self, compute_stream, reader, copy_stream, min_passes, max_passes):
        """Like run_buffer_adaptive with the next buffer taken from `reader`; returns (passes made, rows of the buffer now
        loaded or 0 at the end of the data)."""
        rc, done, rows = bmgd_run_buffer_adaptive_reader(self.h, compute_stream, reader.h, copy_stream, min_passes, max_passes)
        if rc != BMGD_OK:
            raise BmgdError(rc, bmgd_last_error(self.h))
        return done, rows

    def run_device_buffer(self, dev_x, dev_y, rows, compute_stream=None):
        self._check(bmgd_run_device_buffer(self.h, dev_x, dev_y, rows, compute_stream))

    def get_theta(self) -> np.ndarray:
        out = np.empty(self.theta_len, dtype=np.float32)
        self._check(bmgd_get_theta(self.h, out, out.size))
        if self.cfg.model == BMGD_SOFTMAX:
            return out.reshape(self.cfg.p, self.cfg.n_classes)
        return out

    def set_theta(self, theta):
        a = np.ascontiguousarray(theta, dtype=np.float32).reshape(-1)
        self._check(bmgd_set_theta(self.h, a, a.size))

    def set_lr(self, lr):
        self._check(bmgd_set_lr(self.h, lr))

    def eval_loss(self, dev_x, dev_y, rows, stream=None) -> float:
        rc, v = bmgd_eval_loss(self.h, dev_x, dev_y, rows, stream)
        self._check(rc)
        return v

    def reset_optimizer(self):
        self._check(bmgd_reset_optimizer(self.h))

    def set_lr_schedule(self, alphas):
        a = np.ascontiguousarray([] if alphas is None else alphas, dtype=np.float32).reshape(-1)
        self._check(bmgd_set_lr_schedule(self.h, a if a.size else None, a.size))

    def set_passes(self, passes):
        self._check(bmgd_set_passes(self.h, passes))

    def set_position(self, buffer_counter):
        self._check(bmgd_set_position(self.h, buffer_counter))

    def get_perm(self, buffer_counter, pass_, length) -> np.ndarray:
        out = np.empty(length, dtype=np.int32)
        self._check(bmgd_get_perm(self.h, buffer_counter, pass_, out, length))
        return out

    def sync(self):
        self._check(bmgd_sync(self.h))

    def stats(self) -> bmgd_stats:
        rc, st = bmgd_get_stats(self.h)
        self._check(rc)
        return st

    def close(self):
        if getattr(self, "h", None):
            bmgd_destroy(self.h)
            self.h = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
