"""bmgd_reader: buffers read from files by a host thread into a pinned ring (the storage -> host transfer of
Section 2.1) must reach the device unchanged and in order: training through the reader equals, bit for bit, training
through bmgd_load_buffer_async on the same data held in memory, and matches the oracle."""
import numpy as np
import pytest

import workloads as wl
from gpu_util import gpu_run, oracle_run, rel_l2

pytestmark = pytest.mark.gpu


def _files(tmp_path, X, y):
    fx, fy = tmp_path / "x.bin", tmp_path / "y.bin"
    X.tofile(fx)
    y.tofile(fy)
    return str(fx), str(fy)


@pytest.mark.parametrize("ring", [2, 3, 5])
def test_training_through_the_reader(tmp_path, ring):
    import torch
    import paper_2312_08728_amd as B
    w = wl.CONFIGS["cfg3"].scaled(name="case", N=45_000, p=64, N0=10_000, n=500, T=2, R=2, alpha=0.2)
    X, y = wl.dataset(w)
    fx, fy = _files(tmp_path, X, y)
    want, _ = gpu_run(w, X, y)                         # same data from memory through the same two slots
    cs, ks = torch.cuda.Stream(), torch.cuda.Stream()
    ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T, model=w.model, n_buffers=5)
    rd = B.Reader(fx, fy, w.p, w.N, w.N0, ring_slots=ring, loop=True)
    rows = []
    for _ in range(10):                                 # two iterations over the five buffers
        rows.append(rd.load_into(ctx, cs))
        ctx.run_buffer(ks)
    got = ctx.get_theta()
    nbytes, secs = rd.stats()
    rd.close()
    ctx.close()
    assert rows == [10_000, 10_000, 10_000, 10_000, 5_000] * 2
    assert nbytes >= 2 * (X.nbytes + y.nbytes) and secs > 0       # it may have read ahead
    assert np.array_equal(got, want)
    assert rel_l2(got, oracle_run(w, X, y)) <= 1e-4


def test_end_of_data_and_manual_acquire(tmp_path):
    import ctypes
    import paper_2312_08728_amd as B
    rng = np.random.default_rng(0)
    X = rng.standard_normal((2500, 7)).astype(np.float32)
    y = rng.standard_normal(2500).astype(np.float32)
    fx, fy = _files(tmp_path, X, y)
    rd = B.Reader(fx, fy, 7, 2500, 1000, ring_slots=2, loop=False)
    seen = []
    for _ in range(3):
        ax, ay, rows = rd.acquire()
        xs = np.ctypeslib.as_array(ctypes.cast(ax, ctypes.POINTER(ctypes.c_float)), shape=(rows, 7)).copy()
        ys = np.ctypeslib.as_array(ctypes.cast(ay, ctypes.POINTER(ctypes.c_float)), shape=(rows,)).copy()
        seen.append((xs, ys))
        rd.release(after_stream=False)
    assert [s[0].shape[0] for s in seen] == [1000, 1000, 500]
    assert np.array_equal(np.concatenate([s[0] for s in seen]), X)
    assert np.array_equal(np.concatenate([s[1] for s in seen]), y)
    assert rd.acquire()[2] == 0 and rd.acquire()[2] == 0          # end of the data, repeatedly
    with pytest.raises(B.BmgdError):
        rd.release()                                              # nothing is handed out
    rd.close()


def test_ring_exhaustion_and_errors(tmp_path):
    import paper_2312_08728_amd as B
    X = np.zeros((400, 4), dtype=np.float32)
    y = np.zeros(400, dtype=np.float32)
    fx, fy = _files(tmp_path, X, y)
    rd = B.Reader(fx, fy, 4, 400, 100, ring_slots=2, loop=True)
    rd.acquire(); rd.acquire()
    with pytest.raises(B.BmgdError) as e:
        rd.acquire()                                              # both slots are handed out
    assert e.value.code == B.BMGD_ESTATE
    rd.release(after_stream=False)
    assert rd.acquire()[2] == 100
    rd.close()                                                    # with slots still handed out
    for kw in (dict(n_rows=401), dict(ring_slots=1), dict(p=0)):
        args = dict(p=4, n_rows=400, buffer_n=100, ring_slots=2)
        args.update(kw)
        with pytest.raises(B.BmgdError) as e:
            B.Reader(fx, fy, args["p"], args["n_rows"], args["buffer_n"], ring_slots=args["ring_slots"])
        assert e.value.code == B.BMGD_EINVAL
    with pytest.raises(B.BmgdError):
        B.Reader(str(tmp_path / "missing.bin"), fy, 4, 400, 100)


@pytest.mark.parametrize("chain,max_passes", [(3, 6), (1, 6), (3, 1)])
def test_adaptive_passes_fed_by_the_reader(tmp_path, chain, max_passes):
    """Reader -> loader -> passes until the next buffer is on the device: the counts the library reports, replayed in
    the oracle, give the same estimate; the data set ends after its five buffers."""
    import torch
    import paper_2312_08728_amd as B
    from oracle import bmgd as O
    w = wl.CONFIGS["cfg2"].scaled(name="case", N=45_000, p=40, N0=10_000, n=500, T=1, R=1, alpha=0.02)
    X, y = wl.dataset(w)
    fx, fy = _files(tmp_path, X, y)
    cs, ks = torch.cuda.Stream(), torch.cuda.Stream()
    ctx = B.Context(w.p, w.N0, w.n, w.alpha, 1, chain=chain, n_buffers=5)
    rd = B.Reader(fx, fy, w.p, w.N, w.N0, ring_slots=2, loop=False)
    assert rd.load_into(ctx, cs) == 10_000
    used, sizes = [], [10_000]
    while True:
        done, nxt = ctx.run_buffer_adaptive_reader(ks, rd, cs, 1, max_passes)
        used.append(done)
        if nxt == 0:
            break
        sizes.append(nxt)
    got = ctx.get_theta()
    st = ctx.stats()
    with pytest.raises(B.BmgdError) as e:
        ctx.run_buffer_adaptive_reader(ks, rd, cs, 1, 2)          # nothing is loaded any more
    assert e.value.code == B.BMGD_ESTATE
    rd.close()
    ctx.close()
    assert sizes == [10_000, 10_000, 10_000, 10_000, 5_000] and len(used) == 5
    assert all(1 <= u <= max_passes for u in used) and st.buffers_run == 5
    assert st.h2d_bytes == X.nbytes + y.nbytes
    ref = O.BMGD(w.model, w.p, w.n, w.alpha, 1)
    for k, T in enumerate(used):
        ref.T = T
        ref.run_buffer(X[k * 10_000:(k + 1) * 10_000], y[k * 10_000:(k + 1) * 10_000])
    assert rel_l2(got, ref.theta) <= 1e-4, used


def test_softmax_buffers_from_bf16_files(tmp_path):
    """bf16 predictors and int32 class ids through the reader: same estimate, bit for bit, as from pinned memory."""
    import torch
    import paper_2312_08728_amd as B
    w = wl.CONFIGS["cfg5"].scaled(name="case", N=2500, p=96, C=12, N0=1000, n=256, T=1, R=1)
    X, y = wl.dataset(w)                                       # uint16 bit patterns of bf16, int32 labels
    fx, fy = _files(tmp_path, X, y)
    want, _ = gpu_run(w, X, y)
    cs, ks = torch.cuda.Stream(), torch.cuda.Stream()
    ctx = B.Context(w.p, w.N0, w.n, w.alpha, w.T, model=w.model, n_classes=w.C, n_buffers=3)
    rd = B.Reader(fx, fy, w.p, w.N, w.N0, x_dtype=B.BMGD_BF16, ring_slots=2)
    rows = []
    while True:
        r = rd.load_into(ctx, cs)
        if r == 0:
            break
        rows.append(r)
        ctx.run_buffer(ks)
    got = ctx.get_theta()
    rd.close()
    ctx.close()
    assert rows == [1000, 1000, 500]
    assert np.array_equal(got, want)
    assert rel_l2(got, oracle_run(w, X, y)) <= 2e-3
