"""The C-ABI library loads, exports every function include/bmgd.h declares, and rejects bad arguments
before touching a GPU.  No compute is attempted here."""
import ctypes
import os
import re

import pytest

import paper_2312_08728_amd as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "bmgd.h")


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bmgd_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = _declared()
    assert len(names) >= 15
    raw = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), n
        assert n in B.EXPORTS and callable(getattr(B, n)), n
    assert sorted(B.EXPORTS) == names


def test_struct_layouts_match_header_order():
    text = open(HEADER).read()
    body = re.search(r"typedef struct bmgd_config \{(.*?)\} bmgd_config;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"\b(\w+);", body)
    assert fields == [f[0] for f in B.bmgd_config._fields_]
    body = re.search(r"typedef struct bmgd_stats \{(.*?)\} bmgd_stats;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    assert re.findall(r"\b(\w+);", body) == [f[0] for f in B.bmgd_stats._fields_]


def _cfg(**kw):
    c = B.bmgd_default_config()
    c.p, c.buffer_n, c.batch_n, c.lr, c.passes = 100, 1000, 100, 0.1, 2
    for k, v in kw.items():
        setattr(c, k, v)
    return c


def test_defaults():
    c = B.bmgd_default_config()
    assert (c.model, c.n_classes, c.x_dtype, c.seed, c.reshuffle, c.chain, c.n_workgroups) == (0, 1, 0, 0, 0, 0, 0)
    assert c.workspace is None and c.workspace_bytes == 0


def test_workspace_size_needs_no_gpu_and_grows_with_the_buffer():
    a = B.bmgd_workspace_bytes(_cfg())
    b = B.bmgd_workspace_bytes(_cfg(buffer_n=2000))
    assert a >= 2 * (1000 * 100 * 4 + 1000 * 4) and b > a + 2 * 1000 * 100 * 4 - 1
    assert a % 256 == 0


def test_invalid_arguments_are_rejected_without_a_device():
    bad = [dict(p=0), dict(buffer_n=0), dict(buffer_n=1 << 30), dict(batch_n=0), dict(batch_n=1001),
           dict(lr=0.0), dict(lr=float("nan")), dict(lr=float("inf")), dict(lr=-1.0), dict(passes=0),
           dict(model=7), dict(x_dtype=1), dict(reshuffle=5), dict(chain=9), dict(n_workgroups=-1),
           dict(n_workgroups=257), dict(p=4100), dict(p=2050), dict(p=1025), dict(workspace=8),
           dict(model=2, n_classes=1, x_dtype=1), dict(model=2, n_classes=10, x_dtype=0)]
    for kw in bad:
        cfg = _cfg(**kw)
        assert B.bmgd_workspace_bytes(cfg) == 0, kw
        rc, h = B.bmgd_create_ex(cfg)
        assert rc == B.BMGD_EINVAL and h is None, kw
        assert B.bmgd_last_error(None) != ""
    assert B.bmgd_create(0, 10, 10, 0.1, 1) is None
    for fn in (B.bmgd_sync, B.bmgd_run_buffer):
        assert fn(None) == B.BMGD_EINVAL
    B.bmgd_destroy(None)                        # ignored


def test_no_silent_cpu_path():
    """Without a GPU, creating a context must fail with BMGD_EHIP rather than compute anywhere else."""
    import torch
    if torch.cuda.is_available():
        return
    rc, h = B.bmgd_create_ex(_cfg())
    assert rc == B.BMGD_EHIP and h is None


def test_null_contexts_and_readers_are_rejected():
    assert B.bmgd_swa_update(None) == B.BMGD_EINVAL
    assert B.bmgd_swa_reset(None) == B.BMGD_EINVAL
    assert B.bmgd_set_row_subset(None, None, 0) == B.BMGD_EINVAL
    assert B.bmgd_run_buffer_adaptive(None, None, None, None, 0, None, 1, 1)[0] == B.BMGD_EINVAL
    assert B.bmgd_run_buffer_adaptive_reader(None, None, None, None, 1, 1)[0] == B.BMGD_EINVAL
    assert B.bmgd_load_from_reader(None, None)[0] == B.BMGD_EINVAL
    assert B.bmgd_reader_acquire(None)[0] == B.BMGD_EINVAL
    assert B.bmgd_reader_release(None) == B.BMGD_EINVAL
    assert B.bmgd_reader_stats(None)[0] == B.BMGD_EINVAL
    B.bmgd_reader_close(None)                   # ignored


def test_reader_arguments_are_checked_before_any_device_call(tmp_path):
    import numpy as np
    fx, fy = tmp_path / "x.bin", tmp_path / "y.bin"
    np.zeros((50, 3), dtype=np.float32).tofile(fx)
    np.zeros(50, dtype=np.float32).tofile(fy)
    ok = dict(p=3, x_dtype=B.BMGD_F32, n_rows=50, buffer_n=20, ring_slots=2, loop=0)
    for kw in (dict(p=0), dict(n_rows=0), dict(n_rows=51), dict(buffer_n=0), dict(buffer_n=1 << 30), dict(ring_slots=1),
               dict(ring_slots=65), dict(x_dtype=3)):
        a = dict(ok, **kw)
        rc, h = B.bmgd_reader_open(str(fx), str(fy), a["p"], a["x_dtype"], a["n_rows"], a["buffer_n"], a["ring_slots"], a["loop"])
        assert rc == B.BMGD_EINVAL and h is None, kw
        assert B.bmgd_reader_last_error(None) != ""
    rc, h = B.bmgd_reader_open(str(tmp_path / "nothing.bin"), str(fy), 3, B.BMGD_F32, 50, 20, 2, 0)
    assert rc == B.BMGD_EINVAL and "cannot open" in B.bmgd_reader_last_error(None)
    import torch
    if not torch.cuda.is_available():
        # the ring is pinned memory from the HIP runtime: without a device the open fails, it does not fall back
        rc, h = B.bmgd_reader_open(str(fx), str(fy), 3, B.BMGD_F32, 50, 20, 2, 0)
        assert rc in (B.BMGD_EHIP, B.BMGD_ENOMEM) and h is None


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """include/bmgd.h must be usable from C (C99, pedantic) and C++; a C program that only needs host-side entry points
    links against libbmgd.so and runs without a device."""
    import shutil
    import subprocess
    src = tmp_path / "use.c"
    src.write_text('#include "bmgd.h"\n#include <stdio.h>\n'
                   'int main(void) {\n'
                   '    bmgd_config c;\n    bmgd_default_config(&c);\n'
                   '    c.p = 100; c.buffer_n = 1000; c.batch_n = 100; c.lr = 0.1; c.passes = 2;\n'
                   '    printf("%lu %d\\n", (unsigned long)bmgd_workspace_bytes(&c), bmgd_sync(NULL));\n'
                   '    return 0;\n}\n')
    inc = os.path.join(ROOT, "include")
    gcc = shutil.which("gcc")
    gxx = shutil.which("g++")
    if not gcc or not gxx:
        pytest.skip("no host compiler")
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", inc, str(src)], check=True)
    subprocess.run([gxx, "-std=c++11", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c++", "-I", inc, str(src)],
                   check=True)
    exe = tmp_path / "use"
    libdir = os.path.dirname(B.LIB_PATH)
    subprocess.run([gcc, "-std=c99", "-I", inc, str(src), "-o", str(exe), "-L", libdir, "-lbmgd", "-Wl,-rpath," + libdir,
                    "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert int(out[0]) == B.bmgd_workspace_bytes(_cfg()) and int(out[1]) == B.BMGD_EINVAL
