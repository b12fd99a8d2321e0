"""Pins for the oracle's mini-batch partition (Algorithm 1, "random partition of the buffer";
Section 2.2: the parts are disjoint, cover the buffer and have n rows each)."""
import os

import numpy as np
import pytest

from oracle import perm as P

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "perm_small.txt")


@pytest.mark.parametrize("N0", [1, 2, 3, 4, 5, 7, 8, 15, 16, 17, 63, 64, 65, 255, 257, 1000, 4097])
def test_is_bijection_and_forms_agree(N0):
    for seed, b, t in [(0, 0, 1), (0, 0, 2), (7, 3, 1), ((5 << 32) | 9, 11, 0)]:
        v = P.perm(seed, b, t, N0)
        assert v.dtype == np.int32 and v.shape == (N0,)
        assert np.array_equal(np.sort(v), np.arange(N0))
        assert v.tolist() == P.perm_scalar(seed, b, t, N0)


@pytest.mark.parametrize("N0", [2, 3, 5, 11, 16])
def test_brute_force_cycle_table(N0):
    """Tabulate E on its whole domain, check it is a bijection there, then follow cycles by hand."""
    h = P.half_width(N0)
    dom = 1 << (2 * h)
    assert N0 <= dom < 4 * N0 or N0 <= 2
    keys = P.round_keys(3, 2, 1)
    table = [P.feistel_scalar(x, keys, h) for x in range(dom)]
    assert sorted(table) == list(range(dom))
    for x in range(dom):                      # a true Feistel network inverts round by round
        assert P.feistel_inverse_scalar(table[x], keys, h) == x
    want = []
    for j in range(N0):
        x = table[j]
        while x >= N0:
            x = table[x]
        want.append(x)
    assert P.perm(3, 2, 1, N0).tolist() == want


def test_depends_on_seed_buffer_and_pass():
    N0 = 2000
    base = P.perm(0, 0, 1, N0)
    assert np.array_equal(base, P.perm(0, 0, 1, N0))          # deterministic
    for other in [P.perm(0, 0, 2, N0), P.perm(0, 1, 1, N0), P.perm(1, 0, 1, N0), P.perm(1 << 32, 0, 1, N0)]:
        assert np.mean(other == base) < 0.01                   # ~1/N0 coincidences expected


def test_minibatches_are_a_partition():
    N0, n = 1000, 96                                           # ragged last batch of 40
    parts = P.minibatches(P.perm(0, 5, 2, N0), n)
    assert [len(s) for s in parts] == [96] * 10 + [40]
    allrows = np.concatenate(parts)
    assert np.array_equal(np.sort(allrows), np.arange(N0))     # disjoint and covering


def test_membership_is_close_to_uniform():
    """Over many passes every row should land in every mini-batch about equally often."""
    N0, n, trials = 64, 16, 4000
    counts = np.zeros((N0, N0 // n))
    for t in range(1, trials + 1):
        v = P.perm(0, t // 50, t % 50 + 1, N0)
        pos = np.empty(N0, dtype=np.int64)
        pos[v] = np.arange(N0)
        counts[np.arange(N0), pos // n] += 1
    expected = trials / (N0 // n)
    chi2 = ((counts - expected) ** 2 / expected).sum()
    dof = N0 * (N0 // n - 1)
    assert chi2 < dof + 6 * np.sqrt(2 * dof)
    # and the first position is not stuck on a few values
    firsts = {int(P.perm(0, b, 1, N0)[0]) for b in range(400)}
    assert len(firsts) > 55


def test_golden_values():
    """Values written by tests/golden/make_golden.py (which calls only the oracle)."""
    with open(GOLDEN) as fh:
        lines = [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]
    assert len(lines) >= 6
    for ln in lines:
        seed, b, t, N0 = (int(v) for v in ln[:4])
        want = [int(v) for v in ln[4:]]
        assert P.perm(seed, b, t, N0)[:len(want)].tolist() == want


def test_mix_reference_values():
    """Hand evaluation of the mixer on x = 1, step by step, in plain integers."""
    x = 1
    x ^= x >> 16                       # 1
    x = (x * 0x7FEB352D) % 2**32       # 0x7FEB352D
    assert x == 0x7FEB352D
    x ^= x >> 15                       # 0x7FEB352D ^ 0xFFD6
    assert x == 0x7FEB352D ^ 0xFFD6
    x = (x * 0x846CA68B) % 2**32
    x ^= x >> 16
    assert P.mix_scalar(1) == x
    assert P.mix_scalar(0) == 0
    assert int(P._mix_vec(np.array([1], dtype=np.uint32))[0]) == x
