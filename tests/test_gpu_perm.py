"""Bit-exact parity of the device-side partition with the oracle (Algorithm 1's per-pass random partition)."""
import numpy as np
import pytest

from oracle import perm as P

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("N0", [1, 2, 3, 16, 17, 255, 256, 257, 2000, 4097, 100_000, 250_000, 1_000_000])
def test_partition_matches_oracle(N0):
    import paper_2312_08728_amd as B
    for seed in (0, (77 << 32) | 12345):
        ctx = B.Context(4, N0, 1, 0.1, 2, seed=seed)
        try:
            for b, t in [(0, 1), (0, 2), (3, 1), (49, 3), (7, 0)]:
                got = ctx.get_perm(b, t, N0)
                assert np.array_equal(got, P.perm(seed, b, t, N0)), (N0, seed, b, t)
            if N0 > 100:                      # a shorter last buffer draws its own partition of its own length
                short = N0 - 37
                assert np.array_equal(ctx.get_perm(2, 1, short), P.perm(seed, 2, 1, short))
        finally:
            ctx.close()
