"""Plain fp64 CPU reference for buffered mini-batch gradient descent.

TEST INFRASTRUCTURE ONLY: nothing here is part of the GPU library and nothing
here may be imported by it.  Only the tests, the smoke check and the
benchmark's CPU-baseline leg use this package.

Pinned functions (see tests/test_oracle_*.py): perm.perm, bmgd.minibatch_gradient,
bmgd.loss, bmgd.BMGD.run_buffer, bmgd.run.  None is "parity unpinned" at small
scale; final estimates of the large synthetic runs have no published value to
compare with and rest on those small-scale pins.
"""
