"""MI355X-native buffered mini-batch gradient descent: Python face of libbmgd.

Importing this package loads the HIP shared library built from ``csrc/``; if it
is missing the import raises (no CPU or eager fallback exists).
"""
from .binding import *  # noqa: F401,F403
from .binding import Context, Reader, BmgdError, bmgd_config, bmgd_stats, lib, LIB_PATH, EXPORTS  # noqa: F401
