"""CPU oracle (test infrastructure) for the 2-bit-weight matmul.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline
leg may import this package.  It wraps ``w2_oracle.c`` (plain C, built with
gcc) through ctypes and holds no arithmetic of its own: every function here
marshals numpy arrays and calls the C routine of the same name.
"""
from .w2_oracle import *  # noqa: F401,F403
