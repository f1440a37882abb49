"""Worker of bench.py's CPU baseline: one process, one tree, the oracle as it stands.

Imports numpy and the oracle only (no torch, nothing of the HIP package), so that a worker
started with the `spawn` method costs a fraction of a second and holds no GPU state.
"""

import time

import numpy as np  # noqa: F401  (the arrays arrive as numpy arrays)


def verify_repeatedly(args):
    """Verify one tree over and over until `budget_s` seconds of wall time have passed.
    Returns (trees verified, seconds used)."""
    method, parent, tokens, zt, zd, T, u, ud, budget_s = args
    from oracle import mpv_oracle as orc
    done = 0
    t0 = time.perf_counter()
    while True:
        orc.verify_tree(method, parent, tokens, zt, zd, T, u, ud)
        done += 1
        elapsed = time.perf_counter() - t0
        if elapsed >= budget_s:
            return done, elapsed
