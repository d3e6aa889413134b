"""Shared by the GPU parity tests: tensor <-> oracle conversions and the error metric."""
from oracle.checks import (GRAD_TOL, GRAD_TOL_SAME, ORC_DT, TOL, chain_tol, rel_err, round_like, to_bits, to_f64,  # noqa: F401
                           weights_bits)

import numpy as np


def layer_rows(n_dst, budget, rng=None):
    """Row ranges of a layer to check: all of it, or its head, its tail and blocks of rows inside
    it that straddle multiples of 256 rows (a boundary of every projection tile height) - some of
    them multiples of 2048, where the row tiles wrap around the 8 XCDs."""
    if n_dst <= budget:
        return [(0, n_dst)]
    h = budget // 4
    out = [(0, h), (n_dst - h, n_dst)]
    rng = rng or np.random.default_rng(n_dst)
    n_blocks, w = 8, max(budget // 2 // 8, 16)
    for j in range(n_blocks):
        unit = 2048 if j % 2 else 256
        c = int(rng.integers(1, max(n_dst // unit, 2))) * unit
        lo, hi = max(h, c - w // 2), min(n_dst - h, c + w // 2)
        if hi > lo:
            out.append((lo, hi))
    return out
