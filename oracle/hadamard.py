"""Fixed Walsh-Hadamard rotation, plain numpy in double (test infrastructure only, like everything under oracle/).

Paper, section "Hadamard Transform": H_1 = [1], H_2n = [[H_n, H_n], [H_n, -H_n]] (Sylvester's construction); the
rotation used as the fixed baseline is H_n / sqrt(n).  Written out as the recursion's butterflies: for strides
1, 2, 4, ..., n/2 every pair (a, a + stride) becomes (a + b, a - b).
"""
from __future__ import annotations

import numpy as np


def hadamard(x, n: int, heads: int = 1):
    """y = H_n x / sqrt(n) for every block of n consecutive elements of every row of x (float64 in and out)."""
    x = np.asarray(x, dtype=np.float64)
    rows, w = x.shape
    assert w == n * heads and n >= 1 and (n & (n - 1)) == 0
    y = x.reshape(rows * heads, n).copy()
    h = 1
    while h < n:
        v = y.reshape(-1, n // (2 * h), 2, h)
        a = v[:, :, 0, :].copy()
        b = v[:, :, 1, :].copy()
        v[:, :, 0, :] = a + b
        v[:, :, 1, :] = a - b
        h *= 2
    return (y / np.sqrt(float(n))).reshape(rows, w)
