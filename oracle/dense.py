"""Dense definitional form of the butterfly transform, for tiny n only (TEST INFRASTRUCTURE).

Each layer B_i is written out as an n x n matrix exactly as the paper defines it (a Givens block
G(theta) = [[cos, -sin], [sin, cos]] on every index pair (a, a + 2^(i-1)); section "Structure and
Parameterization" and the printed 8x8 layers of the appendix), and the transform is the plain
matrix product with layer 1 applied first:  B = B_k ... B_2 B_1.
"""
from __future__ import annotations

import numpy as np


def pair_indices(n: int, i: int):
    """Index pairs (a, b) of layer i (1-based), in the order of the layer's angles: all a whose
    bit (i-1) is clear, ascending; b = a + 2^(i-1)."""
    h = 1 << (i - 1)
    lows = [a for a in range(n) if not (a & h)]
    return [(a, a + h) for a in lows]


def dense_layer(theta_i, n: int, i: int) -> np.ndarray:
    """n x n matrix of layer i from its n/2 angles (float64)."""
    theta_i = np.asarray(theta_i, dtype=np.float64)
    B = np.zeros((n, n), dtype=np.float64)
    for j, (a, b) in enumerate(pair_indices(n, i)):
        c, s = np.cos(theta_i[j]), np.sin(theta_i[j])
        B[a, a] = c
        B[a, b] = -s
        B[b, a] = s
        B[b, b] = c
    return B


def dense_butterfly(theta, n: int) -> np.ndarray:
    """B = B_k ... B_1 for theta of shape [k, n/2]; float32 angles are widened exactly."""
    k = int(n).bit_length() - 1
    theta = np.asarray(theta).astype(np.float64).reshape(k, n // 2)
    B = np.eye(n)
    for i in range(1, k + 1):
        B = dense_layer(theta[i - 1], n, i) @ B
    return B
