"""Oracle for the composite transform of non-power-of-two widths (paper, "Composite Butterfly Transforms
for Non-Power-of-2 Dimensions"):  Q = Q1 (x) Q2  with Q1 a d1 x d1 Cayley-parameterised orthogonal matrix
and Q2 the butterfly B(theta) of size d2 = 2^k (5120 = 40 x 128 in the paper's example).

TEST INFRASTRUCTURE ONLY, numpy in double; shares nothing with the HIP library.

Conventions (this project's; the paper fixes none): an element of a row has index i * d2 + j with
i in [0, d1), j in [0, d2) — the natural reading of "40 x 128" — so that with X the d1 x d2 matrix of
a row,  (Q1 (x) Q2) x  is  Q1 X Q2^T  flattened the same way: the butterfly acts on every length-d2
sub-row, Q1 mixes the d1 sub-rows.  The d1 (d1 - 1) / 2 Cayley parameters fill the strict upper triangle
of the skew-symmetric A row by row (A[i][j] = p, A[j][i] = -p for i < j);  Q1 = (I - A)(I + A)^-1.
"""
from __future__ import annotations

import numpy as np

import oracle


def skew_from_params(params, d1: int) -> np.ndarray:
    params = np.asarray(params, dtype=np.float64)
    assert params.size == d1 * (d1 - 1) // 2
    A = np.zeros((d1, d1))
    iu = np.triu_indices(d1, 1)
    A[iu] = params
    return A - A.T


def cayley(params, d1: int) -> np.ndarray:
    """Q1 = (I - A)(I + A)^-1 in double (float32 parameters are converted exactly)."""
    A = skew_from_params(np.asarray(params, dtype=np.float32), d1)
    I = np.eye(d1)
    return np.linalg.solve((I + A).T, (I - A).T).T  # (I - A) (I + A)^-1


def kron_forward(x, q1, theta, d2: int) -> np.ndarray:
    """y = (Q1 (x) B(theta)) x for every row of x ([T, d1*d2], double)."""
    x = np.asarray(x, dtype=np.float64)
    T = x.shape[0]
    d1 = q1.shape[0]
    z = oracle.forward(x.reshape(T * d1, d2), theta, d2).reshape(T, d1, d2)
    return np.einsum("ik,tkj->tij", np.asarray(q1, dtype=np.float64), z).reshape(T, d1 * d2)


def kron_inverse(y, q1, theta, d2: int) -> np.ndarray:
    """x = (Q1 (x) B(theta))^T y."""
    y = np.asarray(y, dtype=np.float64)
    T = y.shape[0]
    d1 = q1.shape[0]
    z = np.einsum("ki,tkj->tij", np.asarray(q1, dtype=np.float64), y.reshape(T, d1, d2))
    return oracle.inverse(z.reshape(T * d1, d2), theta, d2).reshape(T, d1 * d2)
