"""Pins for the composite-transform oracle (paper, "Composite Butterfly Transforms for Non-Power-of-2
Dimensions"): closed forms, the library's Kronecker product, the invariants and counts the paper states."""
import math

import numpy as np

import oracle
from oracle import dense, kron


def test_cayley_2x2_is_a_rotation_by_twice_the_arctangent():
    # (I - A)(I + A)^-1 with A = [[0, a], [-a, 0]]  =  1/(1+a^2) [[1-a^2, -2a], [2a, 1-a^2]]
    for a in (0.0, 0.3, -1.7, 5.0):
        q = kron.cayley([a], 2)
        phi = 2.0 * math.atan(a)
        want = np.array([[math.cos(phi), -math.sin(phi)], [math.sin(phi), math.cos(phi)]])
        np.testing.assert_allclose(q, want, atol=1e-7)  # the parameter is float32
    np.testing.assert_array_equal(kron.cayley([0.0] * 3, 3), np.eye(3))  # A = 0: identity


def test_cayley_is_orthogonal_and_matches_its_definition():
    rng = np.random.default_rng(3)
    for d1 in (3, 5, 40):
        p = rng.standard_normal(d1 * (d1 - 1) // 2).astype(np.float32)
        q = kron.cayley(p, d1)
        np.testing.assert_allclose(q.T @ q, np.eye(d1), atol=1e-12)
        A = kron.skew_from_params(p, d1)
        np.testing.assert_allclose(A.T, -A)
        assert np.all(np.diag(A) == 0)
        np.testing.assert_allclose(q @ (np.eye(d1) + A), np.eye(d1) - A, atol=1e-11)
        assert abs(np.linalg.det(q) - 1.0) < 1e-10  # Cayley images have determinant +1


def test_paper_counts_for_5120():
    d1, d2 = 40, 128
    assert d1 * d2 == 5120
    assert d1 * (d1 - 1) // 2 == 780 and (d2 // 2) * 7 == 448 and 780 + 448 == 1228
    assert round(5120 * 5120 / 1228) == 21347  # the reduction factor the paper quotes


def test_composite_equals_the_dense_kronecker_product():
    rng = np.random.default_rng(4)
    for d1, d2 in ((3, 8), (5, 16), (6, 4)):
        k = int(math.log2(d2))
        theta = rng.uniform(-math.pi, math.pi, size=(1, k, d2 // 2)).astype(np.float32)
        q1 = kron.cayley(rng.standard_normal(d1 * (d1 - 1) // 2).astype(np.float32), d1)
        bdense = dense.dense_butterfly(theta[0].astype(np.float64), d2)
        big = np.kron(q1, bdense)
        x = rng.standard_normal((7, d1 * d2))
        np.testing.assert_allclose(kron.kron_forward(x, q1, theta, d2), x @ big.T, atol=1e-12)
        np.testing.assert_allclose(kron.kron_inverse(x, q1, theta, d2), x @ big, atol=1e-12)
        np.testing.assert_allclose(big.T @ big, np.eye(d1 * d2), atol=1e-12)  # orthogonality is preserved


def test_composite_invariants_at_5120():
    rng = np.random.default_rng(5)
    d1, d2 = 40, 128
    theta = rng.uniform(-math.pi, math.pi, size=(1, 7, 64)).astype(np.float32)
    q1 = kron.cayley(0.2 * rng.standard_normal(780).astype(np.float32), d1)
    x = rng.standard_normal((5, 5120))
    y = kron.kron_forward(x, q1, theta, d2)
    np.testing.assert_allclose(np.linalg.norm(y, axis=1), np.linalg.norm(x, axis=1), rtol=1e-12)
    np.testing.assert_allclose(kron.kron_inverse(y, q1, theta, d2), x, atol=1e-12)
    # the two factors act on different indices: their order does not matter
    z = np.einsum("ik,tkj->tij", q1, x.reshape(5, d1, d2)).reshape(5 * d1, d2)
    np.testing.assert_allclose(oracle.forward(z, theta, d2).reshape(5, 5120), y, atol=1e-12)
    # identity factors
    np.testing.assert_array_equal(kron.kron_forward(x, np.eye(d1), np.zeros_like(theta), d2), x)
