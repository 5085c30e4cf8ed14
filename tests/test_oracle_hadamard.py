"""Pins of the Hadamard oracle (CPU): scipy's Sylvester matrix, and the butterfly at pi/4 (paper, "Hadamard as a
Special Case of Butterfly": H_2 = G(pi/4) diag(1, -1))."""
import numpy as np
import pytest
import scipy.linalg

import oracle


@pytest.mark.parametrize("n", [1, 2, 4, 8, 64, 256])
def test_hadamard_equals_scipy_sylvester_matrix(n):
    rng = np.random.default_rng(n)
    x = rng.standard_normal((5, n))
    ref = x @ (scipy.linalg.hadamard(n).astype(np.float64) / np.sqrt(n)).T
    assert np.allclose(oracle.hadamard(x, n), ref, rtol=0, atol=1e-13)


def test_hadamard_blocks_are_independent_and_the_map_is_an_involution():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((4, 3 * 32))
    y = oracle.hadamard(x, 32, heads=3)
    for h in range(3):
        assert np.array_equal(y[:, 32 * h:32 * (h + 1)], oracle.hadamard(x[:, 32 * h:32 * (h + 1)], 32))
    assert np.allclose(oracle.hadamard(y, 32, heads=3), x, atol=1e-13)
    assert np.allclose(np.linalg.norm(y, axis=1), np.linalg.norm(x, axis=1))


@pytest.mark.parametrize("n", [8, 128])
def test_butterfly_with_all_angles_at_a_quarter_pi_is_the_signed_hadamard_rotation(n):
    # B(pi/4) = H_n diag((-1)^popcount(column)) / sqrt(n): two independent routes to the same matrix
    k = n.bit_length() - 1
    theta = np.full((1, k, n // 2), np.pi / 4, dtype=np.float32)
    rng = np.random.default_rng(n)
    x = rng.standard_normal((6, n))
    sign = np.array([(-1.0) ** bin(c).count("1") for c in range(n)])
    assert np.allclose(oracle.forward(x, theta, n), oracle.hadamard(x * sign, n), atol=1e-6)  # float32 angle: pi/4 rounded
