"""Pins for the oracle's Dequant, bin histogram and uniformity KL (paper, "Loss Function" and
"Uniformity Regularization"): hand-computed values, closed forms, properties, library routines."""
import math

import numpy as np
import pytest
from scipy.stats import entropy

import oracle


def test_dequant_hand_vector():
    codes = np.array([[1, -1, 0, 1, -2, 0, 0, 1]], dtype=np.int8)
    scales = np.array([[0.5, 2.0]], dtype=np.float32)
    np.testing.assert_array_equal(oracle.dequantize(codes, scales, 4),
                                  np.array([[0.5, -0.5, 0.0, 0.5, -4.0, 0.0, 0.0, 2.0]], dtype=np.float32))


@pytest.mark.parametrize("bits,group,sd", [(4, 16, "f32"), (2, 32, "f16"), (4, 64, "f16"), (2, 64, "f32")])
def test_dequant_error_bound_and_idempotence(bits, group, sd):
    rng = np.random.default_rng(bits * 100 + group)
    y = (rng.standard_t(3, size=(37, 256)) * 3).astype(np.float32)
    q, s = oracle.quantize(y, group, bits, sd)
    yq = oracle.dequantize(q, s, group)
    srep = np.repeat(s, group, axis=1).astype(np.float64)
    # rounding to the nearest code: off by at most half a step, unless the value was clipped (binary16 scales
    # can round below amax / qmax), in which case it lies beyond the last code
    qmax = (1 << (bits - 1)) - 1
    err = np.abs(y.astype(np.float64) - yq.astype(np.float64))
    inside = np.abs(y.astype(np.float64)) <= srep * (qmax + 0.5)
    assert np.all(err[inside] <= srep[inside] * 0.5 * (1 + 1e-6) + 1e-30)
    # Quant(Dequant(q)) = q with the same scales: every dequantised value sits exactly on a code
    # (compare by quantising each group again: the group's abs-max is qmax' * s for the largest |q| present)
    t = np.rint(yq.astype(np.float64) / np.where(srep == 0, 1, srep))
    np.testing.assert_array_equal(t.astype(np.int8), q)


def test_histogram_counts_and_library_bincount():
    rng = np.random.default_rng(5)
    for bits in (2, 4):
        off = 1 << (bits - 1)
        codes = rng.integers(-off, off, size=(13, 96)).astype(np.int8)
        h = oracle.bin_histogram(codes, bits)
        assert h.dtype == np.uint64 and h.sum() == codes.size
        np.testing.assert_array_equal(h, np.bincount(codes.ravel().astype(np.int64) + off, minlength=1 << bits))
    # hand vector
    np.testing.assert_array_equal(oracle.bin_histogram(np.array([[1, -1, 0, 1, -2, 0, 0, 1]], dtype=np.int8), 2),
                                  np.array([1, 1, 3, 3], dtype=np.uint64))


def test_uniformity_kl_closed_forms():
    for bits in (2, 4):
        nb = 1 << bits
        assert oracle.uniformity_kl(np.full(nb, 7, dtype=np.uint64), bits) == 0.0          # uniform: zero
        one = np.zeros(nb, dtype=np.uint64); one[3] = 11
        assert abs(oracle.uniformity_kl(one, bits) - bits * math.log(2)) < 1e-15           # one bin: log 2^b
        assert oracle.uniformity_kl(np.zeros(nb, dtype=np.uint64), bits) == 0.0            # empty: defined as 0
    # worked by hand: P = (1, 1, 3, 3) / 8:  2 * (1/8) ln(1/2) + 2 * (3/8) ln(3/2)
    want = 0.25 * math.log(0.5) + 0.75 * math.log(1.5)
    assert abs(oracle.uniformity_kl(np.array([1, 1, 3, 3], dtype=np.uint64), 2) - want) < 1e-15
    # scale invariance and a library routine
    rng = np.random.default_rng(1)
    h = rng.integers(0, 1000, size=16).astype(np.uint64)
    kl = oracle.uniformity_kl(h, 4)
    assert abs(oracle.uniformity_kl(h * np.uint64(3), 4) - kl) < 1e-15
    assert abs(kl - entropy(h.astype(np.float64), np.full(16, 1 / 16))) < 1e-12
    assert kl >= 0.0


def test_int2_histogram_of_a_quantised_row_has_an_empty_lowest_bin():
    # s = amax / qmax with qmax = 1: codes are ternary, bin -2 stays empty with float32 scales (clip range as written)
    rng = np.random.default_rng(9)
    y = rng.standard_normal((64, 128)).astype(np.float32)
    q, _ = oracle.quantize(y, 32, 2, "f32")
    h = oracle.bin_histogram(q, 2)
    assert h[0] == 0 and h.sum() == y.size and h[1] > 0 and h[3] > 0
