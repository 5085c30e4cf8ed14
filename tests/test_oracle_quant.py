"""Pins for the oracle's quantiser: hand-computed vectors, properties that follow from the
definition (paper, equation for Quant/Dequant), the binary16 rounding against numpy's independent
implementation, and the packing layout.  CPU only."""
import numpy as np
import pytest

import oracle


def test_hand_vector_int4():
    # amax = 7 => s = 1, inv = 1: codes are rint(y) with ties to even
    y = np.array([[7.0, -7.0, 0.5, 1.5, 2.5, -0.5, -1.5, 3.49]], np.float32)
    codes, scales = oracle.quantize(y, group=8, bits=4)
    assert scales.tolist() == [[1.0]]
    assert codes.tolist() == [[7, -7, 0, 2, 2, 0, -2, 3]]


def test_hand_vector_int4_scale():
    # amax = 3.5 => s = 0.5 exactly, inv = 2: codes = rint(2 y)
    y = np.array([[3.5, -1.0, 0.25, 0.75, -3.5, 1.3, 0.0, -0.26]], np.float32)
    codes, scales = oracle.quantize(y, group=8, bits=4)
    assert scales.tolist() == [[0.5]]
    assert codes.tolist() == [[7, -2, 0, 2, -7, 3, 0, -1]]


def test_hand_vector_int2_is_ternary():
    # qmax = 1 => s = amax, codes in {-1,0,1}; 0.5*amax is a tie and goes to 0 (even)
    y = np.array([[4.0, 2.0, 2.0001, -4.0, -2.0, -1.9, 0.0, 3.0]], np.float32)
    codes, scales = oracle.quantize(y, group=8, bits=2)
    assert scales.tolist() == [[4.0]]
    assert codes.tolist() == [[1, 0, 1, -1, 0, 0, 0, 1]]


def test_groups_are_independent_runs_of_consecutive_channels():
    y = np.array([[1.0, -0.6, 14.0, 7.0], [0.0, 0.0, -21.0, 3.0]], np.float32)
    codes, scales = oracle.quantize(y, group=2, bits=4)
    # row 0 group 0: amax 1 -> s = 1/7 (rounded), group 1: s = 2; row 1 group 0: zero group
    assert scales[0, 1] == 2.0 and scales[1, 1] == 3.0
    assert scales[0, 0] == np.float32(1.0) / np.float32(7.0)
    assert scales[1, 0] == 0.0
    assert codes.tolist() == [[7, -4, 7, 4], [0, 0, -7, 1]]


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("scale_dtype", ["f32", "f16"])
def test_properties_random(bits, scale_dtype):
    rng = np.random.default_rng(bits * 10 + (scale_dtype == "f16"))
    y = (rng.standard_t(3.0, size=(64, 1024)) * rng.choice([1e-3, 1.0, 50.0], size=(64, 1))).astype(np.float32)
    g = 128
    codes, scales = oracle.quantize(y, g, bits, scale_dtype)
    qmax = 2 ** (bits - 1) - 1
    assert codes.max() <= qmax and codes.min() >= -qmax  # -2^(b-1) unreachable with s = amax/qmax
    cg = codes.reshape(64, -1, g)
    yg = y.reshape(64, -1, g).astype(np.float64)
    s = scales.astype(np.float64)[:, :, None]
    assert (np.abs(cg).max(axis=2) == qmax).all()  # the largest element always maps to +-qmax
    # reconstruction error at most half a step (tiny slack for the float32 reciprocal)
    err = np.abs(yg - s * cg)
    slack = 2e-3 if scale_dtype == "f16" else 1e-6
    assert (err <= s * (0.5 + slack) + 1e-30).all()
    # idempotence: quantising the dequantised values returns the same codes
    deq = (scales[:, :, None] * cg.astype(np.float32)).reshape(64, -1).astype(np.float32)
    codes2, scales2 = oracle.quantize(deq, g, bits, scale_dtype)
    assert np.array_equal(codes2, codes)
    if scale_dtype == "f32":
        assert np.array_equal(scales2, scales)
        # literal definition in float64: round(y / s); may differ only at half-way cases
        lit = np.clip(np.rint(yg / s), -(qmax + 1), qmax)
        frac = np.mean(lit != cg)
        assert frac < 1e-5
    else:
        assert np.array_equal(scales, scales.astype(np.float16).astype(np.float32))


def test_scale_equals_amax_over_qmax_in_float32():
    rng = np.random.default_rng(11)
    y = rng.standard_normal((16, 256)).astype(np.float32)
    _, s4 = oracle.quantize(y, 64, 4)
    amax = np.abs(y).reshape(16, 4, 64).max(axis=2)
    assert np.array_equal(s4, amax / np.float32(7.0))
    _, s2 = oracle.quantize(y, 64, 2)
    assert np.array_equal(s2, amax)


def test_zero_group_and_f16_saturation():
    y = np.zeros((1, 8), np.float32)
    codes, scales = oracle.quantize(y, 8, 4, "f16")
    assert not codes.any() and scales[0, 0] == 0.0
    y = np.full((1, 8), 3.0e38, np.float32)
    codes, scales = oracle.quantize(y, 8, 2, "f16")
    assert scales[0, 0] == 65504.0 and (codes == 1).all()
    # a scale that underflows binary16 entirely becomes 0 => codes 0
    y = np.full((1, 8), 1e-9, np.float32)
    codes, scales = oracle.quantize(y, 8, 4, "f16")
    assert scales[0, 0] == 0.0 and not codes.any()
    # binary16-subnormal scale rounded down: ratio exceeds qmax and is clipped
    y = np.array([[8.5e-8 * 7] * 8], np.float32)
    codes, scales = oracle.quantize(y, 8, 4, "f16")
    assert scales[0, 0] == np.float32(2.0 ** -24) and (codes == 7).all()


def test_f16_rounding_matches_numpy():
    rng = np.random.default_rng(2)
    vals = np.concatenate([
        rng.standard_normal(2000).astype(np.float32) * np.float32(10.0) ** rng.integers(-9, 5, 2000).astype(np.float32),
        np.array([0.0, 65504.0, 65519.9, 65520.0, 1e5, 6.1e-5, 5.96e-8, 2.98e-8, 2.9802325e-8, 3e-8, 1e-10],
                 np.float32),
        (np.arange(1024, 2048, dtype=np.float32) + 0.5) * np.float32(2.0 ** -5),  # exact ties
    ])
    for v in vals:
        for sv in (v, -v):
            want = int(np.float32(sv).astype(np.float16).view(np.uint16))
            assert oracle.f32_to_f16_bits(float(sv)) == want
    for h in list(range(0, 0x7C00, 37)) + [0x7BFF, 0x0001, 0x03FF, 0x0400, 0x8001]:
        assert oracle.f16_bits_to_f32(h) == float(np.uint16(h).view(np.float16))


@pytest.mark.parametrize("bits", [2, 4])
def test_pack_layout_and_roundtrip(bits):
    # parity unpinned by the paper: the layout is this project's (little-endian fields, two's complement)
    if bits == 4:
        codes = np.array([[1, -1, 7, -8, 0, 3, -7, 2]], np.int8)
        want = [[0xF1, 0x87, 0x30, 0x29]]
    else:
        codes = np.array([[1, -1, 0, -2, 0, 0, 1, 1]], np.int8)
        want = [[0b10001101, 0b01010000]]
    packed = oracle.pack_codes(codes, bits)
    assert packed.tolist() == want
    assert np.array_equal(oracle.unpack_codes(packed, bits), codes)
    rng = np.random.default_rng(bits)
    c = rng.integers(-(2 ** (bits - 1)), 2 ** (bits - 1), size=(5, 64)).astype(np.int8)
    assert np.array_equal(oracle.unpack_codes(oracle.pack_codes(c, bits), bits), c)
