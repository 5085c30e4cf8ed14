"""A seeded sweep over shapes, types, strides and quantiser settings, small enough for the oracle to check every
element: it visits every kernel family and the borders between them (sizes 2 .. 16384, one and several heads,
row widths that do and do not tile a workgroup, row counts around the block sizes, padded rows, every group
size from 8 channels to the whole row)."""
import numpy as np
import pytest

import oracle
from paper_2509_09679_amd import synth

pytestmark = pytest.mark.gpu
gu = pytest.importorskip("gpu_util")


def _cases():
    rng = np.random.default_rng(20250927)
    sizes = [2, 4, 8, 16, 32, 64, 128, 256, 512, 1024, 2048, 4096, 8192, 16384]
    out = []
    for i in range(300):
        n = int(sizes[rng.integers(len(sizes))])
        heads = int(rng.choice([1, 1, 1, 2, 3, 4, 5, 8, 12, 16, 40]))
        while n * heads > 16384:
            heads = max(1, heads // 2)
        budget = 200_000  # elements per case, so that the oracle stays fast
        rows = int(rng.integers(1, max(2, min(70, budget // (n * heads)) + 1)))
        dtype = str(rng.choice(["f32", "f16", "bf16"]))
        pad = int(rng.choice([0, 0, 8, 24]))
        groups = [g for g in (8, 16, 32, 64, 128, 256, 512, 1024, 2048, 4096, 8192, 16384) if g <= n]
        group = int(groups[rng.integers(len(groups))]) if groups else n
        bits = int(rng.choice([2, 4]))
        sd = str(rng.choice(["f16", "f32"]))
        out.append((i, n, heads, rows, dtype, pad, bits, group, sd))
    return out


@pytest.mark.parametrize("i,n,heads,rows,dtype,pad,bits,group,sd", _cases())
def test_sweep(i, n, heads, rows, dtype, pad, bits, group, sd):
    x, th, dy = synth.small_case(n, rows, dtype, heads=heads, seed=1000 + i, with_dy=True)
    x64 = synth.to_f64(x, dtype)
    tag = f"case {i}: n={n} H={heads} T={rows} {dtype} pad={pad}"
    y_ref = oracle.forward(x64, th, n, heads)
    gu.check_rotated(gu.run_transform(x, th, n, heads, dtype, pad=pad), y_ref, dtype, tag + " fwd")
    gu.check_rotated(gu.run_transform(x, th, n, heads, dtype, inverse=True, pad=pad),
                     oracle.inverse(x64, th, n, heads), dtype, tag + " inv")
    if group >= 8:
        codes, scales = gu.run_fwd_quant(x, th, n, heads, dtype, bits, group, sd)
        gu.check_fused_codes(codes, scales, y_ref, bits, group, sd, dtype, tag + f" int{bits} g={group} {sd}")
        yq, hist = gu.run_fwd_fakequant(x, th, n, heads, dtype, bits, group, sd)
        c = oracle.unpack_codes(codes, bits)
        want = synth.cast_storage(oracle.dequantize(c, scales.astype(np.float32), group).astype(np.float64), dtype)
        u = np.uint16 if dtype != "f32" else np.uint32
        np.testing.assert_array_equal(yq.view(u), want.view(u), err_msg=tag + " fake-quantised values")
        np.testing.assert_array_equal(hist, oracle.bin_histogram(c, bits), err_msg=tag + " histogram")
    # backward: rows without the x100 outlier channels, as in the backward workload (with them, float32 rounding
    # of the large elements that pass through a pair exceeds 1e-5 of a small pair's own products)
    x, _, dy = synth.small_case(n, rows, dtype, heads=heads, seed=2000 + i, with_dy=True, outliers=0)
    x64 = synth.to_f64(x, dtype)
    rdx, rdth, ab = oracle.backward(x64, synth.to_f64(dy, dtype), th, n, heads)
    dx, dth = gu.run_bwd(x, dy, th, n, heads, dtype, pad=pad)
    gu.check_rotated(dx, rdx, dtype, tag + " dx")
    # With a handful of rows there is no averaging: an angle whose own products nearly vanish (cancellation inside
    # the rotations) still carries the float32 rounding of the ordinary-sized elements of its layer, so its bound
    # is taken relative to the layer's median product sum; the norm-wise bound holds as it is.
    floor = np.median(ab, axis=2, keepdims=True)
    gu.check_dtheta(dth, rdth, np.maximum(ab, floor) if rows < 32 else ab, what=tag + " dtheta")
    d = np.abs(dth.astype(np.float64) - rdth)
    assert np.linalg.norm(d) <= 1e-5 * np.linalg.norm(ab), tag + " dtheta norm"


def _deep_cases():
    # the same idea with many rows per workgroup, so that the kernels' row buffers and input slots are reused
    # dozens of times (n >= 256, where a workgroup pipelines its rows through LDS)
    rng = np.random.default_rng(77)
    out = []
    for i in range(16):
        n = int(rng.choice([256, 512, 1024, 2048, 4096, 4096, 8192, 8192]))
        heads = int(rng.choice([1, 1, 2])) if n <= 2048 else 1
        rows = int(rng.integers(2500, 6000)) * 4096 // (n * heads)
        dtype = str(rng.choice(["f32", "f16", "bf16"]))
        pad = int(rng.choice([0, 8]))
        groups = [g for g in (32, 64, 128, 128, 512, n) if g <= n]
        out.append((i, n, heads, rows, dtype, pad, int(rng.choice([2, 4])), int(groups[rng.integers(len(groups))]),
                    str(rng.choice(["f16", "f32"]))))
    return out


@pytest.mark.parametrize("i,n,heads,rows,dtype,pad,bits,group,sd", _deep_cases())
def test_sweep_many_rows(i, n, heads, rows, dtype, pad, bits, group, sd):
    x, th, _ = synth.small_case(n, rows, dtype, heads=heads, seed=3000 + i)
    x64 = synth.to_f64(x, dtype)
    tag = f"deep case {i}: n={n} H={heads} T={rows} {dtype} pad={pad}"
    y_ref = oracle.forward(x64, th, n, heads)
    gu.check_rotated(gu.run_transform(x, th, n, heads, dtype, pad=pad), y_ref, dtype, tag + " fwd")
    gu.check_rotated(gu.run_transform(x, th, n, heads, dtype, inverse=True, pad=pad),
                     oracle.inverse(x64, th, n, heads), dtype, tag + " inv")
    codes, scales = gu.run_fwd_quant(x, th, n, heads, dtype, bits, group, sd)
    gu.check_fused_codes(codes, scales, y_ref, bits, group, sd, dtype, tag + f" int{bits} g={group} {sd}")
    yq, hist = gu.run_fwd_fakequant(x, th, n, heads, dtype, bits, group, sd)
    c = oracle.unpack_codes(codes, bits)
    want = synth.cast_storage(oracle.dequantize(c, scales.astype(np.float32), group).astype(np.float64), dtype)
    u = np.uint16 if dtype != "f32" else np.uint32
    np.testing.assert_array_equal(yq.view(u), want.view(u), err_msg=tag + " fake-quantised values")
    np.testing.assert_array_equal(hist, oracle.bin_histogram(c, bits), err_msg=tag + " histogram")
