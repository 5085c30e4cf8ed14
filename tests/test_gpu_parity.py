"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Rotated values within 1e-5 (float32 I/O) / 2e-3 (half-precision I/O), quantiser codes and
scales bit-exact when the quantiser is fed the oracle's rotated values."""
import math

import numpy as np
import pytest

import oracle
from paper_2509_09679_amd import synth

pytestmark = pytest.mark.gpu

gu = pytest.importorskip("gpu_util")


def _ref_fwd(x_store, theta, n, heads, dtype):
    return oracle.forward(synth.to_f64(x_store, dtype), theta, n, heads)


# ---- transform: shape sweep (several tiles, ragged tails, every n) ----------------------------

@pytest.mark.parametrize("n", [2, 4, 8, 16, 32, 64, 128, 256, 512, 1024, 2048, 4096, 8192, 16384])
def test_fwd_inv_all_sizes_f32(n):
    rows = 37 if n <= 1024 else 5
    x, th, _ = synth.small_case(n, rows, "f32", seed=n)
    y = gu.run_transform(x, th, n, 1, "f32")
    gu.check_rotated(y, _ref_fwd(x, th, n, 1, "f32"), "f32", f"fwd n={n}")
    xi = gu.run_transform(x, th, n, 1, "f32", inverse=True)
    gu.check_rotated(xi, oracle.inverse(synth.to_f64(x, "f32"), th, n), "f32", f"inv n={n}")


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("n,heads,rows", [(128, 1, 100), (128, 32, 67), (64, 3, 33), (4096, 1, 19),
                                           (8192, 1, 7), (512, 2, 45)])
def test_fwd_inv_half_types(dtype, n, heads, rows):
    x, th, _ = synth.small_case(n, rows, dtype, heads=heads, seed=7)
    y = gu.run_transform(x, th, n, heads, dtype)
    gu.check_rotated(y, _ref_fwd(x, th, n, heads, dtype), dtype, f"fwd {dtype} n={n} H={heads}")
    xi = gu.run_transform(x, th, n, heads, dtype, inverse=True)
    gu.check_rotated(xi, oracle.inverse(synth.to_f64(x, dtype), th, n, heads), dtype, f"inv {dtype} n={n}")


@pytest.mark.parametrize("n,heads,dtype", [(128, 1, "f32"), (4096, 1, "f16"), (128, 32, "bf16")])
def test_padded_rows_and_inplace(n, heads, dtype):
    x, th, _ = synth.small_case(n, 21, dtype, heads=heads, seed=3)
    ref = _ref_fwd(x, th, n, heads, dtype)
    y = gu.run_transform(x, th, n, heads, dtype, pad=24)
    gu.check_rotated(y, ref, dtype, "padded")
    y2 = gu.run_transform(x, th, n, heads, dtype, inplace=True)
    assert np.array_equal(y2, gu.run_transform(x, th, n, heads, dtype))


def test_single_row_and_zero_rows():
    import torch
    from paper_2509_09679_amd import binding as B

    x, th, _ = synth.small_case(4096, 1, "f16", seed=1)
    gu.check_rotated(gu.run_transform(x, th, 4096, 1, "f16"), _ref_fwd(x, th, 4096, 1, "f16"), "f16", "T=1")
    thd = torch.from_numpy(th).cuda()
    plan = B.alloc_plan(thd, 4096, 1)
    e = torch.empty((0, 4096), dtype=torch.float16, device="cuda:0")
    r = B.make_rows(e, 4096, 1)
    B.bq_butterfly_fwd(e, e, plan, r)  # no launch, no error
    torch.cuda.synchronize()


def test_theta_zero_is_identity_and_roundtrip():
    n = 4096
    x, th, _ = synth.small_case(n, 9, "f32", seed=5)
    y = gu.run_transform(x, np.zeros_like(th), n, 1, "f32")
    assert np.array_equal(y, x)
    y = gu.run_transform(x, th, n, 1, "f32")
    xb = gu.run_transform(y, th, n, 1, "f32", inverse=True)
    gu.check_rotated(xb, synth.to_f64(x, "f32"), "f32", "inverse o forward", tol=2e-5)


def test_hadamard_angles():
    n = 1024
    k = 10
    th = np.full((1, k, n // 2), math.pi / 4, np.float32)
    x, _, _ = synth.small_case(n, 4, "f32", seed=2)
    gu.check_rotated(gu.run_transform(x, th, n, 1, "f32"), _ref_fwd(x, th, n, 1, "f32"), "f32", "theta=pi/4")


def test_cosines_near_zero_take_the_safe_path():
    # theta = pi/2 everywhere: cos = -4.4e-8 in float32; scale-deferred tables would overflow
    for n, dtype in [(4096, "f16"), (128, "f32"), (8192, "bf16")]:
        k = n.bit_length() - 1
        th = np.full((1, k, n // 2), np.float32(math.pi / 2), np.float32)
        th[0, ::2, ::3] = np.float32(-math.pi / 2)
        x, _, _ = synth.small_case(n, 6, dtype, seed=4)
        gu.check_rotated(gu.run_transform(x, th, n, 1, dtype), _ref_fwd(x, th, n, 1, dtype), dtype, f"pi/2 n={n}")
        gu.check_rotated(gu.run_transform(x, th, n, 1, dtype, inverse=True),
                         oracle.inverse(synth.to_f64(x, dtype), th, n), dtype, f"pi/2 inv n={n}")


@pytest.mark.parametrize("n,heads,rows,dtype", [(8, 1, 1000, "f16"), (16, 4, 301, "bf16"), (32, 64, 77, "f16"),
                                                 (64, 2, 515, "f32"), (128, 16, 130, "f16"), (128, 2, 49, "bf16"),
                                                 (64, 32, 3, "f32")])
def test_small_transforms_many_heads_ragged_rows(n, heads, rows, dtype):
    x, th, _ = synth.small_case(n, rows, dtype, heads=heads, seed=21)
    gu.check_rotated(gu.run_transform(x, th, n, heads, dtype), _ref_fwd(x, th, n, heads, dtype), dtype,
                     f"small fwd n={n} H={heads}")
    gu.check_rotated(gu.run_transform(x, th, n, heads, dtype, inverse=True),
                     oracle.inverse(synth.to_f64(x, dtype), th, n, heads), dtype, f"small inv n={n} H={heads}")


@pytest.mark.parametrize("n,heads,bits,group,scale_dtype,rows", [(64, 4, 4, 16, "f16", 100), (128, 16, 2, 64, "f32", 37),
                                                                  (32, 8, 4, 32, "f32", 250), (16, 2, 2, 8, "f16", 999)])
def test_small_transforms_fused_quant(n, heads, bits, group, scale_dtype, rows):
    x, th, _ = synth.small_case(n, rows, "bf16", heads=heads, seed=22)
    y_ref = _ref_fwd(x, th, n, heads, "bf16")
    codes, scales = gu.run_fwd_quant(x, th, n, heads, "bf16", bits, group, scale_dtype)
    gu.check_fused_codes(codes, scales, y_ref, bits, group, scale_dtype, "bf16", f"small n={n}")


# ---- quantiser: bit-exact when fed the oracle's rotated values ---------------------------------

@pytest.mark.parametrize("n,heads,bits,group,scale_dtype",
                         [(128, 1, 4, 128, "f32"), (4096, 1, 4, 128, "f16"), (4096, 1, 2, 128, "f16"),
                          (128, 32, 4, 128, "f32"), (4096, 1, 4, 4096, "f32"), (256, 2, 2, 8, "f16"),
                          (4096, 1, 2, 32, "f32"), (1024, 1, 4, 64, "f16"), (64, 32, 4, 8, "f16"),
                          (128, 16, 2, 128, "f16"), (4096, 1, 4, 8, "f16"), (4096, 1, 4, 128, "f32")])
def test_quantiser_bit_exact_on_oracle_rotated_values(n, heads, bits, group, scale_dtype):
    rows = 29
    x, th, _ = synth.small_case(n, rows, "f16", heads=heads, seed=11)
    y32 = _ref_fwd(x, th, n, heads, "f16").astype(np.float32)
    y32[3, :group] = 0.0                      # an all-zero group
    y32[4, :group] *= np.float32(1e-7)        # a scale in the binary16 subnormal range
    y32[5, group:2 * group] *= np.float32(3e4)  # a scale that saturates binary16
    # theta = 0 and float32 input: the cascade passes the values through exactly
    codes, scales = gu.run_fwd_quant(y32, np.zeros_like(th), n, heads, "f32", bits, group, scale_dtype)
    ref_codes, ref_scales = oracle.quantize(y32, group, bits, scale_dtype)
    assert np.array_equal(scales.view(np.uint32), ref_scales.view(np.uint32))
    assert np.array_equal(codes, oracle.pack_codes(ref_codes, bits))


@pytest.mark.parametrize("bits", [2, 4])
def test_quantiser_every_binary16_scale_bit_exact(bits):
    # The fused kernels compute 1/s with a hardware estimate plus one Newton step and, for INT4, amax/7
    # with a multiply-remainder-correct sequence; both must reproduce correctly rounded division.
    # Sweep every positive finite binary16 scale value: one group per value, amax = qmax * s exactly.
    n, group = 4096, 128
    qmax = 2 ** (bits - 1) - 1
    hbits = np.arange(1, 0x7C00, dtype=np.uint16)  # all positive finite binary16 values
    pad = (-len(hbits)) % 32
    hbits = np.concatenate([hbits, np.full(pad, 0x3C00, np.uint16)])
    s_vals = hbits.view(np.float16).astype(np.float32)
    rng = np.random.default_rng(bits)
    frac = rng.uniform(-1.0, 1.0, size=(len(s_vals), group)).astype(np.float32)
    # plant exact rounding boundaries (k + 1/2) * s and values just around them
    ks = rng.integers(0, qmax + 1, size=(len(s_vals), 8)).astype(np.float32)
    frac[:, 1:9] = (ks + np.float32(0.5)) / np.float32(qmax) * rng.choice([-1.0, 1.0], size=ks.shape).astype(np.float32)
    frac[:, 0] = rng.choice([-1.0, 1.0], size=len(s_vals))
    y = (frac * (np.float32(qmax) * s_vals)[:, None]).astype(np.float32).reshape(-1, n)
    th = np.zeros((1, 12, n // 2), np.float32)
    codes, scales = gu.run_fwd_quant(y, th, n, 1, "f32", bits, group, "f16")
    ref_codes, ref_scales = oracle.quantize(y, group, bits, "f16")
    assert np.array_equal(scales.view(np.uint32), ref_scales.view(np.uint32))
    assert np.array_equal(codes, oracle.pack_codes(ref_codes, bits))


def test_quantiser_int4_scale_division_bit_exact_on_random_mantissas():
    n, group, rows = 4096, 128, 4096
    rng = np.random.default_rng(7)
    mant = rng.integers(0, 2 ** 23, size=rows * 32, dtype=np.uint32)
    mant[:64] = np.uint32(2 ** 23 - 1) - np.arange(64, dtype=np.uint32)  # significands near all-ones
    mant[64:128] = np.arange(64, dtype=np.uint32)                        # and near a power of two
    expo = rng.integers(127 - 30, 127 + 18, size=rows * 32, dtype=np.uint32)
    amax = ((expo << np.uint32(23)) | mant).view(np.float32)
    frac = rng.uniform(-1.0, 1.0, size=(rows * 32, group)).astype(np.float32)
    frac[:, 0] = 1.0
    y = (frac * amax[:, None]).astype(np.float32).reshape(rows, n)
    th = np.zeros((1, 12, n // 2), np.float32)
    for scale_dtype in ("f16", "f32"):
        codes, scales = gu.run_fwd_quant(y, th, n, 1, "f32", 4, group, scale_dtype)
        ref_codes, ref_scales = oracle.quantize(y, group, 4, scale_dtype)
        assert np.array_equal(scales.view(np.uint32), ref_scales.view(np.uint32)), scale_dtype
        assert np.array_equal(codes, oracle.pack_codes(ref_codes, 4)), scale_dtype


# ---- fused forward + quantisation on the five workloads ----------------------------------------

@pytest.mark.parametrize("cfg,rows", [(1, None), (2, 1), (2, 8), (2, 64), (3, 300), (4, 200)])
def test_workload_fused_forward_quant(cfg, rows):
    w = synth.make_workload(cfg, rows=rows)
    y_ref = _ref_fwd(w.x, w.theta, w.n, w.heads, w.dtype)
    codes, scales = gu.run_fwd_quant(w.x, w.theta, w.n, w.heads, w.dtype, w.bits, w.group, w.scale_dtype)
    gu.check_fused_codes(codes, scales, y_ref, w.bits, w.group, w.scale_dtype, w.dtype, w.name)
    if cfg == 3:  # the metric kernel is also run with INT4
        codes, scales = gu.run_fwd_quant(w.x, w.theta, w.n, w.heads, w.dtype, 4, w.group, w.scale_dtype)
        gu.check_fused_codes(codes, scales, y_ref, 4, w.group, w.scale_dtype, w.dtype, w.name + " int4")


@pytest.mark.parametrize("cfg,rows", [(1, None), (3, 300)])
def test_workload_forward_then_inverse(cfg, rows):
    w = synth.make_workload(cfg, rows=rows)
    y = gu.run_transform(w.x, w.theta, w.n, w.heads, w.dtype)
    gu.check_rotated(y, _ref_fwd(w.x, w.theta, w.n, w.heads, w.dtype), w.dtype, w.name)
    xi = gu.run_transform(y, w.theta, w.n, w.heads, w.dtype, inverse=True)
    gu.check_rotated(xi, oracle.inverse(synth.to_f64(y, w.dtype), w.theta, w.n, w.heads), w.dtype, w.name + " inv")


# ---- backward ----------------------------------------------------------------------------------

@pytest.mark.parametrize("n,heads,rows,dtype", [(8, 1, 5, "f32"), (128, 1, 70, "f32"), (128, 4, 33, "bf16"),
                                                 (1024, 1, 40, "f16"), (4096, 1, 12, "bf16"),
                                                 (8192, 1, 9, "bf16"), (16384, 1, 3, "f32")])
def test_backward_shapes(n, heads, rows, dtype):
    x, th, dy = synth.small_case(n, rows, dtype, heads=heads, seed=13, with_dy=True, outliers=0)
    dx, dth = gu.run_bwd(x, dy, th, n, heads, dtype)
    rdx, rdth, ab = oracle.backward(synth.to_f64(x, dtype), synth.to_f64(dy, dtype), th, n, heads)
    gu.check_rotated(dx, rdx, dtype, f"dx n={n}")
    gu.check_dtheta(dth, rdth, ab, what=f"n={n} H={heads} {dtype}")


def test_backward_workload5_sample_and_determinism():
    w = synth.make_workload(5, rows=600)
    dx, dth = gu.run_bwd(w.x, w.dy, w.theta, w.n, w.heads, w.dtype)
    rdx, rdth, ab = oracle.backward(synth.to_f64(w.x, w.dtype), synth.to_f64(w.dy, w.dtype), w.theta, w.n)
    gu.check_rotated(dx, rdx, w.dtype, "c5 dx")
    gu.check_dtheta(dth, rdth, ab, what="c5")
    dx2, dth2 = gu.run_bwd(w.x, w.dy, w.theta, w.n, w.heads, w.dtype)
    assert np.array_equal(dth, dth2) and np.array_equal(dx, dx2)  # no atomics: run-to-run bit equality


@pytest.mark.parametrize("n,rows,dtype", [(8192, 2300, "bf16"), (4096, 4500, "f16"), (4096, 700, "f32")])
def test_backward_several_chunks(n, rows, dtype):
    # many rows per workgroup slice (several chunks of rows are covered at full size in test_gpu_full_size.py)
    x, th, dy = synth.small_case(n, rows, dtype, seed=17, with_dy=True, outliers=0)
    dx, dth = gu.run_bwd(x, dy, th, n, 1, dtype)
    rdx, rdth, ab = oracle.backward(synth.to_f64(x, dtype), synth.to_f64(dy, dtype), th, n)
    gu.check_rotated(dx, rdx, dtype, f"dx n={n}")
    gu.check_dtheta(dth, rdth, ab, what=f"n={n} rows={rows}")


def test_backward_flagged_plan_takes_the_plain_path():
    n = 4096
    th = np.full((1, 12, n // 2), np.float32(math.pi / 2), np.float32)
    th[0, 1::2, ::5] = np.float32(-math.pi / 2)
    x, _, dy = synth.small_case(n, 40, "bf16", seed=19, with_dy=True, outliers=0)
    dx, dth = gu.run_bwd(x, dy, th, n, 1, "bf16")
    rdx, rdth, ab = oracle.backward(synth.to_f64(x, "bf16"), synth.to_f64(dy, "bf16"), th, n)
    gu.check_rotated(dx, rdx, "bf16", "dx flagged")
    gu.check_dtheta(dth, rdth, ab, what="flagged plan")


def test_backward_optional_outputs_and_zero_rows():
    x, th, dy = synth.small_case(256, 10, "f32", seed=2, with_dy=True)
    dx, _ = gu.run_bwd(x, dy, th, 256, 1, "f32", want_dtheta=False)
    gu.check_rotated(dx, oracle.inverse(synth.to_f64(dy, "f32"), th, 256), "f32", "dx only")
    _, dth = gu.run_bwd(x, dy, th, 256, 1, "f32", want_dx=False)
    _, rdth, ab = oracle.backward(synth.to_f64(x, "f32"), synth.to_f64(dy, "f32"), th, 256)
    gu.check_dtheta(dth, rdth, ab)
    _, dth0 = gu.run_bwd(x[:0], dy[:0], th, 256, 1, "f32", want_dx=False)
    assert not dth0.any()  # dtheta is overwritten, also by an empty batch


# n = 256 .. 2048, one head: 4096 / n consecutive rows are processed as one block by the n = 4096 kernels (layers
# above log2 n get weight zero); rows that do not fill a block go through the general kernel.
MID = [(256, 16 * 9 + 5, "f16"), (512, 8 * 7 + 3, "bf16"), (1024, 4 * 11 + 1, "f32"), (2048, 2 * 13 + 1, "f16"),
       (2048, 64, "bf16"), (256, 16, "f32")]


@pytest.mark.parametrize("n,rows,dtype", MID)
def test_mid_sizes_forward_inverse_padded_inplace(n, rows, dtype):
    x, th, _ = synth.small_case(n, rows, dtype, seed=60 + n)
    ref = _ref_fwd(x, th, n, 1, dtype)
    gu.check_rotated(gu.run_transform(x, th, n, 1, dtype), ref, dtype, f"mid fwd n={n}")
    gu.check_rotated(gu.run_transform(x, th, n, 1, dtype, pad=16), ref, dtype, f"mid fwd padded n={n}")
    a = gu.run_transform(x, th, n, 1, dtype)
    b = gu.run_transform(x, th, n, 1, dtype, inplace=True)
    np.testing.assert_array_equal(a.view(np.uint8), b.view(np.uint8))
    xi = gu.run_transform(x, th, n, 1, dtype, inverse=True)
    gu.check_rotated(xi, oracle.inverse(synth.to_f64(x, dtype), th, n, 1), dtype, f"mid inv n={n}")


@pytest.mark.parametrize("n,rows,dtype", MID)
@pytest.mark.parametrize("bits,group,sd", [(4, 128, "f16"), (2, 32, "f32")])
def test_mid_sizes_fused_quant(n, rows, dtype, bits, group, sd):
    x, th, _ = synth.small_case(n, rows, dtype, seed=61 + n)
    y_ref = _ref_fwd(x, th, n, 1, dtype)
    codes, scales = gu.run_fwd_quant(x, th, n, 1, dtype, bits, group, sd)
    gu.check_fused_codes(codes, scales, y_ref, bits, group, sd, dtype, f"mid quant n={n}")
    # the fake-quantised forward repeats these codes and scales exactly, block rows and leftover rows alike
    yq, hist = gu.run_fwd_fakequant(x, th, n, 1, dtype, bits, group, sd)
    c = oracle.unpack_codes(codes, bits)
    want = synth.cast_storage(oracle.dequantize(c, scales.astype(np.float32), group).astype(np.float64), dtype)
    u = np.uint16 if dtype != "f32" else np.uint32
    np.testing.assert_array_equal(yq.view(u), want.view(u))
    np.testing.assert_array_equal(hist, oracle.bin_histogram(c, bits))


@pytest.mark.parametrize("n", [256, 1024, 2048])
def test_mid_sizes_flagged_plan(n):
    k = n.bit_length() - 1
    rng = np.random.default_rng(n)
    th = rng.uniform(-math.pi, math.pi, size=(1, k, n // 2)).astype(np.float32)
    th[0, 0, ::2] = np.float32(math.pi / 2)
    th[0, k - 1, :] = np.float32(-math.pi / 2)
    x, _, _ = synth.small_case(n, 3 * (4096 // n) + 1, "f16", seed=5)
    gu.check_rotated(gu.run_transform(x, th, n, 1, "f16"), _ref_fwd(x, th, n, 1, "f16"), "f16", "mid flagged fwd")
    gu.check_rotated(gu.run_transform(x, th, n, 1, "f16", inverse=True),
                     oracle.inverse(synth.to_f64(x, "f16"), th, n, 1), "f16", "mid flagged inv")


# the backward pass takes the same route: blocks of 4096 / n rows, the last one possibly short
@pytest.mark.parametrize("n,rows,dtype", MID + [(256, 5, "bf16"), (512, 1, "f32"), (1024, 4 * 300 + 2, "f16")])
@pytest.mark.parametrize("pad", [0, 24])
def test_mid_sizes_backward(n, rows, dtype, pad):
    x, th, dy = synth.small_case(n, rows, dtype, seed=70 + n, with_dy=True, outliers=0)
    rdx, rdth, ab = oracle.backward(synth.to_f64(x, dtype), synth.to_f64(dy, dtype), th, n)
    dx, dth = gu.run_bwd(x, dy, th, n, 1, dtype, pad=pad)
    gu.check_rotated(dx, rdx, dtype, f"mid dx n={n} rows={rows}")
    gu.check_dtheta(dth, rdth, ab, what=f"mid n={n} rows={rows} {dtype}")
    _, dth_only = gu.run_bwd(x, dy, th, n, 1, dtype, want_dx=False, pad=pad)
    np.testing.assert_array_equal(dth, dth_only)


@pytest.mark.parametrize("n", [256, 2048])
def test_mid_sizes_backward_flagged_plan(n):
    k = n.bit_length() - 1
    rng = np.random.default_rng(n + 1)
    th = rng.uniform(-math.pi, math.pi, size=(1, k, n // 2)).astype(np.float32)
    th[0, 1, ::3] = np.float32(math.pi / 2)
    th[0, k - 1, :] = np.float32(-math.pi / 2)
    x, _, dy = synth.small_case(n, 2 * (4096 // n) + 1, "f16", seed=6, with_dy=True, outliers=0)
    dx, dth = gu.run_bwd(x, dy, th, n, 1, "f16")
    rdx, rdth, ab = oracle.backward(synth.to_f64(x, "f16"), synth.to_f64(dy, "f16"), th, n)
    gu.check_rotated(dx, rdx, "f16", "mid flagged dx")
    gu.check_dtheta(dth, rdth, ab, what="mid flagged")


# ---- n = 8192: 1024-thread workgroups, both halves of a row side by side, layer 13 across them -----------
WIDE = [(1, 1, "f16"), (1, 23, "bf16"), (1, 1300, "f16"), (2, 9, "f16"), (1, 11, "f32"), (3, 700, "bf16")]


@pytest.mark.parametrize("heads,rows,dtype", WIDE)
def test_n8192_forward_inverse_padded_inplace(heads, rows, dtype):
    n = 8192
    x, th, _ = synth.small_case(n, rows, dtype, heads=heads, seed=80 + rows)
    ref = _ref_fwd(x, th, n, heads, dtype)
    gu.check_rotated(gu.run_transform(x, th, n, heads, dtype), ref, dtype, f"wide fwd H={heads} T={rows}")
    gu.check_rotated(gu.run_transform(x, th, n, heads, dtype, pad=40), ref, dtype, "wide fwd padded")
    a = gu.run_transform(x, th, n, heads, dtype)
    b = gu.run_transform(x, th, n, heads, dtype, inplace=True)
    np.testing.assert_array_equal(a.view(np.uint8), b.view(np.uint8))
    xi = gu.run_transform(x, th, n, heads, dtype, inverse=True)
    gu.check_rotated(xi, oracle.inverse(synth.to_f64(x, dtype), th, n, heads), dtype, f"wide inv H={heads} T={rows}")
    xi2 = gu.run_transform(x, th, n, heads, dtype, inverse=True, inplace=True)
    np.testing.assert_array_equal(xi.view(np.uint8), xi2.view(np.uint8))


@pytest.mark.parametrize("heads,rows,dtype", [(1, 5, "f16"), (1, 900, "bf16"), (2, 33, "f32")])
@pytest.mark.parametrize("bits,group,sd", [(4, 128, "f16"), (2, 128, "f16"), (2, 32, "f32"), (4, 64, "f32")])
def test_n8192_fused_quant_and_fakequant(heads, rows, dtype, bits, group, sd):
    n = 8192
    x, th, _ = synth.small_case(n, rows, dtype, heads=heads, seed=81 + rows)
    y_ref = _ref_fwd(x, th, n, heads, dtype)
    codes, scales = gu.run_fwd_quant(x, th, n, heads, dtype, bits, group, sd)
    gu.check_fused_codes(codes, scales, y_ref, bits, group, sd, dtype, f"wide quant H={heads} T={rows}")
    yq, hist = gu.run_fwd_fakequant(x, th, n, heads, dtype, bits, group, sd)
    c = oracle.unpack_codes(codes, bits)
    want = synth.cast_storage(oracle.dequantize(c, scales.astype(np.float32), group).astype(np.float64), dtype)
    u = np.uint16 if dtype != "f32" else np.uint32
    np.testing.assert_array_equal(yq.view(u), want.view(u))
    np.testing.assert_array_equal(hist, oracle.bin_histogram(c, bits))


def test_n8192_flagged_plan():
    n, k = 8192, 13
    rng = np.random.default_rng(8192)
    th = rng.uniform(-math.pi, math.pi, size=(1, k, n // 2)).astype(np.float32)
    th[0, 0, ::2] = np.float32(math.pi / 2)
    th[0, k - 1, :] = np.float32(-math.pi / 2)
    x, _, _ = synth.small_case(n, 7, "f16", seed=5)
    gu.check_rotated(gu.run_transform(x, th, n, 1, "f16"), _ref_fwd(x, th, n, 1, "f16"), "f16", "wide flagged fwd")
    gu.check_rotated(gu.run_transform(x, th, n, 1, "f16", inverse=True),
                     oracle.inverse(synth.to_f64(x, "f16"), th, n, 1), "f16", "wide flagged inv")
    codes, scales = gu.run_fwd_quant(x, th, n, 1, "f16", 4, 128, "f16")
    gu.check_fused_codes(codes, scales, _ref_fwd(x, th, n, 1, "f16"), 4, 128, "f16", "f16", "wide flagged quant")


# ---- backward for n = 8 .. 128: everything in registers, one slot of partial sums per row position ----------
SMALL_BWD = [(8, 1, 1000, "f32"), (8, 256, 19, "f16"), (16, 4, 301, "bf16"), (32, 64, 77, "f16"), (64, 2, 513, "f32"),
             (64, 32, 40, "bf16"), (128, 1, 1, "f16"), (128, 16, 33, "f32"), (128, 32, 300, "bf16"), (128, 64, 21, "f16")]


@pytest.mark.parametrize("n,heads,rows,dtype", SMALL_BWD)
def test_small_transforms_backward(n, heads, rows, dtype):
    x, th, dy = synth.small_case(n, rows, dtype, heads=heads, seed=90 + n + heads, with_dy=True, outliers=0)
    rdx, rdth, ab = oracle.backward(synth.to_f64(x, dtype), synth.to_f64(dy, dtype), th, n, heads)
    dx, dth = gu.run_bwd(x, dy, th, n, heads, dtype)
    gu.check_rotated(dx, rdx, dtype, f"small dx n={n} H={heads}")
    gu.check_dtheta(dth, rdth, ab, what=f"small n={n} H={heads} T={rows} {dtype}")
    dx_p, dth_p = gu.run_bwd(x, dy, th, n, heads, dtype, pad=16)  # padded rows: same arithmetic, same bits
    np.testing.assert_array_equal(dth, dth_p)
    np.testing.assert_array_equal(dx.view(np.uint8), dx_p.view(np.uint8))
    _, dth_only = gu.run_bwd(x, dy, th, n, heads, dtype, want_dx=False)
    np.testing.assert_array_equal(dth, dth_only)


def test_small_transforms_backward_flagged_plan():
    n, heads, k = 128, 4, 7
    rng = np.random.default_rng(77)
    th = rng.uniform(-math.pi, math.pi, size=(heads, k, n // 2)).astype(np.float32)
    th[2, 3, ::4] = np.float32(math.pi / 2)
    x, _, dy = synth.small_case(n, 45, "f16", heads=heads, seed=8, with_dy=True, outliers=0)
    dx, dth = gu.run_bwd(x, dy, th, n, heads, "f16")
    rdx, rdth, ab = oracle.backward(synth.to_f64(x, "f16"), synth.to_f64(dy, "f16"), th, n, heads)
    gu.check_rotated(dx, rdx, "f16", "small flagged dx")
    gu.check_dtheta(dth, rdth, ab, what="small flagged")


# ---- quantiser groups of more than 128 channels, up to one scale per row (per-token), n = 256 .. 8192 --------
BIG_GROUPS = [(4096, 256, 19, "f16"), (4096, 512, 5, "bf16"), (4096, 1024, 33, "f32"), (4096, 4096, 300, "f16"),
              (8192, 512, 7, "bf16"), (8192, 2048, 3, "f16"), (8192, 8192, 130, "f16"), (512, 256, 8 * 5 + 3, "f16"),
              (512, 512, 8 * 40, "bf16"), (2048, 2048, 2 * 9 + 1, "f32"), (1024, 512, 4 * 7, "f16"),
              # several rows per workgroup (the row buffers are reused)
              (8192, 2048, 1500, "f16"), (4096, 4096, 5100, "f32"), (8192, 8192, 1100, "f32"), (1024, 1024, 4 * 5000, "f16")]


@pytest.mark.parametrize("n,group,rows,dtype", BIG_GROUPS)
@pytest.mark.parametrize("bits,sd", [(4, "f16"), (2, "f32")])
def test_large_quantiser_groups(n, group, rows, dtype, bits, sd):
    x, th, _ = synth.small_case(n, rows, dtype, seed=100 + n + group)
    y_ref = _ref_fwd(x, th, n, 1, dtype)
    codes, scales = gu.run_fwd_quant(x, th, n, 1, dtype, bits, group, sd)
    gu.check_fused_codes(codes, scales, y_ref, bits, group, sd, dtype, f"big group n={n} g={group}")
    yq, hist = gu.run_fwd_fakequant(x, th, n, 1, dtype, bits, group, sd)
    c = oracle.unpack_codes(codes, bits)
    want = synth.cast_storage(oracle.dequantize(c, scales.astype(np.float32), group).astype(np.float64), dtype)
    u = np.uint16 if dtype != "f32" else np.uint32
    np.testing.assert_array_equal(yq.view(u), want.view(u))
    np.testing.assert_array_equal(hist, oracle.bin_histogram(c, bits))


def test_large_quantiser_groups_flagged_plan():
    n, k = 4096, 12
    th = np.random.default_rng(3).uniform(-math.pi, math.pi, size=(1, k, n // 2)).astype(np.float32)
    th[0, 5, ::7] = np.float32(math.pi / 2)
    x, _, _ = synth.small_case(n, 9, "f16", seed=12)
    codes, scales = gu.run_fwd_quant(x, th, n, 1, "f16", 4, n, "f16")
    gu.check_fused_codes(codes, scales, _ref_fwd(x, th, n, 1, "f16"), 4, n, "f16", "f16", "per-token flagged")


# row widths that are a multiple of 512 but not of 2048 elements (e.g. 5120 = 40 x 128): narrower workgroups
@pytest.mark.parametrize("n,heads,rows,dtype", [(128, 40, 37, "f16"), (64, 24, 50, "bf16"), (128, 12, 9, "f32")])
def test_small_transforms_odd_row_widths(n, heads, rows, dtype):
    x, th, dy = synth.small_case(n, rows, dtype, heads=heads, seed=110 + heads, with_dy=True, outliers=0)
    y_ref = _ref_fwd(x, th, n, heads, dtype)
    gu.check_rotated(gu.run_transform(x, th, n, heads, dtype), y_ref, dtype, f"odd width fwd H={heads}")
    gu.check_rotated(gu.run_transform(x, th, n, heads, dtype, inverse=True),
                     oracle.inverse(synth.to_f64(x, dtype), th, n, heads), dtype, f"odd width inv H={heads}")
    codes, scales = gu.run_fwd_quant(x, th, n, heads, dtype, 4, n, "f32")
    gu.check_fused_codes(codes, scales, y_ref, 4, n, "f32", dtype, f"odd width quant H={heads}")
    yq, hist = gu.run_fwd_fakequant(x, th, n, heads, dtype, 4, n, "f32")
    np.testing.assert_array_equal(hist, oracle.bin_histogram(oracle.unpack_codes(codes, 4), 4))
    rdx, rdth, ab = oracle.backward(synth.to_f64(x, dtype), synth.to_f64(dy, dtype), th, n, heads)
    dx, dth = gu.run_bwd(x, dy, th, n, heads, dtype)
    gu.check_rotated(dx, rdx, dtype, f"odd width dx H={heads}")
    gu.check_dtheta(dth, rdth, ab, what=f"odd width H={heads}")


# n = 256 .. 2048 with several heads: 4096 consecutive elements of the [rows][heads * n] array form a block, either
# several whole rows (width <= 4096) or a piece of a wider row; every 2^k-element piece has its own angles
MID_HEADS = [(256, 4, 4 * 9 + 3, "f16"), (256, 16, 21, "bf16"), (512, 8, 13, "f32"), (1024, 2, 2 * 17 + 1, "f16"),
             (1024, 8, 11, "bf16"), (2048, 2, 7, "f16"), (2048, 6, 5, "f32"), (512, 2, 4 * 5, "bf16")]


@pytest.mark.parametrize("n,heads,rows,dtype", MID_HEADS)
def test_mid_sizes_several_heads(n, heads, rows, dtype):
    x, th, _ = synth.small_case(n, rows, dtype, heads=heads, seed=120 + n + heads)
    ref = _ref_fwd(x, th, n, heads, dtype)
    gu.check_rotated(gu.run_transform(x, th, n, heads, dtype), ref, dtype, f"mid heads fwd n={n} H={heads}")
    gu.check_rotated(gu.run_transform(x, th, n, heads, dtype, pad=16), ref, dtype, "mid heads fwd padded")
    a = gu.run_transform(x, th, n, heads, dtype)
    b = gu.run_transform(x, th, n, heads, dtype, inplace=True)
    np.testing.assert_array_equal(a.view(np.uint8), b.view(np.uint8))
    gu.check_rotated(gu.run_transform(x, th, n, heads, dtype, inverse=True),
                     oracle.inverse(synth.to_f64(x, dtype), th, n, heads), dtype, f"mid heads inv n={n} H={heads}")
    for bits, group, sd in ((4, 128, "f16"), (2, n, "f32")):
        codes, scales = gu.run_fwd_quant(x, th, n, heads, dtype, bits, group, sd)
        gu.check_fused_codes(codes, scales, ref, bits, group, sd, dtype, f"mid heads quant n={n} H={heads} g={group}")
        yq, hist = gu.run_fwd_fakequant(x, th, n, heads, dtype, bits, group, sd)
        c = oracle.unpack_codes(codes, bits)
        want = synth.cast_storage(oracle.dequantize(c, scales.astype(np.float32), group).astype(np.float64), dtype)
        u = np.uint16 if dtype != "f32" else np.uint32
        np.testing.assert_array_equal(yq.view(u), want.view(u))
        np.testing.assert_array_equal(hist, oracle.bin_histogram(c, bits))


def test_mid_sizes_several_heads_flagged_plan():
    n, heads, k = 512, 4, 9
    rng = np.random.default_rng(55)
    th = rng.uniform(-math.pi, math.pi, size=(heads, k, n // 2)).astype(np.float32)
    th[1, 2, ::3] = np.float32(math.pi / 2)
    th[3, k - 1, :] = np.float32(-math.pi / 2)
    x, _, _ = synth.small_case(n, 2 * 3 + 1, "f16", heads=heads, seed=9)
    gu.check_rotated(gu.run_transform(x, th, n, heads, "f16"), _ref_fwd(x, th, n, heads, "f16"), "f16", "mid heads flagged fwd")
    gu.check_rotated(gu.run_transform(x, th, n, heads, "f16", inverse=True),
                     oracle.inverse(synth.to_f64(x, "f16"), th, n, heads), "f16", "mid heads flagged inv")


@pytest.mark.parametrize("n,heads,rows,dtype", MID_HEADS)
@pytest.mark.parametrize("pad", [0, 16])
def test_mid_sizes_several_heads_backward(n, heads, rows, dtype, pad):
    # rows of up to 4096 elements run on the fused backward kernels (blocks of whole rows), wider ones on the general one
    x, th, dy = synth.small_case(n, rows, dtype, heads=heads, seed=130 + n + heads, with_dy=True, outliers=0)
    rdx, rdth, ab = oracle.backward(synth.to_f64(x, dtype), synth.to_f64(dy, dtype), th, n, heads)
    dx, dth = gu.run_bwd(x, dy, th, n, heads, dtype, pad=pad)
    gu.check_rotated(dx, rdx, dtype, f"mid heads dx n={n} H={heads}")
    floor = np.median(ab, axis=2, keepdims=True)  # few rows: see tests/test_gpu_sweep.py
    gu.check_dtheta(dth, rdth, np.maximum(ab, floor), what=f"mid heads n={n} H={heads} T={rows} {dtype}")
    _, dth_only = gu.run_bwd(x, dy, th, n, heads, dtype, want_dx=False, pad=pad)
    np.testing.assert_array_equal(dth, dth_only)


# ---- float32 rows over many pipeline steps (several rows per workgroup, every element compared) ----------
@pytest.mark.parametrize("n,heads,rows", [(4096, 1, 5200), (8192, 1, 1500), (1024, 1, 20000 + 3), (2048, 2, 2600)])
def test_float32_rows_many_steps(n, heads, rows):
    dtype = "f32"
    x, th, _ = synth.small_case(n, rows, dtype, heads=heads, seed=300 + n)
    ref = _ref_fwd(x, th, n, heads, dtype)
    gu.check_rotated(gu.run_transform(x, th, n, heads, dtype), ref, dtype, f"f32 fwd n={n} T={rows}")
    gu.check_rotated(gu.run_transform(x, th, n, heads, dtype, pad=12), ref, dtype, f"f32 fwd padded n={n}")
    xi = gu.run_transform(x, th, n, heads, dtype, inverse=True)
    gu.check_rotated(xi, oracle.inverse(synth.to_f64(x, dtype), th, n, heads), dtype, f"f32 inv n={n} T={rows}")
    for bits, group, sd in [(4, 128, "f16"), (2, 64, "f32")]:
        codes, scales = gu.run_fwd_quant(x, th, n, heads, dtype, bits, group, sd)
        gu.check_fused_codes(codes, scales, ref, bits, group, sd, dtype, f"f32 quant n={n} T={rows}")
        yq, hist = gu.run_fwd_fakequant(x, th, n, heads, dtype, bits, group, sd)
        c = oracle.unpack_codes(codes, bits)
        want = synth.cast_storage(oracle.dequantize(c, scales.astype(np.float32), group).astype(np.float64), dtype)
        np.testing.assert_array_equal(yq.view(np.uint32), want.view(np.uint32))
        np.testing.assert_array_equal(hist, oracle.bin_histogram(c, bits))
