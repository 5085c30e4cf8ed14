"""GPU parity of bq_butterfly_fwd_fakequant (Dequant(Quant(Bx)) and the code-bin histogram).

Two legs: (1) with theta = 0 the cascade passes float values through exactly, so outputs and counters
must equal the oracle's bit for bit; (2) with the GPU's own rotation, the call must reproduce exactly
what bq_butterfly_fwd_quant's codes and scales imply (those are checked against the oracle in
test_gpu_parity.py), and stay within half a quantisation step of the oracle's rotated values."""
import numpy as np
import pytest

import oracle
from paper_2509_09679_amd import synth

pytestmark = pytest.mark.gpu

import gpu_util as gu  # noqa: E402

CASES = [
    # n, heads, rows, dtype, bits, group, scale dtype
    (128, 1, 37, "f32", 4, 128, "f32"),
    (128, 32, 19, "bf16", 4, 128, "f32"),
    (64, 3, 50, "f16", 2, 16, "f16"),
    (4096, 1, 21, "f16", 2, 128, "f16"),
    (4096, 1, 9, "f16", 4, 128, "f16"),
    (4096, 1, 5, "f32", 4, 64, "f32"),
    (4096, 1, 7, "bf16", 2, 32, "f16"),
    (4096, 1, 6, "f16", 4, 4096, "f32"),
    (8192, 1, 3, "bf16", 4, 128, "f16"),
    (1024, 2, 11, "f16", 2, 256, "f32"),
]


def _case(n, heads, rows, dtype, seed):
    x, theta, _ = synth.small_case(n, rows, dtype, heads=heads, seed=seed)
    return x, theta


@pytest.mark.parametrize("n,heads,rows,dtype,bits,group,sd", CASES)
def test_fakequant_bit_exact_with_identity_rotation(n, heads, rows, dtype, bits, group, sd):
    x, theta = _case(n, heads, rows, dtype, 31)
    theta0 = np.zeros_like(theta)
    yq, hist = gu.run_fwd_fakequant(x, theta0, n, heads, dtype, bits, group, sd)
    y32 = synth.to_f64(x, dtype).astype(np.float32)  # exact: the row type is no wider than float32
    codes, scales = oracle.quantize(y32.reshape(rows * heads, n), group, bits, sd)
    ref = oracle.dequantize(codes, scales, group).reshape(rows, heads * n)
    want = synth.cast_storage(ref.astype(np.float64), dtype)
    np.testing.assert_array_equal(yq.view(np.uint16 if dtype != "f32" else np.uint32),
                                  want.view(np.uint16 if dtype != "f32" else np.uint32))
    np.testing.assert_array_equal(hist, oracle.bin_histogram(codes, bits))


@pytest.mark.parametrize("n,heads,rows,dtype,bits,group,sd", CASES)
def test_fakequant_matches_fwd_quant_and_oracle_rotation(n, heads, rows, dtype, bits, group, sd):
    x, theta = _case(n, heads, rows, dtype, 32)
    yq, hist = gu.run_fwd_fakequant(x, theta, n, heads, dtype, bits, group, sd)
    packed, scales = gu.run_fwd_quant(x, theta, n, heads, dtype, bits, group, sd)
    codes = oracle.unpack_codes(packed, bits).reshape(rows * heads, n)
    scales = scales.reshape(rows * heads, n // group).astype(np.float32)
    # the same quantiser as bq_butterfly_fwd_quant, to the bit
    want = synth.cast_storage(oracle.dequantize(codes, scales, group).astype(np.float64).reshape(rows, heads * n), dtype)
    u = np.uint16 if dtype != "f32" else np.uint32
    np.testing.assert_array_equal(yq.view(u), want.view(u))
    np.testing.assert_array_equal(hist, oracle.bin_histogram(codes, bits))
    assert hist.sum() == rows * heads * n
    # against the oracle's rotation: within half a step (plus the rotation and output tolerances) unless clipped
    y_ref = oracle.forward(synth.to_f64(x, dtype), theta, n, heads).reshape(rows * heads, n)
    s = np.repeat(scales.astype(np.float64), group, axis=1)
    qmax = (1 << (bits - 1)) - 1
    inside = np.abs(y_ref) <= s * (qmax + 0.5)
    err = np.abs(synth.to_f64(yq, dtype).reshape(rows * heads, n) - y_ref)
    rms = np.sqrt((y_ref ** 2).mean(axis=1, keepdims=True))
    # rotation tolerance, plus the rounding of s * q (up to |y| + s / 2 in size) to a 16-bit row type
    slack = 2e-5 * np.maximum(np.abs(y_ref), rms) + gu.ELEM_TOL[dtype] * (np.abs(y_ref) + s) * (dtype != "f32") + 1e-30
    assert np.all(err[inside] <= 0.5 * s[inside] + slack[inside])


def test_fakequant_optional_outputs_and_empty_batch():
    import torch
    from paper_2509_09679_amd import binding as B

    n, heads, rows, dtype = 256, 2, 12, "f16"
    x, theta = _case(n, heads, rows, dtype, 33)
    yq_only, _ = gu.run_fwd_fakequant(x, theta, n, heads, dtype, 4, 64, "f16", want_hist=False)
    _, hist_only = gu.run_fwd_fakequant(x, theta, n, heads, dtype, 4, 64, "f16", want_y=False)
    yq, hist = gu.run_fwd_fakequant(x, theta, n, heads, dtype, 4, 64, "f16")
    np.testing.assert_array_equal(yq_only.view(np.uint16), yq.view(np.uint16))
    np.testing.assert_array_equal(hist_only, hist)
    # empty batch: the counters are still an output (cleared); neither output given: an error
    th = torch.from_numpy(theta).to("cuda:0")
    plan = B.alloc_plan(th, n, heads)
    xe = torch.empty((0, heads * n), dtype=torch.float16, device="cuda:0")
    h = torch.full((16,), 5, dtype=torch.int64, device="cuda:0")
    B.bq_butterfly_fwd_fakequant(xe, plan, None, h, B.make_quant(4, 64, "f16"), B.make_rows(xe, n, heads))
    torch.cuda.synchronize()
    assert int(h.abs().sum()) == 0
    with pytest.raises(B.BqError):
        B.bq_butterfly_fwd_fakequant(xe, plan, None, None, B.make_quant(4, 64, "f16"), B.make_rows(xe, n, heads))


@pytest.mark.parametrize("n,heads,group", [(4096, 1, 128), (128, 4, 128), (1024, 1, 64)])
@pytest.mark.parametrize("bits", [2, 4])
def test_fakequant_clipping_scales_bit_exact(n, heads, group, bits):
    # binary16 scales that underflow, are subnormal, or saturate at 65504: the clip acts, the lowest code
    # (-2 / -8) appears.  theta = 0 and float32 rows: outputs and counters must equal the oracle's exactly.
    rng = np.random.default_rng(77 + n + bits)
    rows = 24
    x = rng.standard_normal((rows, heads * n)).astype(np.float32)
    mag = np.array([1e-9, 3e-8, 2e-7, 6e-6, 5e-5, 1.0, 3e4, 7e4, 5e5, 4e6, 1e9, 0.0], dtype=np.float32)
    x *= np.repeat(mag, 2)[:, None]
    x[3, : heads * n : 2] *= -1.0
    theta0 = np.zeros((heads, int(np.log2(n)), n // 2), dtype=np.float32)
    yq, hist = gu.run_fwd_fakequant(x, theta0, n, heads, "f32", bits, group, "f16")
    codes, scales = oracle.quantize(x.reshape(rows * heads, n), group, bits, "f16")
    ref = oracle.dequantize(codes, scales, group).reshape(rows, heads * n)
    np.testing.assert_array_equal(yq.view(np.uint32), ref.view(np.uint32))
    want = oracle.bin_histogram(codes, bits)
    np.testing.assert_array_equal(hist, want)
    assert want[0] > 0, "the case is meant to reach the lowest code"


@pytest.mark.parametrize("n,heads,rows,dtype,bits,group,sd", [
    (4096, 1, 40000, "f16", 4, 128, "f16"),   # 39-40 rows per workgroup: the 8-bit counters drain inside the loop
    (4096, 1, 40000, "f16", 2, 128, "f16"),
    (128, 32, 70000, "bf16", 4, 128, "f32"),  # 34 row groups per workgroup of the small-transform kernel
])
def test_fakequant_many_rows_per_workgroup(n, heads, rows, dtype, bits, group, sd):
    import torch
    from paper_2509_09679_amd import binding as B

    cfg = 3 if n == 4096 else 4
    x, th, _ = synth.device_rows(cfg, rows, "cuda:0")
    theta = torch.from_numpy(th).to("cuda:0")
    plan = B.alloc_plan(theta, n, heads)
    r = B.make_rows(x, n, heads)
    q = B.make_quant(bits, group, sd)
    yq = torch.empty_like(x)
    hist = torch.zeros(1 << bits, dtype=torch.int64, device="cuda:0")
    B.bq_butterfly_fwd_fakequant(x, plan, yq, hist, q, r)
    codes, scales = B.alloc_quant_outputs(rows, n, heads, bits, group, sd, "cuda:0")
    B.bq_butterfly_fwd_quant(x, plan, codes, scales, q, r)
    torch.cuda.synchronize()
    c = oracle.unpack_codes(codes.cpu().numpy(), bits)
    want_hist = oracle.bin_histogram(c, bits)
    np.testing.assert_array_equal(hist.cpu().numpy().astype(np.uint64), want_hist)
    pick = np.unique(np.concatenate([[0, rows - 1], np.random.default_rng(3).integers(0, rows, 64)]))
    sc = scales.float().cpu().numpy()[pick].reshape(len(pick) * heads, n // group)
    ref = oracle.dequantize(c[pick].reshape(len(pick) * heads, n), sc, group).reshape(len(pick), heads * n)
    got = synth.torch_to_storage(yq[torch.as_tensor(pick, device="cuda:0")], dtype)
    np.testing.assert_array_equal(got.view(np.uint16), synth.cast_storage(ref.astype(np.float64), dtype).view(np.uint16))
    # and the counters agree with the oracle's own rotation up to the rare boundary codes
    y_ref = oracle.forward(synth.to_f64(synth.torch_to_storage(x[:2048], dtype), dtype), th, n, heads)
    oc, _ = oracle.quantize(y_ref.reshape(-1, n).astype(np.float32), group, bits, sd)
    oh = oracle.bin_histogram(oc, bits).astype(np.int64)
    gh = oracle.bin_histogram(c[:2048], bits).astype(np.int64)
    assert np.abs(oh - gh).sum() <= 1e-3 * oh.sum()


@pytest.mark.parametrize("n,heads,rows", [(4096, 1, 1024), (128, 32, 1024), (8192, 1, 512), (1024, 1, 4096)])
def test_fakequant_float32_scales_binary16_rows_is_product_then_rounding(n, heads, rows):
    # With float32 scales the product s * q needs up to 27 bits: it is rounded to float32 first and then to
    # binary16.  Rounding the exact product once would differ where the float32 product is a binary16 tie
    # (a few elements per 10^5), so this compares every element of several million.
    import torch
    from paper_2509_09679_amd import binding as B

    x, th, _ = synth.small_case(n, rows, "f16", heads=heads, seed=5 + n)
    theta = torch.from_numpy(th).to("cuda:0")
    plan = B.alloc_plan(theta, n, heads)
    xd = synth.storage_to_torch(x, "f16", "cuda:0")
    r = B.make_rows(xd, n, heads)
    q = B.make_quant(4, min(n, 128), "f32")
    yq = torch.empty_like(xd)
    B.bq_butterfly_fwd_fakequant(xd, plan, yq, None, q, r)
    codes, scales = B.alloc_quant_outputs(rows, n, heads, 4, min(n, 128), "f32", "cuda:0")
    B.bq_butterfly_fwd_quant(xd, plan, codes, scales, q, r)
    torch.cuda.synchronize()
    c = oracle.unpack_codes(codes.cpu().numpy(), 4)
    deq = oracle.dequantize(c, scales.cpu().numpy(), min(n, 128))
    want = synth.cast_storage(deq.astype(np.float64), "f16")
    got = synth.torch_to_storage(yq, "f16")
    np.testing.assert_array_equal(got.view(np.uint16), want.view(np.uint16))
    # the case must contain such ties, or it would not tell the two roundings apart
    exact = scales.cpu().numpy().astype(np.float64).repeat(min(n, 128), axis=1) * c.astype(np.float64)
    once = synth.cast_storage(exact, "f16")
    assert (once.view(np.uint16) != want.view(np.uint16)).sum() > 0


@pytest.mark.parametrize("n,rows,group", [(4096, 9000, 128), (1024, 30000, 64), (4096, 7001, 4096)])
def test_fakequant_every_row_over_many_pipeline_steps(n, rows, group):
    # Several rows per workgroup, so that the kernels' row buffers and input slots are reused many times;
    # every element of every row is compared, for both outputs together and for each one alone.
    import torch
    from paper_2509_09679_amd import binding as B

    x, th, _ = synth.small_case(n, rows, "f16", heads=1, seed=77 + n + group)
    theta = torch.from_numpy(th).to("cuda:0")
    plan = B.alloc_plan(theta, n, 1)
    xd = synth.storage_to_torch(x, "f16", "cuda:0")
    r = B.make_rows(xd, n, 1)
    for bits in (4, 2):
        q = B.make_quant(bits, group, "f16")
        codes, scales = B.alloc_quant_outputs(rows, n, 1, bits, group, "f16", "cuda:0")
        B.bq_butterfly_fwd_quant(xd, plan, codes, scales, q, r)
        yq_both, yq_only = torch.empty_like(xd), torch.empty_like(xd)
        h_both = torch.zeros(1 << bits, dtype=torch.int64, device="cuda:0")
        h_only = torch.zeros_like(h_both)
        B.bq_butterfly_fwd_fakequant(xd, plan, yq_both, h_both, q, r)
        B.bq_butterfly_fwd_fakequant(xd, plan, yq_only, None, q, r)
        B.bq_butterfly_fwd_fakequant(xd, plan, None, h_only, q, r)
        torch.cuda.synchronize()
        c = oracle.unpack_codes(codes.cpu().numpy(), bits)
        want_hist = oracle.bin_histogram(c, bits)
        np.testing.assert_array_equal(h_both.cpu().numpy().astype(np.uint64), want_hist)
        np.testing.assert_array_equal(h_only.cpu().numpy().astype(np.uint64), want_hist)
        deq = oracle.dequantize(c, scales.float().cpu().numpy(), group)
        want = synth.cast_storage(deq.astype(np.float64), "f16").view(np.uint16)
        np.testing.assert_array_equal(synth.torch_to_storage(yq_both, "f16").view(np.uint16), want)
        np.testing.assert_array_equal(synth.torch_to_storage(yq_only, "f16").view(np.uint16), want)
