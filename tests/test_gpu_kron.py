"""GPU parity of the composite transform Q1 (x) B(theta) (bq_cayley_build, bq_kron_fwd, bq_kron_inv) against
the double-precision oracle in oracle/kron.py."""
import math

import numpy as np
import pytest

import oracle
from oracle import kron
from paper_2509_09679_amd import synth

pytestmark = pytest.mark.gpu

import gpu_util as gu  # noqa: E402

DEV = "cuda:0"


@pytest.mark.parametrize("d1", [2, 3, 5, 12, 40, 64])
def test_cayley_build(d1):
    import torch
    from paper_2509_09679_amd import binding as B

    rng = np.random.default_rng(d1)
    p = (rng.standard_normal(d1 * (d1 - 1) // 2) * (2.0 if d1 < 8 else 0.3)).astype(np.float32)
    q = torch.empty((d1, d1), dtype=torch.float32, device=DEV)
    B.bq_cayley_build(torch.from_numpy(p).to(DEV), d1, q)
    torch.cuda.synchronize()
    ref = kron.cayley(p, d1)
    got = q.cpu().numpy().astype(np.float64)
    assert np.abs(got - ref).max() <= 2e-7
    assert np.abs(got.T @ got - np.eye(d1)).max() <= 1e-6


def _run(x_store, q1, theta, d1, d2, dtype, inverse=False, inplace=False):
    import torch
    from paper_2509_09679_amd import binding as B

    th = torch.from_numpy(np.ascontiguousarray(theta)).to(DEV)
    plan = B.alloc_plan(th, d2, 1)
    x = synth.storage_to_torch(x_store, dtype, DEV)
    y = x if inplace else torch.full_like(x, 7.0)
    qd = torch.from_numpy(np.ascontiguousarray(q1, dtype=np.float32)).to(DEV)
    (B.bq_kron_inv if inverse else B.bq_kron_fwd)(x, y, qd, d1, plan, B.make_kron_rows(x, d2))
    torch.cuda.synchronize()
    return synth.torch_to_storage(y, dtype)


def _half_ulp(ref64, dtype):
    """Half a unit in the last place of the row type at the correctly rounded value."""
    _, e = np.frexp(gu.round_to_storage(ref64, dtype))  # |v| = m * 2^e, m in [0.5, 1)
    return np.ldexp(1.0, e - 1 - (11 if dtype == "f16" else 8))


def _check(got_store, ref64, dtype, what, fused=True, shape=None):
    """float32 rows: the stated row-norm bound.  16-bit rows of the fused kernel: every element is a correct
    rounding of a value within the arithmetic's error of the exact one, |got - ref| <= half a unit in the last
    place + slack, where slack is 1e-5 of max(|ref|, row rms) for float32 arithmetic and, for binary16 rows (which
    mix on the bfloat16 matrix instruction, shape = (d1, d2)), also 3 * 2^-16 of the norm of the element's column
    over the sub-rows.  (A distance from the correctly rounded row would not do: one dominant element that
    rounds the other way moves a short row by more than the whole tolerance.)
    Widths other than d2 = 128 take two passes and the butterfly factor's result goes through memory in the
    row type: there the row-norm distance from the rounded oracle row is bounded, by the stated tolerance
    (for bfloat16, whose second rounding alone moves a row by about 3e-3 of its norm, by 6e-3).  Element bound
    everywhere: five times the tolerance, relative to max(|ref|, rms of the row)."""
    got = synth.to_f64(got_store, dtype)
    rn = np.linalg.norm(ref64, axis=1)
    rms = np.sqrt((ref64 ** 2).mean(axis=1, keepdims=True))
    if dtype == "f32" or not fused:
        tol = gu.TOL[dtype] if (fused or dtype != "bf16") else 6e-3
        target = ref64 if dtype == "f32" else gu.round_to_storage(ref64, dtype)
        dn = np.linalg.norm(got - target, axis=1)
        assert np.all(dn <= tol * rn + 1e-30), f"{what}: row error {np.max(dn / np.maximum(rn, 1e-300)):.3e}"
    else:
        slack = 1e-5 * np.maximum(np.abs(ref64), rms)
        if dtype == "f16":
            rows, (d1, d2) = ref64.shape[0], shape
            col = np.sqrt((ref64.reshape(rows, d1, d2) ** 2).sum(axis=1, keepdims=True))
            slack = slack + (3 * 2.0 ** -16 * np.broadcast_to(col, (rows, d1, d2))).reshape(rows, d1 * d2)
        excess = np.abs(got - ref64) - _half_ulp(ref64, dtype)
        assert np.all(excess <= slack), f"{what}: {np.max(excess / slack):.3f} of the allowed excess over half a unit"
    assert np.all(np.abs(got - ref64) <= 5 * gu.ELEM_TOL[dtype] * np.maximum(np.abs(ref64), rms) + 1e-30), what


CASES = [
    # d1, d2, rows, dtype
    (40, 128, 37, "f16"),
    (40, 128, 5, "f32"),
    (40, 128, 300, "bf16"),
    (3, 8, 10, "f32"),
    (5, 16, 11, "bf16"),
    (12, 64, 9, "f16"),
    (64, 32, 6, "f16"),
    (7, 4096, 3, "f16"),
    (24, 256, 17, "f32"),
    (64, 128, 9, "bf16"),
    (37, 128, 21, "f16"),
    (2, 128, 1, "f32"),
    (8, 128, 3000, "f16"),   # d1 <= 8: two workgroups per compute unit, several rows each
    (4, 128, 5000, "bf16"),
    (40, 128, 1400, "f32"),  # several rows per workgroup on the float32 matrix path
]


@pytest.mark.parametrize("d1,d2,rows,dtype", CASES)
def test_kron_forward_and_inverse(d1, d2, rows, dtype):
    rng = np.random.default_rng(1000 * d1 + d2)
    k = int(math.log2(d2))
    theta = rng.uniform(-math.pi, math.pi, size=(1, k, d2 // 2)).astype(np.float32)
    p = (0.4 * rng.standard_normal(d1 * (d1 - 1) // 2)).astype(np.float32)
    q1 = kron.cayley(p, d1).astype(np.float32)  # the float32 matrix both sides use
    x, _, _ = synth.small_case(d2, rows * d1, dtype, seed=d1)
    x = x.reshape(rows, d1 * d2)
    x64 = synth.to_f64(x, dtype)
    q64 = q1.astype(np.float64)
    fused = d2 == 128 and d1 <= 40  # else two passes
    _check(_run(x, q1, theta, d1, d2, dtype), kron.kron_forward(x64, q64, theta, d2), dtype, "kron fwd", fused, (d1, d2))
    _check(_run(x, q1, theta, d1, d2, dtype, inverse=True), kron.kron_inverse(x64, q64, theta, d2), dtype, "kron inv", fused,
           (d1, d2))
    # in place gives the same bits as out of place
    a = _run(x, q1, theta, d1, d2, dtype)
    b = _run(x, q1, theta, d1, d2, dtype, inplace=True)
    np.testing.assert_array_equal(a.view(np.uint8), b.view(np.uint8))


def test_kron_5120_with_device_built_cayley_roundtrip():
    import torch
    from paper_2509_09679_amd import binding as B

    d1, d2, rows, dtype = 40, 128, 2048, "f16"
    rng = np.random.default_rng(7)
    theta = rng.uniform(-math.pi, math.pi, size=(1, 7, 64)).astype(np.float32)
    p = (0.3 * rng.standard_normal(780)).astype(np.float32)
    x, _, _ = synth.small_case(d2, rows * d1, dtype, seed=3)
    xd = synth.storage_to_torch(x.reshape(rows, d1 * d2), dtype, DEV)
    q = torch.empty((d1, d1), dtype=torch.float32, device=DEV)
    B.bq_cayley_build(torch.from_numpy(p).to(DEV), d1, q)
    plan = B.alloc_plan(torch.from_numpy(theta).to(DEV), d2, 1)
    r = B.make_kron_rows(xd, d2)
    y = torch.empty_like(xd)
    back = torch.empty_like(xd)
    B.bq_kron_fwd(xd, y, q, d1, plan, r)
    B.bq_kron_inv(y, back, q, d1, plan, r)
    torch.cuda.synchronize()
    nx, ny = xd.float().norm(dim=1), y.float().norm(dim=1)
    assert float(((nx - ny).abs() / nx).max()) < 2e-3                       # orthogonal: norms preserved
    assert float(((back.float() - xd.float()).norm(dim=1) / nx).max()) < 2e-3  # inverse o forward = identity
    ref = kron.kron_forward(synth.to_f64(x.reshape(rows, d1 * d2)[:64], dtype), kron.cayley(p, d1), theta, d2)
    _check(synth.torch_to_storage(y[:64], dtype), ref, dtype, "5120 forward", True, (d1, d2))


@pytest.mark.parametrize("d1,d2,dtype", [(40, 128, "f16"), (6, 64, "f32")])
def test_kron_with_a_plan_flagged_singular(d1, d2, dtype):
    # cos(theta) = 0 somewhere: the scale-deferred tables are unusable, the kernels fall back to plain rotations
    rng = np.random.default_rng(11)
    k = int(math.log2(d2))
    theta = rng.uniform(-math.pi, math.pi, size=(1, k, d2 // 2)).astype(np.float32)
    theta[0, 1, :] = np.float32(math.pi / 2)
    theta[0, k - 1, ::3] = np.float32(-math.pi / 2)
    q1 = kron.cayley((0.4 * rng.standard_normal(d1 * (d1 - 1) // 2)).astype(np.float32), d1).astype(np.float32)
    x, _, _ = synth.small_case(d2, 13 * d1, dtype, seed=5)
    x = x.reshape(13, d1 * d2)
    x64 = synth.to_f64(x, dtype)
    _check(_run(x, q1, theta, d1, d2, dtype), kron.kron_forward(x64, q1.astype(np.float64), theta, d2), dtype, "flagged fwd", True, (d1, d2))
    _check(_run(x, q1, theta, d1, d2, dtype, inverse=True), kron.kron_inverse(x64, q1.astype(np.float64), theta, d2), dtype,
           "flagged inv", True, (d1, d2))


def _sweep_cases():
    rng = np.random.default_rng(5120)
    out = []
    for i in range(40):
        d1 = int(rng.integers(2, 65))
        d2 = int(rng.choice([8, 16, 32, 64, 128, 128, 128, 256, 512, 1024]))
        rows = int(rng.integers(1, max(2, min(40, 60000 // (d1 * d2)) + 1)))
        out.append((i, d1, d2, rows, str(rng.choice(["f32", "f16", "bf16"]))))
    return out


@pytest.mark.parametrize("i,d1,d2,rows,dtype", _sweep_cases())
def test_kron_sweep(i, d1, d2, rows, dtype):
    # seeded sweep over both code paths (fused for d2 = 128 and d1 <= 40, two passes otherwise) and their borders
    rng = np.random.default_rng(7000 + i)
    k = int(math.log2(d2))
    theta = rng.uniform(-math.pi, math.pi, size=(1, k, d2 // 2)).astype(np.float32)
    q1 = kron.cayley((0.4 * rng.standard_normal(d1 * (d1 - 1) // 2)).astype(np.float32), d1).astype(np.float32)
    x = synth.small_case(d2, rows * d1, dtype, seed=200 + i)[0].reshape(rows, d1 * d2)
    x64, q64 = synth.to_f64(x, dtype), q1.astype(np.float64)
    fused = d2 == 128 and d1 <= 40
    _check(_run(x, q1, theta, d1, d2, dtype), kron.kron_forward(x64, q64, theta, d2), dtype, f"kron sweep {i} fwd", fused, (d1, d2))
    _check(_run(x, q1, theta, d1, d2, dtype, inverse=True), kron.kron_inverse(x64, q64, theta, d2), dtype,
           f"kron sweep {i} inv", fused, (d1, d2))


@pytest.mark.parametrize("d1", [40, 24, 9])
def test_kron_binary16_rows_mixing_error_is_far_below_the_output_rounding(d1):
    # binary16 rows mix on the bfloat16 matrix instruction with two-way splits of both factors: every product
    # Q[i][k] z[k][j] carries a relative error below 3 * 2^-16, so an output is off by at most
    # 3 * 2^-16 * sum_k |Q[i][k]| |z[k][j]| <= 3 * 2^-16 * ||z[:, j]||_2 = 3 * 2^-16 * ||y[:, j]||_2 (rows of Q1 have
    # norm one, and Q1 preserves the norm of a column): that bound is what _check allows beyond half a unit in
    # the last place.  Here also: the typical error is far smaller.  Inputs have outlier channels (x100), whose
    # products dominate a row; several rows per workgroup.
    d2, rows, dtype = 128, 700, "f16"
    rng = np.random.default_rng(55 + d1)
    theta = rng.uniform(-math.pi, math.pi, size=(1, 7, 64)).astype(np.float32)
    q1 = kron.cayley((0.4 * rng.standard_normal(d1 * (d1 - 1) // 2)).astype(np.float32), d1).astype(np.float32)
    x, _, _ = synth.small_case(d2, rows * d1, dtype, seed=9 + d1)
    x = x.reshape(rows, d1 * d2)
    x64 = synth.to_f64(x, dtype)
    for inverse in (False, True):
        ref = (kron.kron_inverse if inverse else kron.kron_forward)(x64, q1.astype(np.float64), theta, d2)
        out = _run(x, q1, theta, d1, d2, dtype, inverse=inverse)
        _check(out, ref, dtype, f"d1={d1} inv={inverse}", True, (d1, d2))
        col = np.sqrt((ref.reshape(rows, d1, d2) ** 2).sum(axis=1, keepdims=True))
        bound = (3 * 2.0 ** -16 * np.broadcast_to(col, (rows, d1, d2))).reshape(rows, d1 * d2)
        rms = np.sqrt((ref ** 2).mean(axis=1, keepdims=True))
        excess = np.abs(synth.to_f64(out, dtype) - ref) - _half_ulp(ref, dtype)
        assert np.mean(excess > bound / 3 + 1e-5 * rms) < 1e-3  # all but a few elements in 10^4 within a third
