"""Pins for the oracle's backward pass: finite differences of the forward, the printed derivative
of the Givens block, and identities that follow from orthogonality.  CPU only."""
import math

import numpy as np
import pytest

import oracle
from oracle.dense import dense_butterfly


def _theta(rng, n, heads=1):
    k = n.bit_length() - 1
    return rng.uniform(-math.pi, math.pi, size=(heads, k, n // 2)).astype(np.float32)


@pytest.mark.parametrize("n,heads", [(2, 1), (8, 1), (16, 2), (64, 1)])
def test_dtheta_and_dx_match_central_differences(n, heads):
    rng = np.random.default_rng(n * 7 + heads)
    rows = 3
    # angles that are exact in float32 after +-eps so that the difference quotient is clean
    eps = 2.0 ** -10
    th = (np.round(_theta(rng, n, heads) * 256) / 256).astype(np.float32)
    x = rng.standard_normal((rows, n * heads))
    dy = rng.standard_normal((rows, n * heads))
    dx, dth, ab = oracle.backward(x, dy, th, n, heads)

    def loss(theta):
        return float((dy * oracle.forward(x, theta, n, heads)).sum())

    flat = th.reshape(-1)
    idx = rng.choice(flat.size, size=min(flat.size, 24), replace=False)
    for q in idx:
        tp, tm = flat.copy(), flat.copy()
        tp[q] += np.float32(eps)
        tm[q] -= np.float32(eps)
        num = (loss(tp.reshape(th.shape)) - loss(tm.reshape(th.shape))) / (2 * eps)
        # central difference error ~ eps^2/6 * |third derivative| <= eps^2/6 * abs-sum bound
        assert abs(num - dth.reshape(-1)[q]) <= 1e-6 * max(1.0, ab.reshape(-1)[q])
    # dx is linear in dy: check against differences in x as well
    j = rng.integers(0, n * heads)
    xp, xm = x.copy(), x.copy()
    xp[1, j] += 1e-3
    xm[1, j] -= 1e-3
    num = (float((dy * oracle.forward(xp, th, n, heads)).sum()) - float((dy * oracle.forward(xm, th, n, heads)).sum())) / 2e-3
    assert abs(num - dx[1, j]) < 1e-9
    assert np.allclose(dx, oracle.inverse(dy, th, n, heads), atol=1e-14)


def test_dtheta_against_dense_matrix_derivative_n4():
    # d/dtheta of the dense product, using the printed dG/dtheta = [[-sin,-cos],[cos,-sin]]
    rng = np.random.default_rng(0)
    n = 4
    th = _theta(rng, n)
    x = rng.standard_normal(n)
    dy = rng.standard_normal(n)
    _, dth, _ = oracle.backward(x[None], dy[None], th, n)
    t64 = th[0].astype(np.float64)

    def layer(i, deriv_j=None):
        h = 1 << (i - 1)
        M = np.zeros((n, n))
        lows = [a for a in range(n) if not a & h]
        for j, a in enumerate(lows):
            b = a + h
            c, s = math.cos(t64[i - 1, j]), math.sin(t64[i - 1, j])
            if deriv_j is None:
                M[a, a], M[a, b], M[b, a], M[b, b] = c, -s, s, c
            elif deriv_j == j:
                M[a, a], M[a, b], M[b, a], M[b, b] = -s, -c, c, -s
        return M

    for j in range(2):
        d1 = dy @ layer(2) @ layer(1, j) @ x
        d2 = dy @ layer(2, j) @ layer(1) @ x
        assert abs(d1 - dth[0, 0, j]) < 1e-14
        assert abs(d2 - dth[0, 1, j]) < 1e-14
    assert np.allclose(dense_butterfly(th[0], n), layer(2) @ layer(1))


def test_dy_equal_to_output_gives_zero_dtheta_and_dx_equal_x():
    # L = 1/2 |B x|^2 = 1/2 |x|^2 does not depend on theta
    rng = np.random.default_rng(4)
    n = 128
    th = _theta(rng, n)
    x = rng.standard_normal((5, n))
    y = oracle.forward(x, th, n)
    dx, dth, ab = oracle.backward(x, y, th, n)
    assert np.allclose(dx, x, atol=1e-13)
    assert np.abs(dth).max() < 1e-12 * ab.max()


def test_dtheta_is_sum_over_rows_and_overwritten():
    rng = np.random.default_rng(6)
    n, heads, rows = 32, 2, 6
    th = _theta(rng, n, heads)
    x = rng.standard_normal((rows, n * heads))
    dy = rng.standard_normal((rows, n * heads))
    _, dth, _ = oracle.backward(x, dy, th, n, heads)
    acc = np.zeros_like(dth)
    for r in range(rows):
        acc += oracle.backward(x[r:r + 1], dy[r:r + 1], th, n, heads)[1]
    assert np.allclose(dth, acc, atol=1e-13)


def test_output_form_of_the_angle_gradient():
    # d y_a / d theta = -y_b and d y_b / d theta = y_a for the layer's own outputs, hence
    # dtheta_{i,j} = g_i[b] * x_i[a] - g_i[a] * x_i[b]; checked on a single layer (n = 2)
    th = np.array([[[0.7]]], np.float32)
    x = np.array([[0.3, -1.1]])
    dy = np.array([[2.0, 0.5]])
    y = oracle.forward(x, th, 2)
    _, dth, _ = oracle.backward(x, dy, th, 2)
    assert abs(dth[0, 0, 0] - (dy[0, 1] * y[0, 0] - dy[0, 0] * y[0, 1])) < 1e-15


def _plain_float32_backward(x, dy, theta, n, heads):
    """dtheta with every operation in float32: (cos, sin) rounded to float32, all layer outputs kept, the printed
    derivative's pair expression summed over the rows, transposed layers on the gradient."""
    k = theta.shape[1]
    dth = np.zeros(theta.shape, np.float32)
    e = np.arange(n)
    for h in range(heads):
        c = np.cos(theta[h].astype(np.float64)).astype(np.float32)
        s = np.sin(theta[h].astype(np.float64)).astype(np.float32)
        xs = [x[:, h * n:(h + 1) * n].astype(np.float32)]
        for i in range(1, k + 1):
            st = 1 << (i - 1)
            a = e[(e & st) == 0]
            b = a | st
            p = ((a >> i) << (i - 1)) | (a & (st - 1))
            cur, nxt = xs[-1], np.empty_like(xs[-1])
            nxt[:, a] = c[i - 1][p] * cur[:, a] - s[i - 1][p] * cur[:, b]
            nxt[:, b] = s[i - 1][p] * cur[:, a] + c[i - 1][p] * cur[:, b]
            xs.append(nxt)
        g = dy[:, h * n:(h + 1) * n].astype(np.float32)
        for i in range(k, 0, -1):
            st = 1 << (i - 1)
            a = e[(e & st) == 0]
            b = a | st
            p = ((a >> i) << (i - 1)) | (a & (st - 1))
            acc = np.zeros(n // 2, np.float32)
            for r in range(x.shape[0]):
                acc += g[r, b] * xs[i][r, a] - g[r, a] * xs[i][r, b]
            dth[h, i - 1][p] = acc
            ng = np.empty_like(g)
            ng[:, a] = c[i - 1][p] * g[:, a] + s[i - 1][p] * g[:, b]
            ng[:, b] = -s[i - 1][p] * g[:, a] + c[i - 1][p] * g[:, b]
            g = ng
    return dth


def test_a_plain_float32_backward_misses_the_per_angle_bound_on_a_single_row():
    # Why the seeded GPU sweep floors the per-angle bound at the layer's median for batches of fewer than 32 rows:
    # with one row there is no averaging, an angle whose own two products nearly cancel still carries the float32
    # rounding of the ordinary-sized elements of its layer, and ANY float32 implementation then exceeds
    # 1e-5 x (sum of the absolute products of that angle) on some angle, while it stays far inside the floored
    # bound and inside the norm-wise bound.  (One of the sweep's own cases: n = 512, two heads, one bfloat16 row.)
    from paper_2509_09679_amd import synth

    n, heads, rows, dtype, seed = 512, 2, 1, "bf16", 2248
    x, th, dy = synth.small_case(n, rows, dtype, heads=heads, seed=seed, with_dy=True, outliers=0)
    x64, g64 = synth.to_f64(x, dtype), synth.to_f64(dy, dtype)
    _, ref, ab = oracle.backward(x64, g64, th, n, heads)
    d = np.abs(_plain_float32_backward(x64, g64, th, n, heads).astype(np.float64) - ref)
    assert (d / np.maximum(1e-5 * ab, 1e-300)).max() > 1.0          # the unfloored per-angle bound is missed
    floor = np.median(ab, axis=2, keepdims=True)
    assert (d / (1e-5 * np.maximum(ab, floor))).max() < 0.5         # the floored one is met with room
    assert np.linalg.norm(d) < 0.5 * 1e-5 * np.linalg.norm(ab)      # and so is the norm-wise one
