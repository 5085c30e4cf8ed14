"""The calibration step assembled from library calls (paper_2509_09679_amd/calibration.py) against the same
step written with the oracle and numpy in double; then a short SGD run from identity on synthetic
heavy-tailed activations, whose reconstruction loss must fall."""
import numpy as np
import pytest

import oracle
from paper_2509_09679_amd import synth

gpu = pytest.mark.gpu


def _through_quantiser(v, vq, g, bits, group):
    """The gradient rule of calibration.py's module text, written out with loops over groups (numpy, double)."""
    rows, n = v.shape
    qmax = (1 << (bits - 1)) - 1
    dv = g.copy()
    for r in range(rows):
        for c0 in range(0, n, group):
            seg = slice(c0, c0 + group)
            m = c0 + int(np.argmax(np.abs(v[r, seg])))
            s = abs(v[r, m]) / qmax
            if s > 0:
                dv[r, m] += np.sign(v[r, m]) / qmax * float(np.dot(g[r, seg], (vq[r, seg] - v[r, seg]) / s))
    return dv


def _oracle_step(X, W, theta, n, act, wgt, Xq_given=None, Wq_given=None):
    """L_recon, dtheta and the code-bin histogram with the oracle: float64 throughout, except the quantiser, which
    is float32 by definition.  Xq_given / Wq_given replace the oracle's own fake-quantised values (see the test)."""
    Xr = oracle.forward(X, theta, n)
    Wr = oracle.forward(W, theta, n)
    qx, sx = oracle.quantize(Xr.astype(np.float32), act[1], act[0], act[2])
    qw, sw = oracle.quantize(Wr.astype(np.float32), wgt[1], wgt[0], wgt[2])
    Xq = oracle.dequantize(qx, sx, act[1]).astype(np.float64) if Xq_given is None else Xq_given
    Wq = oracle.dequantize(qw, sw, wgt[1]).astype(np.float64) if Wq_given is None else Wq_given
    E = Xq @ Wq.T - X @ W.T
    loss = float((E * E).sum())
    _, dth_x, _ = oracle.backward(X, _through_quantiser(Xr, Xq, 2.0 * E @ Wq, act[0], act[1]), theta, n)
    _, dth_w, _ = oracle.backward(W, _through_quantiser(Wr, Wq, 2.0 * E.T @ Xq, wgt[0], wgt[1]), theta, n)
    return loss, dth_x + dth_w, oracle.bin_histogram(qx, act[0])


def test_gradient_rule_equals_autograd_of_a_straight_through_quantiser():
    # CPU check of the rule itself against torch autograd on  s * (v/s + (round(v/s) - v/s).detach())
    import torch

    torch.manual_seed(0)
    rows, n, group, bits = 5, 64, 16, 4
    qmax = (1 << (bits - 1)) - 1
    v = torch.randn(rows, n, dtype=torch.float64, requires_grad=True)
    g = torch.randn(rows, n, dtype=torch.float64)
    vg = v.reshape(rows, n // group, group)
    s = vg.abs().amax(dim=-1, keepdim=True) / qmax
    t = vg / s
    vq = (s * (t + (torch.round(t) - t).detach())).reshape(rows, n)
    (vq * g).sum().backward()
    mine = _through_quantiser(v.detach().numpy(), vq.detach().numpy(), g.numpy(), bits, group)
    np.testing.assert_allclose(mine, v.grad.numpy(), rtol=1e-10, atol=1e-12)


@gpu
@pytest.mark.parametrize("n,m,T,dtype", [(128, 96, 192, "f32"), (256, 64, 160, "f32")])
def test_step_matches_the_oracle(n, m, T, dtype):
    import torch
    from paper_2509_09679_amd.calibration import ButterflyCalibrator, QuantSpec

    X, theta, _ = synth.small_case(n, T, dtype, seed=41)
    Wn, _, _ = synth.small_case(n, m, dtype, seed=42, outliers=0, dist="normal")
    theta = (0.3 * theta).astype(np.float32)  # away from identity, so that every layer matters
    act, wgt = (4, n, "f32"), (4, 32, "f32")
    dev = "cuda:0"
    cal = ButterflyCalibrator(synth.storage_to_torch(Wn, dtype, dev), QuantSpec(*act), QuantSpec(*wgt),
                              theta=torch.from_numpy(theta).to(dev))
    loss, g, kl = cal.loss_and_grad(synth.storage_to_torch(X, dtype, dev))
    torch.cuda.synchronize()
    X64, W64 = synth.to_f64(X, dtype), synth.to_f64(Wn, dtype)
    ref_loss, ref_g, ref_hist = _oracle_step(X64, W64, theta, n, act, wgt)
    # The GPU's rotation differs from the oracle's in the last float32 bits, so a few values that sit on a rounding
    # boundary get the neighbouring code (each of them a valid rounding: tests/test_gpu_parity.py).  Counted here:
    Xq_gpu = cal.Xq.double().cpu().numpy()
    Wq_gpu = cal.Wq.double().cpu().numpy()
    Xq_ref = oracle.dequantize(*oracle.quantize(oracle.forward(X64, theta, n).astype(np.float32), act[1], act[0], act[2]),
                               act[1]).astype(np.float64)
    Wq_ref = oracle.dequantize(*oracle.quantize(oracle.forward(W64, theta, n).astype(np.float32), wgt[1], wgt[0], wgt[2]),
                               wgt[1]).astype(np.float64)
    differ = int((np.abs(Xq_gpu - Xq_ref) > 1e-4 * np.abs(Xq_ref).max()).sum() +
                 (np.abs(Wq_gpu - Wq_ref) > 1e-4 * np.abs(Wq_ref).max()).sum())
    assert differ <= 1e-3 * (T * n + m * n), differ
    # With the fake-quantised values the GPU actually produced, the rest of the step -- error matrix, loss, the
    # gradient rule through the quantiser, both backward passes -- must agree with the oracle's arithmetic in
    # double to float32 accuracy; what the `differ` codes move is then no longer part of the comparison.
    same_loss, same_g, _ = _oracle_step(X64, W64, theta, n, act, wgt, Xq_given=Xq_gpu, Wq_given=Wq_gpu)
    assert abs(float(loss) - same_loss) <= 1e-4 * same_loss, (float(loss), same_loss, differ)
    gd = g.cpu().numpy().astype(np.float64) - same_g
    assert np.linalg.norm(gd) <= 1e-3 * np.linalg.norm(same_g), (np.linalg.norm(gd) / np.linalg.norm(same_g), differ)
    # and with the oracle's own codes the loss moves by no more than those codes can move it:
    # |L - L'| <= (2 |E| + |dE|) |dE| with dE the change of the error matrix
    dE = Xq_gpu @ Wq_gpu.T - Xq_ref @ Wq_ref.T
    nE = np.sqrt(ref_loss)
    assert abs(same_loss - ref_loss) <= (2 * nE + np.linalg.norm(dE)) * np.linalg.norm(dE) * (1 + 1e-9) + 1e-12 * ref_loss
    h = cal.hist.cpu().numpy().astype(np.int64)
    assert h.sum() == T * n and np.abs(h - ref_hist.astype(np.int64)).sum() <= 2 * differ
    # L_uniform from the kernel's histogram = the oracle's KL on the same counts, and close to the oracle's own
    assert abs(float(kl) - oracle.uniformity_kl(h.astype(np.uint64), act[0])) <= 1e-12
    assert abs(float(kl) - oracle.uniformity_kl(ref_hist, act[0])) <= 1e-2 * max(1e-3, oracle.uniformity_kl(ref_hist, act[0])) + 8.0 * differ / (T * n)


@gpu
def test_sgd_from_identity_lowers_the_reconstruction_loss():
    import torch
    from paper_2509_09679_amd.calibration import ButterflyCalibrator, QuantSpec

    n, m, T, dtype = 512, 256, 2048, "f16"
    X, _, _ = synth.small_case(n, T, dtype, seed=43, outliers=6)
    Wn, _, _ = synth.small_case(n, m, dtype, seed=44, outliers=0, dist="normal")
    dev = "cuda:0"
    cal = ButterflyCalibrator(synth.storage_to_torch(Wn, dtype, dev), QuantSpec(4, 128, "f16"), QuantSpec(4, 128, "f16"))
    Xd = synth.storage_to_torch(X, dtype, dev)
    # identity is a stationary point by symmetry (theta -> -theta), so the first steps wander before the loss falls
    losses = cal.fit(Xd, steps=100, lr=1.0)
    torch.cuda.synchronize()
    final, _, kl = cal.loss_and_grad(Xd)
    assert np.isfinite(cal.kl_seen).all() and float(kl) >= 0.0
    assert np.isfinite(losses).all()
    assert float(final) < 0.85 * losses[0], (losses[0], float(final))
    # theta moved away from the identity and the transform is still orthogonal: norms are preserved
    assert float(cal.theta.abs().max()) > 0
    from paper_2509_09679_amd import binding as B
    Y = torch.empty_like(Xd)
    B.bq_butterfly_fwd(Xd, Y, cal.plan, B.make_rows(Xd, n, 1))
    torch.cuda.synchronize()
    nx, ny = Xd.float().norm(dim=1), Y.float().norm(dim=1)
    assert float(((nx - ny).abs() / nx).max()) < 2e-3
