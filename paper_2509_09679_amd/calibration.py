"""One calibration step of the learnable butterfly rotation on a single linear layer, built from the
library's calls (paper, sections "Loss Function", "Uniformity Regularization" and "Implementation Details").

    L_recon   = || X W^T - Dequant(Quant(B X)) . Dequant(Quant(W B^T))^T ||^2      (rows of X are tokens)
    L_uniform = D_KL(P_bins || U): P_bins the occupancy of the 2^b activation code bins, U uniform

L_uniform is evaluated from the histogram the fake-quantising kernel counts in the same pass and is REPORTED beside
L_recon; it is not differentiated (the paper does not say how a gradient passes the hard bin assignment), so the
descent direction is that of L_recon alone.

The butterfly work — B X, W B^T (the forward transform over the rows of W), both fake quantisations and both
backward passes — runs in the HIP library; torch supplies memory, the two dense products with W (they
belong to the layer, not to the transform) and the element-wise rule that carries the loss gradient from
the fake-quantised values back to the rotated values.

The paper does not say how gradients pass `round` and the scale.  Reading taken here (what automatic
differentiation of  s * round(v / s),  s = max|v| / qmax,  gives with a straight-through `round`): with
g = dL/d(Dequant(Quant(v))) on a group,
    dL/dv_j = g_j                                          (straight-through),
    dL/dv_m += sign(v_m) / qmax * sum_j g_j (q_j - v_j / s)   for m = argmax |v|   (through the scale),
the binary16 rounding of s being treated as the identity.  Without the second term the gradient cannot see
that a rotation which lowers the group maxima lowers the quantisation noise: (W B^T)(B x) = W x for every
theta, so the straight-through term alone only sees noise cross terms.  SGD with a cosine learning-rate
schedule from theta = 0 (identity), as in the paper's set-up.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

from . import binding as B


@dataclass
class QuantSpec:
    bits: int
    group: int
    scale_dtype: str = "f16"


class ButterflyCalibrator:
    """Holds theta (float32, [1][k][n/2]) for one layer and the buffers of a step.  X: [T, n], W: [m, n], both
    of the same 16-bit or 32-bit row type, resident on the GPU."""

    def __init__(self, W, act: QuantSpec, wgt: QuantSpec, theta=None):
        import torch

        self.torch = torch
        self.W = W
        self.m, self.n = W.shape
        self.k = self.n.bit_length() - 1
        assert 1 << self.k == self.n
        self.act, self.wgt = act, wgt
        dev = W.device
        self.theta = (torch.zeros((1, self.k, self.n // 2), dtype=torch.float32, device=dev)
                      if theta is None else theta.clone())
        self.plan = torch.empty(B.bq_plan_bytes(self.n, 1), dtype=torch.uint8, device=dev)
        self.Wq = torch.empty_like(W)
        self.dW = torch.empty_like(W)
        self.dth_x = torch.empty_like(self.theta)
        self.dth_w = torch.empty_like(self.theta)
        self.hist = torch.zeros(1 << act.bits, dtype=torch.int64, device=dev)
        self._ws = None

    def _workspace(self, rows):
        need = max(256, B.bq_butterfly_bwd_workspace_bytes(rows))
        if self._ws is None or self._ws.numel() < need:
            self._ws = self.torch.empty(need, dtype=self.torch.uint8, device=self.W.device)
        return self._ws

    def _through_quantiser(self, V, Vq, G, spec: QuantSpec):
        """dL/dV from G = dL/dVq (all float32, [rows, n]); see the module text."""
        torch = self.torch
        rows, n = V.shape
        g = spec.group
        qmax = float((1 << (spec.bits - 1)) - 1)
        v = V.reshape(rows, n // g, g)
        amax, idx = v.abs().max(dim=-1, keepdim=True)
        s = amax / qmax
        ok = s > 0
        inv = torch.where(ok, 1.0 / torch.where(ok, s, torch.ones_like(s)), torch.zeros_like(s))
        r = (Vq.reshape(rows, n // g, g) - v) * inv  # q_j - v_j / s
        Gg = G.reshape(rows, n // g, g)
        through_scale = (Gg * r).sum(dim=-1, keepdim=True) * torch.sign(torch.gather(v, -1, idx)) / qmax
        dV = Gg.clone()
        dV.scatter_add_(-1, idx, through_scale)
        return dV.reshape(rows, n)

    def _bwd_f32(self, X, dV, dtheta):
        """dtheta from (X, dL/dV) with float32 rows: the gradient's entries span many orders of magnitude (the
        term through the scale sits on one element per group), which a 16-bit row type would flush to zero."""
        X32 = X if X.dtype == self.torch.float32 else X.float()
        rows = B.make_rows(X32, self.n, 1)
        B.bq_butterfly_bwd(X32, dV.contiguous(), self.plan, None, dtheta, self._workspace(rows), rows)
        return dtheta

    def uniformity_kl(self):
        """D_KL(P_bins || U) of the activation codes of the last loss_and_grad call, from the kernel's histogram
        (0 log 0 = 0); a 0-dim float64 tensor."""
        torch = self.torch
        h = self.hist.to(torch.float64)
        p = h / h.sum().clamp_min(1.0)
        bins = float(1 << self.act.bits)
        return torch.where(p > 0, p * torch.log(p.clamp_min(1e-300) * bins), torch.zeros_like(p)).sum()

    def loss_and_grad(self, X):
        """Returns (L_recon as a 0-dim float32 tensor, dtheta of L_recon, L_uniform as a 0-dim float64 tensor);
        self.hist holds the activation code bins."""
        torch = self.torch
        B.bq_plan_build(self.theta, self.n, 1, self.plan)
        rx, rw = B.make_rows(X, self.n, 1), B.make_rows(self.W, self.n, 1)
        V, Xq, Wr = torch.empty_like(X), torch.empty_like(X), torch.empty_like(self.W)
        qa = B.make_quant(self.act.bits, self.act.group, self.act.scale_dtype)
        qw = B.make_quant(self.wgt.bits, self.wgt.group, self.wgt.scale_dtype)
        B.bq_butterfly_fwd(X, V, self.plan, rx)
        B.bq_butterfly_fwd_fakequant(X, self.plan, Xq, self.hist, qa, rx)
        B.bq_butterfly_fwd(self.W, Wr, self.plan, rw)
        B.bq_butterfly_fwd_fakequant(self.W, self.plan, self.Wq, None, qw, rw)
        # the layer's dense products (float32 accumulate)
        Xq32, Wq32 = Xq.float(), self.Wq.float()
        E = (Xq32 @ Wq32.t()) - (X.float() @ self.W.float().t())
        loss = (E * E).sum()
        dV = self._through_quantiser(V.float(), Xq32, 2.0 * (E @ Wq32), self.act)
        dWr = self._through_quantiser(Wr.float(), Wq32, 2.0 * (E.t() @ Xq32), self.wgt)
        gx = self._bwd_f32(X, dV, self.dth_x)
        gw = self._bwd_f32(self.W, dWr, self.dth_w)
        self.Xq = Xq
        return loss, gx + gw, self.uniformity_kl()

    def fit(self, X, steps: int, lr: float, log=None):
        """SGD with a cosine learning-rate schedule; returns the losses seen (before each update).  The step
        is lr times the unit-norm gradient (this module's choice: the loss scale varies by orders of
        magnitude with the batch and layer size, the paper gives no learning rate)."""
        losses = []
        self.kl_seen = []
        for t in range(steps):
            loss, g, kl = self.loss_and_grad(X)
            losses.append(float(loss))
            self.kl_seen.append(float(kl))
            step_lr = 0.5 * lr * (1.0 + math.cos(math.pi * t / steps))
            gn = g.norm()
            self.theta -= step_lr * g / (gn + 1e-30)
            if log:
                log(t, losses[-1])
        return losses
