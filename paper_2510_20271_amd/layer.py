"""Differentiable ECC layer over the C ABI (the paper's "differentiable PyTorch layer").

``SoftECCFunction`` is a ``torch.autograd.Function``: forward is ``ecc_soft_fwd_save`` (Eq. 6, plus the
sums of Eq. 9-10, which share its sigmoids, and the saved list of critical vertices), backward is
``ecc_soft_bwd_saved`` (Eq. 8 over that list; appendix on analytical derivatives).  The kernels
return d chi / d tau and d chi / d u uncontracted ([batch, T] and [batch, T, ndim]); the two
small contractions with the upstream gradient that autograd needs are the only arithmetic
done here.  ``SoftECCLayer`` holds the learnable thresholds and a direction kept on the unit
sphere by reparametrisation (an angle in 2D, two angles in 3D), as the main text suggests.

Inputs must live on the GPU; there is no CPU path.
"""
from __future__ import annotations

import math

import torch

from . import api


class SoftECCFunction(torch.autograd.Function):
    """chi[b, j] = sum_p c(p) sigmoid(lambda (tau_j - X_b(p) - alpha <u, p>)), p = (x, y[, z])."""

    @staticmethod
    def forward(ctx, grid, u, tau, alpha: float, lam: float, tilted_c: bool = False):
        ndim = grid.dim() - 1
        grid_c = grid.detach().contiguous().float()
        u_c = u.detach().contiguous().float()
        tau_c = tau.detach().contiguous().float()
        ctx.alpha, ctx.lam, ctx.ndim, ctx.tilted_c = float(alpha), float(lam), ndim, bool(tilted_c)
        need_x, need_u, need_tau = ctx.needs_input_grad[:3]
        if not (need_x or need_u or need_tau):
            return api.ecc_soft_fwd(grid_c, ndim, u_c, alpha, tau_c, lam, tilted_c=ctx.tilted_c)
        # The forward kernel shares its sigmoids with the sums of Eq. 9 / Eq. 10 and finds the vertices
        # with c != 0 that Eq. 8 needs: it returns the former and saves the latter, so backward() neither
        # sweeps the grid again nor, with fixed inputs and learnable thresholds (the usual case), runs a
        # kernel at all.
        want = [n for n, need in (("dchi_du", need_u), ("dchi_dtau", need_tau)) if need]
        chi, dtau, du, state = api.ecc_soft_fwd_save(grid_c, ndim, u_c, alpha, tau_c, lam, tilted_c=ctx.tilted_c,
                                                     want=want)
        ctx.save_for_backward(grid_c, u_c, tau_c, state if need_x else None, dtau, du)
        return chi

    @staticmethod
    def backward(ctx, grad_chi):
        grid, u, tau, state, dtau, du = ctx.saved_tensors
        g = grad_chi.contiguous().float()
        need_x, need_u, need_tau = ctx.needs_input_grad[:3]
        grad_X = None
        if need_x:
            grad_X = api.ecc_soft_bwd_saved(grid, ctx.ndim, u, ctx.alpha, tau, ctx.lam, state, grad_chi=g,
                                            tilted_c=ctx.tilted_c)
        grad_u = torch.einsum("bj,bjd->d", g, du) if need_u else None
        grad_tau = (g * dtau).sum(0) if need_tau else None
        return grad_X, grad_u, grad_tau, None, None, None


def soft_ecc(grid, u, tau, alpha: float, lam: float, tilted_c: bool = False):
    """Functional form: grid [batch, (D,) H, W] float32 on the GPU, u [ndim], tau [T].
    tilted_c: take c(p) from the tilted field X + alpha <u, p> (so that a sharp sigmoid gives
    the directional hard curve) instead of from X; c stays a constant for the derivatives."""
    return SoftECCFunction.apply(grid, u, tau, alpha, lam, tilted_c)


class SoftECCLayer(torch.nn.Module):
    """Soft directional ECC with learnable thresholds and direction.

    tau:   T thresholds, initialised evenly over [tau_min, tau_max].
    theta: the direction's angle(s): u = (cos t, sin t) in 2D; in 3D u = (sin p cos t,
           sin p sin t, cos p) with theta = (t, p).  ||u|| = 1 by construction.
    alpha (weight of the tilt) and lam (sharpness of the sigmoid) are fixed.
    tilted_c: c(p) of the tilted field instead of the field's own (see soft_ecc).
    """

    def __init__(self, ndim: int, T: int, tau_min: float, tau_max: float, alpha: float = 0.01,
                 lam: float = 20.0, theta=None, learn_tau: bool = True, learn_theta: bool = True,
                 tilted_c: bool = False):
        super().__init__()
        if ndim not in (2, 3):
            raise ValueError("ndim must be 2 or 3")
        self.ndim, self.alpha, self.lam, self.tilted_c = ndim, float(alpha), float(lam), bool(tilted_c)
        tau = torch.linspace(float(tau_min), float(tau_max), T, dtype=torch.float32)
        if theta is None:
            theta = [0.3] if ndim == 2 else [0.3, 0.5 * math.pi]
        theta = torch.as_tensor(theta, dtype=torch.float32).reshape(ndim - 1)
        self.tau = torch.nn.Parameter(tau, requires_grad=learn_tau)
        self.theta = torch.nn.Parameter(theta, requires_grad=learn_theta)

    def direction(self) -> torch.Tensor:
        t = self.theta
        if self.ndim == 2:
            return torch.stack([torch.cos(t[0]), torch.sin(t[0])])
        return torch.stack([torch.sin(t[1]) * torch.cos(t[0]), torch.sin(t[1]) * torch.sin(t[0]),
                            torch.cos(t[1])])

    def forward(self, grid: torch.Tensor) -> torch.Tensor:
        return soft_ecc(grid, self.direction(), self.tau, self.alpha, self.lam, self.tilted_c)
