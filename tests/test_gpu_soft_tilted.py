"""GPU parity of the soft ECC with the coefficient of the tilted field (ecc_soft_fwd_tilted /
ecc_soft_bwd_tilted) against the float64 CPU oracle, through the C ABI: the fused 2D path, the
tile path (2D with many thresholds, 3D), and the sharp limit against the directional hard
curves.  Tolerances as for the plain soft path: 1e-4 (chi) and 1e-3 (derivatives) of
max|oracle| per array and item."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import ecc_oracle as O
from paper_2510_20271_amd import api, synth
from paper_2510_20271_amd.layer import SoftECCLayer
from tests.gpu_util import dev, host
from tests.test_gpu_soft import _close, _close_sum

pytestmark = pytest.mark.gpu


def _run_tilted(Xb, u, alpha, tau, lam, G, expect_other_c=True):
    nd = Xb.ndim - 1
    g, ud, td = dev(Xb), dev(u), dev(tau)
    chi = host(api.ecc_soft_fwd(g, nd, ud, alpha, td, lam, tilted_c=True))
    gx, dt, du = api.ecc_soft_bwd(g, nd, ud, alpha, td, lam, grad_chi=dev(G), tilted_c=True)
    gx, dt, du = host(gx), host(dt), host(du)
    differs = False
    for i, X in enumerate(Xb):
        c = O.coeff_tilted(X, u, alpha)
        differs |= not np.array_equal(c, O.coeff(X))
        ref_chi = O.soft_fwd(X, u, alpha, tau, lam, c=c)
        rgx, rdt, rdu = O.soft_bwd(X, u, alpha, tau, lam, G[i], c=c)
        _close_sum(chi[i], ref_chi, 1e-4, f"chi[{i}]")
        _close(gx[i], rgx, 1e-3, f"grad_X[{i}]")
        _close_sum(dt[i], rdt, 1e-3, f"dchi_dtau[{i}]")
        _close_sum(du[i], rdu, 1e-3, f"dchi_du[{i}]")
    assert differs or not expect_other_c  # the case tells the two coefficients apart


@pytest.mark.parametrize("shape", [(1, 9), (9, 1), (7, 13), (64, 64), (100, 259), (45, 2048), (3, 5000)])
def test_soft_tilted_2d_fused(shape):
    B, T = 2, 9
    Xb = np.stack([synth.grf(shape, 2.0, 60 + i) if min(shape) > 1 else
                   np.random.default_rng(i).standard_normal(shape).astype(np.float32) for i in range(B)])
    u = np.array([np.cos(2.1), np.sin(2.1)], np.float32)
    alpha = np.float32(0.05)
    Y = np.stack([O.tilt_field(x, u, alpha) for x in Xb])
    tau = np.linspace(Y.min() - 0.1, Y.max() + 0.5, T).astype(np.float32)
    G = np.random.default_rng(1).standard_normal((B, T)).astype(np.float32)
    _run_tilted(Xb, u, alpha, tau, np.float32(20.0), G, expect_other_c=min(shape) > 1)


def test_soft_tilted_2d_tile_path_many_thresholds():
    B, T = 2, 300  # more thresholds than the fused path takes
    Xb = np.stack([synth.grf((70, 130), 2.0, 70 + i) for i in range(B)])
    u = np.array([-0.8, 0.6], np.float32)
    alpha = np.float32(0.04)
    tau = np.linspace(-3, 9, T).astype(np.float32)
    G = np.random.default_rng(3).standard_normal((B, T)).astype(np.float32)
    _run_tilted(Xb, u, alpha, tau, np.float32(15.0), G)


@pytest.mark.parametrize("shape", [(2, 2, 2), (5, 6, 7), (9, 30, 70), (3, 33, 129)])
def test_soft_tilted_3d(shape):
    B, T = 2, 5
    Xb = np.stack([synth.grf(shape, 1.5, 80 + i) for i in range(B)])
    u = np.array([0.48, -0.6, 0.64], np.float32)
    alpha = np.float32(0.05)
    Y = np.stack([O.tilt_field(x, u, alpha) for x in Xb])
    tau = np.linspace(Y.min(), Y.max() + 1.0, T).astype(np.float32)
    G = np.random.default_rng(2).standard_normal((B, T)).astype(np.float32)
    _run_tilted(Xb, u, alpha, tau, np.float32(8.0), G, expect_other_c=min(shape) > 2)


@pytest.mark.parametrize("shape", [(60, 300), (12, 20, 70)])
def test_sharp_limit_is_the_directional_hard_curve(shape):
    nd = len(shape)
    X = synth.grf(shape, 2.0, 91)[None]
    u = np.array([0.6, -0.8] if nd == 2 else [0.36, 0.48, -0.8], np.float32)
    alpha = 0.02
    bins = 12
    Y = O.tilt_field(X[0], u, alpha)
    lo, hi = float(Y.min()), float(Y.max())
    hard = host(api.ecc_hard_dir(dev(X), nd, dev(u[None]), alpha, bins, range=(lo, hi)))[0, 0]
    t = O.thresholds_equal_width(lo, hi, bins).astype(np.float32)
    # keep the thresholds that no tilted value comes close to (the sigmoid is a step only away from them)
    far = np.array([np.min(np.abs(Y.astype(np.float64) - tb)) > 2e-5 for tb in t])
    assert far.sum() >= bins // 2
    soft = host(api.ecc_soft_fwd(dev(X), nd, dev(u), alpha, dev(t), 2e6, tilted_c=True))[0]
    np.testing.assert_allclose(soft[far], hard[far], atol=2e-3)


def test_layer_with_tilted_coefficient():
    X = torch.from_numpy(np.stack([synth.grf((40, 90), 2.0, 95 + i) for i in range(2)])).cuda()
    layer = SoftECCLayer(2, 7, -1.0, 6.0, alpha=0.05, lam=10.0, theta=[2.0], tilted_c=True).cuda()
    chi = layer(X)
    u = layer.direction().detach().cpu().numpy().astype(np.float32)
    tau = layer.tau.detach().cpu().numpy()
    for i in range(2):
        x = X[i].cpu().numpy()
        _close_sum(chi[i].detach().cpu().numpy(), O.soft_fwd(x, u, 0.05, tau, 10.0, c=O.coeff_tilted(x, u, 0.05)),
               1e-4, "layer chi")
    chi.sum().backward()
    assert layer.tau.grad is not None and torch.isfinite(layer.tau.grad).all()
    assert layer.theta.grad is not None and torch.isfinite(layer.theta.grad).all()
