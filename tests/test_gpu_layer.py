"""The autograd layer over the soft path: gradients that autograd hands back must be the
oracle's (float64) contracted with the same upstream gradient, and a toy fit must move the
direction and the thresholds towards the ones that produced the target curve."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import ecc_oracle as O
from paper_2510_20271_amd import layer, synth
from tests.gpu_util import dev, host

pytestmark = pytest.mark.gpu


from tests.test_gpu_soft import _close, _close_sum  # noqa: E402  (tolerances: see there)


@pytest.mark.parametrize("shape", [(48, 60), (10, 20, 24)])
def test_autograd_gradients_match_the_oracle(shape):
    nd = len(shape)
    B, T, alpha, lam = 3, 24, 0.02, 15.0
    X = np.stack([synth.grf(shape, 2.0, 70 + i) for i in range(B)])
    u = np.array([np.cos(0.4), np.sin(0.4)] if nd == 2 else [0.48, 0.6, 0.64], np.float32)
    tau = np.linspace(X.min(), X.max() + alpha * sum(shape), T).astype(np.float32)
    gup = np.random.default_rng(4).standard_normal((B, T)).astype(np.float32)

    g = dev(X).requires_grad_(True)
    ut = dev(u).requires_grad_(True)
    tt = dev(tau).requires_grad_(True)
    chi = layer.soft_ecc(g, ut, tt, alpha, lam)
    (chi * dev(gup)).sum().backward()

    want_chi = O.soft_fwd_batch(X, u, alpha, tau, lam)
    _close_sum(host(chi.detach()), want_chi, 1e-4, "chi")
    gX = np.zeros(X.shape)
    g_tau = np.zeros(T)
    g_u = np.zeros(nd)
    for b in range(B):
        gx_b, dtau_b, du_b = O.soft_bwd(X[b], u, alpha, tau, lam, gup[b])
        gX[b] = gx_b
        g_tau += gup[b] * dtau_b
        g_u += gup[b] @ du_b
    _close(host(g.grad), gX, 1e-3, "grad_X")
    _close_sum(host(tt.grad), g_tau, 1e-3, "grad_tau")
    _close_sum(host(ut.grad), g_u, 1e-3, "grad_u")


def _setup():
    shape = (64, 64)
    X = dev(np.stack([synth.grf(shape, 3.0, 90 + i) for i in range(4)]))
    lo, hi = float(X.min()), float(X.max()) + 0.01 * 128
    return X, lo, hi


def test_direction_gradient_through_the_angle_matches_finite_differences():
    X, lo, hi = _setup()
    target = layer.SoftECCLayer(2, 16, lo, hi, alpha=0.01, lam=12.0, theta=[0.9]).cuda()
    with torch.no_grad():
        want = target(X)

    def loss_at(theta):
        m = layer.SoftECCLayer(2, 16, lo, hi, alpha=0.01, lam=12.0, theta=[theta]).cuda()
        loss = ((m(X) - want) ** 2).sum()
        return m, loss

    m, loss = loss_at(0.5)
    loss.backward()
    g = float(m.theta.grad[0])
    h = 2e-3
    with torch.no_grad():
        fd = (float(loss_at(0.5 + h)[1]) - float(loss_at(0.5 - h)[1])) / (2 * h)
    assert abs(g - fd) <= 0.05 * max(abs(fd), 1e-6), (g, fd)
    n = m.direction()
    assert abs(float((n * n).sum().detach()) - 1.0) < 1e-6  # the direction stays on the unit circle


def test_layer_learns_its_thresholds_back():
    X, lo, hi = _setup()
    target = layer.SoftECCLayer(2, 16, lo, hi, alpha=0.01, lam=12.0)
    target.cuda()
    with torch.no_grad():
        want = target(X)
    model = layer.SoftECCLayer(2, 16, lo, hi, alpha=0.01, lam=12.0, learn_theta=False).cuda()
    with torch.no_grad():
        model.tau += 0.03
    opt = torch.optim.Adam([model.tau], lr=0.002)
    first = None
    for _ in range(200):
        opt.zero_grad()
        loss = ((model(X) - want) ** 2).mean()
        loss.backward()
        opt.step()
        first = first if first is not None else float(loss.detach())
    assert float(loss.detach()) < 0.1 * first
    assert float((model.tau - target.tau).abs().mean().detach()) < 0.015
