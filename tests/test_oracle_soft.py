"""Pins for the soft single-direction ECC oracle (Eq. 6, Eq. 8-10); no GPU.

Closed forms pin the formula and the coordinate convention (p = (x, y[, z]),
x the fastest axis, 0-based), limits pin the sign of the argument, the hard
curve pins the lambda -> infinity limit, finite differences and the exact
identities between Eq. 8, 9 and 10 pin the derivatives.
"""
import numpy as np
import pytest

from oracle import ecc_oracle as O


def _sig(x):
    return 1.0 / (1.0 + np.exp(-x))


def test_single_pixel_closed_form():
    X = np.array([[0.25]], dtype=np.float32)
    tau = np.array([-1.0, 0.25, 0.3, 2.0])
    chi = O.soft_fwd(X, u=[0.6, 0.8], alpha=0.5, tau=tau, lam=3.0)
    np.testing.assert_allclose(chi, _sig(3.0 * (tau - 0.25)), rtol=1e-14)


def test_reversed_ramp_pins_coordinates_2d_and_3d():
    """X strictly decreasing in linear index: the only critical vertex is the
    last one, so chi(tau) = sigma(lambda (tau - X_last - alpha <u, p_last>))
    with p_last = (W-1, H-1[, D-1])."""
    H, W = 3, 5
    X = (100.0 - np.arange(H * W)).reshape(H, W).astype(np.float32)
    u = np.array([0.3, -0.7])
    alpha, lam = 0.2, 1.5
    tau = np.linspace(80, 95, 7)
    chi = O.soft_fwd(X, u, alpha, tau, lam)
    z = tau - float(X[-1, -1]) - alpha * (u[0] * (W - 1) + u[1] * (H - 1))
    np.testing.assert_allclose(chi, _sig(lam * z), rtol=1e-13)
    gx, dt, du = O.soft_bwd(X, u, alpha, tau, lam)
    ds = lam * _sig(lam * z) * (1 - _sig(lam * z))
    np.testing.assert_allclose(dt, ds, rtol=1e-12)
    np.testing.assert_allclose(du, -alpha * ds[:, None] * np.array([W - 1, H - 1])[None, :], rtol=1e-12)
    assert np.count_nonzero(gx) == 1
    np.testing.assert_allclose(gx[-1, -1], -ds.sum(), rtol=1e-12)

    D, H, W = 2, 3, 4
    X = (100.0 - np.arange(D * H * W)).reshape(D, H, W).astype(np.float32)
    u = np.array([0.3, -0.7, 0.5])
    chi = O.soft_fwd(X, u, alpha, tau, lam)
    z = tau - float(X[-1, -1, -1]) - alpha * (u[0] * (W - 1) + u[1] * (H - 1) + u[2] * (D - 1))
    np.testing.assert_allclose(chi, _sig(lam * z), rtol=1e-13)


def _field(shape, seed):
    from scipy.ndimage import gaussian_filter
    rng = np.random.default_rng(seed)
    return gaussian_filter(rng.standard_normal(shape), 1.5, mode="wrap").astype(np.float32)


def test_limits_in_tau_and_shift_invariance():
    X = _field((12, 15), 1)
    u = [np.cos(0.3), np.sin(0.3)]
    chi = O.soft_fwd(X, u, 0.01, np.array([-1e3, 1e3]), 20.0)
    np.testing.assert_allclose(chi, [0.0, 1.0], atol=1e-12)  # sum of c is 1
    tau = np.linspace(-0.5, 0.5, 9)
    a = O.soft_fwd(X, u, 0.01, tau, 20.0)
    s = 0.375  # exactly representable shift
    b = O.soft_fwd((X + np.float32(s)).astype(np.float32), u, 0.01, tau + s, 20.0)
    np.testing.assert_allclose(a, b, rtol=1e-6, atol=1e-9)


@pytest.mark.parametrize("shape", [(10, 13), (5, 6, 7)])
def test_large_lambda_recovers_hard_curve(shape):
    rng = np.random.default_rng(4)
    X = rng.permutation(np.prod(shape)).reshape(shape).astype(np.float32)  # distinct integers
    c = O.coeff(X)
    tau = np.arange(np.prod(shape)) + 0.5  # never equal to a grid value
    u = np.zeros(len(shape))
    soft = O.soft_fwd(X, u, 0.0, tau, 200.0, c=c)
    hard = O.ecc_bruteforce(X, tau)
    np.testing.assert_allclose(soft, hard, atol=1e-9)
    # alpha != 0: limit is sum_p c(p) 1[X(p) + alpha <u,p> <= tau] with c from X
    u = np.array([np.cos(0.3), np.sin(0.3), 0.1234][: len(shape)])
    P = O.coordinates(shape)
    y = X.ravel().astype(np.float64) + 0.25 * (P @ u)
    tau2 = np.sort(y)[:-1] + np.diff(np.sort(y)) / 2
    gaps = np.diff(np.sort(y)).min()
    lam = 80.0 / gaps
    soft = O.soft_fwd(X, u, 0.25, tau2, lam, c=c)
    ref = np.array([(c.ravel()[y <= t]).sum() for t in tau2])
    np.testing.assert_allclose(soft, ref, atol=1e-9)


@pytest.mark.parametrize("shape", [(9, 11), (4, 5, 6)])
def test_gradients_against_finite_differences(shape):
    X = _field(shape, 2)
    nd = len(shape)
    rng = np.random.default_rng(8)
    u = rng.standard_normal(nd)
    u /= np.linalg.norm(u)
    alpha, lam = 0.05, 6.0
    tau = np.linspace(float(X.min()), float(X.max()) + 0.3, 5)
    g = rng.standard_normal(len(tau))
    c = O.coeff(X)
    gx, dt, du = O.soft_bwd(X, u, alpha, tau, lam, g=g, c=c)
    h = 1e-6
    f = lambda **kw: O.soft_fwd(kw.get("X", X), kw.get("u", u), alpha, kw.get("tau", tau), lam, c=c)
    # tau (diagonal Jacobian)
    fd = (f(tau=tau + h) - f(tau=tau - h)) / (2 * h)
    np.testing.assert_allclose(dt, fd, rtol=1e-6, atol=1e-8)
    # u (ambient)
    for k in range(nd):
        e = np.zeros(nd); e[k] = h
        fd = (f(u=u + e) - f(u=u - e)) / (2 * h)
        np.testing.assert_allclose(du[:, k], fd, rtol=1e-6, atol=1e-8)
    # X at sampled vertices, contracted with g; c is held fixed (the paper
    # differentiates through the sigmoid only)
    Xd = X.astype(np.float64)
    nz = np.flatnonzero(c.ravel())
    picks = list(nz[:6]) + [0, X.size - 1]
    for i in picks:
        Xp, Xm = Xd.copy(), Xd.copy()
        Xp.flat[i] += h
        Xm.flat[i] -= h
        fd = g @ (f(X=Xp) - f(X=Xm)) / (2 * h)
        np.testing.assert_allclose(gx.flat[i], fd, rtol=1e-5, atol=1e-8)
    assert np.all(gx.ravel()[c.ravel() == 0] == 0)
    if nd == 2:  # derivative along the unit circle, u = (cos t, sin t)
        th = 0.3
        uu = lambda t: np.array([np.cos(t), np.sin(t)])
        _, _, du2 = O.soft_bwd(X, uu(th), alpha, tau, lam, c=c)
        fd = (f(u=uu(th + h)) - f(u=uu(th - h))) / (2 * h)
        np.testing.assert_allclose(du2 @ np.array([-np.sin(th), np.cos(th)]), fd, rtol=1e-6, atol=1e-8)


def test_exact_identities_between_eq8_eq9_eq10():
    """dchi/dtau_j = -sum_p dchi_j/dX(p);  dchi_j/du = alpha sum_p p dchi_j/dX(p)."""
    X = _field((8, 9), 3)
    u = np.array([0.8, -0.6])
    alpha, lam = 0.07, 9.0
    tau = np.linspace(-0.4, 0.6, 4)
    _, dt, du = O.soft_bwd(X, u, alpha, tau, lam)
    P = O.coordinates(X.shape)
    for j in range(len(tau)):
        g = np.zeros(len(tau)); g[j] = 1.0
        gx, _, _ = O.soft_bwd(X, u, alpha, tau, lam, g=g)
        np.testing.assert_allclose(dt[j], -gx.sum(), rtol=1e-12)
        np.testing.assert_allclose(du[j], alpha * (gx.ravel() @ P), rtol=1e-10, atol=1e-14)


def test_integral_of_dchi_dtau_is_one():
    X = _field((10, 10), 5)
    tau = np.linspace(-3, 3, 6001)
    _, dt, _ = O.soft_bwd(X, [1.0, 0.0], 0.0, tau, 15.0)
    np.testing.assert_allclose(np.sum((dt[1:] + dt[:-1]) / 2 * np.diff(tau)), 1.0, rtol=1e-6)


def test_batch_wrappers():
    Xb = np.stack([_field((6, 7), s) for s in (1, 2)])
    u, alpha, lam = [0.6, 0.8], 0.1, 4.0
    tau = np.linspace(-0.3, 0.3, 3)
    chi = O.soft_fwd_batch(Xb, u, alpha, tau, lam)
    G = np.array([[1.0, 2.0, 3.0], [-1.0, 0.5, 0.0]])
    gx, dt, du = O.soft_bwd_batch(Xb, u, alpha, tau, lam, G)
    for i in range(2):
        np.testing.assert_array_equal(chi[i], O.soft_fwd(Xb[i], u, alpha, tau, lam))
        a, b, c = O.soft_bwd(Xb[i], u, alpha, tau, lam, g=G[i])
        np.testing.assert_array_equal(gx[i], a)
        np.testing.assert_array_equal(dt[i], b)
        np.testing.assert_array_equal(du[i], c)


def test_tilted_coefficient_makes_the_sharp_limit_a_directional_hard_curve():
    rng = np.random.default_rng(12)
    for shape, u in (((8, 9), [0.6, 0.8]), ((4, 5, 6), [0.48, -0.6, 0.64])):
        X = rng.integers(0, 4, size=shape).astype(np.float32)      # ties that the tilt breaks its own way
        u = np.array(u, np.float32)
        alpha = 0.3
        Y = O.tilt_field(X, u, alpha).astype(np.float64)
        ys = np.unique(Y)
        gaps = np.diff(ys)
        k = np.argsort(gaps)[-6:]                                   # thresholds in the six widest gaps
        tau = np.sort((ys[k] + ys[k + 1]) / 2)
        assert gaps[k].min() > 1e-3
        hard = O.ecc_hard_dir(X[None], u[None], alpha, tau)[0, 0]
        soft = O.soft_fwd(X, u, alpha, tau, 1e5, c=O.coeff_tilted(X, u, alpha))
        assert np.allclose(soft, hard, atol=1e-9)
    # where the coefficient of X itself goes wrong: a constant grid swept against the x axis.
    # Every sublevel set of Y = -x that is not empty is a box (chi = 1), but c_X puts its one
    # nonzero coefficient on the vertex (0, 0), which enters last
    X = np.zeros((3, 3), np.float32)
    u = np.array([-1.0, 0.0], np.float32)
    tau = np.array([-2.5, -1.5, -0.5, 0.5])
    assert O.ecc_hard_dir(X[None], u[None], 1.0, tau)[0, 0].tolist() == [0, 1, 1, 1]
    assert np.allclose(O.soft_fwd(X, u, 1.0, tau, 1e4, c=O.coeff_tilted(X, u, 1.0)), [0, 1, 1, 1], atol=1e-9)
    assert np.allclose(O.soft_fwd(X, u, 1.0, tau, 1e4), [0, 0, 0, 1], atol=1e-9)
