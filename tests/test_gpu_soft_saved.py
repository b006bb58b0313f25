"""ecc_soft_fwd_save / ecc_soft_bwd_saved (the forward pass keeps its critical vertices for the
backward pass) against the float64 oracle and against the stateless pair, through the C ABI."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import ecc_oracle as O
from paper_2510_20271_amd import api, synth
from tests.gpu_util import dev, host
from tests.test_gpu_soft import _close, _close_sum

pytestmark = pytest.mark.gpu


def _case(Xb, u, alpha, tau, lam, G, tilted=False, state=None, tau_bwd=None, lam_bwd=None):
    nd = Xb.ndim - 1
    g, ud, td = dev(Xb), dev(u), dev(tau)
    chi, dt, du, state = api.ecc_soft_fwd_save(g, nd, ud, alpha, td, lam, tilted_c=tilted, state=state)
    # chi is the forward kernel's own, bit for bit
    assert torch.equal(chi, api.ecc_soft_fwd(g, nd, ud, alpha, td, lam, tilted_c=tilted))
    tb = tau if tau_bwd is None else tau_bwd
    lb = lam if lam_bwd is None else lam_bwd
    gx = api.ecc_soft_bwd_saved(g, nd, ud, alpha, dev(tb), lb, state, grad_chi=None if G is None else dev(G),
                                tilted_c=tilted)
    chi, dt, du, gx = host(chi), host(dt), host(du), host(gx)
    for i, X in enumerate(Xb):
        c = O.coeff_tilted(X, u, alpha) if tilted else O.coeff(X)
        _close_sum(chi[i], O.soft_fwd(X, u, alpha, tau, lam, c=c), 1e-4, f"chi[{i}]")
        _, rdt, rdu = O.soft_bwd(X, u, alpha, tau, lam, None if G is None else G[i], c=c)
        _close_sum(dt[i], rdt, 1e-3, f"dchi_dtau[{i}]")
        _close_sum(du[i], rdu, 1e-3, f"dchi_du[{i}]")
        rgx, _, _ = O.soft_bwd(X, u, alpha, tb, lb, None if G is None else G[i], c=c)
        _close(gx[i], rgx, 1e-3, f"grad_X[{i}]")
        assert not np.any((gx[i] != 0) & (c == 0))
    return state


@pytest.mark.parametrize("shape", [(1, 9), (9, 1), (7, 13), (64, 64), (100, 259), (45, 1024), (130, 600), (3, 5000)])
def test_saved_state_2d_shapes(shape):
    B, T = 3, 9
    Xb = np.stack([synth.grf(shape, 1.5, 40 + i) if min(shape) > 1 else
                   np.random.default_rng(i).standard_normal(shape).astype(np.float32) for i in range(B)])
    tau = np.linspace(Xb.min() - 0.1, Xb.max() + 0.5, T).astype(np.float32)
    u = np.array([np.cos(0.3), np.sin(0.3)], np.float32)
    G = np.random.default_rng(1).standard_normal((B, T)).astype(np.float32)
    _case(Xb, u, np.float32(0.01), tau, np.float32(20.0), G)


@pytest.mark.parametrize("T", [1, 64, 65, 256])
def test_saved_state_threshold_counts_and_tilted(T):
    B = 2
    Xb = np.stack([np.round(synth.grf((90, 300), 2.0, 7 + i) * 40) / 8 for i in range(B)]).astype(np.float32)
    u = np.array([-0.8, 0.6], np.float32)
    G = np.random.default_rng(T).standard_normal((B, T)).astype(np.float32)
    for tilted in (False, True):
        Y = np.stack([O.tilt_field(x, u, np.float32(0.03)) for x in Xb])
        tau = np.linspace(Y.min() - 0.1, Y.max() + 0.2, T).astype(np.float32)
        _case(Xb, u, np.float32(0.03), tau, np.float32(9.0), G, tilted=tilted)


def test_saved_state_other_thresholds_in_backward_and_no_upstream():
    Xb = synth.grf_batch(2, (70, 260), 1.5, 5)
    u = np.array([0.6, 0.8], np.float32)
    tau = np.linspace(Xb.min(), Xb.max() + 2.0, 12).astype(np.float32)
    _case(Xb, u, np.float32(0.01), tau, np.float32(20.0), None, tau_bwd=(tau[::-1] * 0.9).astype(np.float32).copy()[:7],
          lam_bwd=np.float32(11.0))


def test_saved_state_overflow_falls_back_per_item():
    # item 0 smooth, item 1 white noise (more than one vertex in eight has c != 0: its lists overflow)
    shape = (64, 520)
    Xb = np.stack([synth.grf(shape, 2.0, 3), np.random.default_rng(4).standard_normal(shape).astype(np.float32),
                   synth.grf(shape, 2.0, 5)])
    tau = np.linspace(-2, 3, 10).astype(np.float32)
    u = np.array([0.28, 0.96], np.float32)
    G = np.random.default_rng(2).standard_normal((3, 10)).astype(np.float32)
    state = _case(Xb, u, np.float32(0.004), tau, np.float32(5.0), G)
    # the overflow word of an item holds the state's generation when one of its units ran out of room
    gen = int(host(state[128:132]).view(np.uint32)[0])
    flags = host(state[256:256 + 12]).view(np.uint32)
    assert [int(f) == gen for f in flags] == [False, True, False]


def test_saved_state_of_another_shape_is_noticed():
    big = torch.empty(api.ecc_soft_state_bytes((300, 520), 2), dtype=torch.uint8, device="cuda")
    u = np.array([1.0, 0.0], np.float32)
    Xa = synth.grf_batch(2, (300, 520), 2.0, 8)
    tau = np.linspace(-0.5, 1.5, 6).astype(np.float32)
    _case(Xa, u, np.float32(0.002), tau, np.float32(12.0), None, state=big)
    # the same buffer, now holding the state of the 300 x 520 batch, handed to a backward call of another shape
    Xb = synth.grf_batch(2, (100, 520), 2.0, 9)
    gx = host(api.ecc_soft_bwd_saved(dev(Xb), 2, dev(u), 0.002, dev(tau), 12.0, big))
    ref = O.soft_bwd_batch(Xb, u, 0.002, tau, 12.0, None)[0]
    for i in range(2):
        _close(gx[i], ref[i], 1e-3, f"grad_X[{i}]")


@pytest.mark.parametrize("shape,T", [((9, 30, 7), 5), ((60, 70), 300), ((9, 30, 70), 300)])
def test_saved_state_entry_points_on_shapes_without_state(shape, T):
    # volumes narrower than 8 and T > 256 keep no state: the same entry points run the stateless kernels
    nd = len(shape)
    Xb = np.stack([synth.grf(shape, 1.5, 60 + i) for i in range(2)])
    u = np.array([0.6, 0.8] if nd == 2 else [0.48, -0.6, 0.64], np.float32)
    tau = np.linspace(Xb.min(), Xb.max() + 1.0, T).astype(np.float32)
    G = np.random.default_rng(3).standard_normal((2, T)).astype(np.float32)
    _case(Xb, u, np.float32(0.02), tau, np.float32(8.0), G)


def test_saved_state_is_deterministic_and_config_c5():
    Xb = synth.config_c5()
    p = synth.soft_params_c5(Xb)
    G = synth.upstream_grad(Xb.shape[0], len(p["tau"]))
    g, ud, td, Gd = dev(Xb), dev(p["u"]), dev(p["tau"]), dev(G)
    a = api.ecc_soft_fwd_save(g, 2, ud, p["alpha"], td, p["lam"])
    b = api.ecc_soft_fwd_save(g, 2, ud, p["alpha"], td, p["lam"])
    for x, y in zip(a[:3], b[:3]):
        assert torch.equal(x, y)
    ga = api.ecc_soft_bwd_saved(g, 2, ud, p["alpha"], td, p["lam"], a[3], grad_chi=Gd)
    gb = api.ecc_soft_bwd_saved(g, 2, ud, p["alpha"], td, p["lam"], b[3], grad_chi=Gd)
    assert torch.equal(ga, gb)
    rgx, rdt, rdu = O.soft_bwd_batch(Xb, p["u"], p["alpha"], p["tau"], p["lam"], G)
    rchi = O.soft_fwd_batch(Xb, p["u"], p["alpha"], p["tau"], p["lam"])
    chi, dt, du, gx = host(a[0]), host(a[1]), host(a[2]), host(ga)
    for i in range(Xb.shape[0]):
        _close_sum(chi[i], rchi[i], 1e-4, f"chi[{i}]")
        _close_sum(dt[i], rdt[i], 1e-3, f"dchi_dtau[{i}]")
        _close_sum(du[i], rdu[i], 1e-3, f"dchi_du[{i}]")
        _close(gx[i], rgx[i], 1e-3, f"grad_X[{i}]")


# ---- volumes: the tube sweep keeps its critical vertices the same way ---------------------------


@pytest.mark.parametrize("shape", [(2, 2, 8), (5, 6, 9), (9, 30, 70), (40, 33, 129), (70, 20, 64), (3, 131, 200)])
def test_saved_state_3d_shapes(shape):
    B, T = 2, 9
    Xb = np.stack([synth.grf(shape, 1.0, 50 + i) for i in range(B)])
    tau = np.linspace(Xb.min() - 0.1, Xb.max() + 0.5, T).astype(np.float32)
    u = np.array([0.48, -0.6, 0.64], np.float32)
    G = np.random.default_rng(2).standard_normal((B, T)).astype(np.float32)
    _case(Xb, u, np.float32(0.02), tau, np.float32(8.0), G)


@pytest.mark.parametrize("T", [1, 64, 65, 256])
def test_saved_state_3d_threshold_counts_tilted_and_quantised(T):
    B = 2
    Xb = np.stack([np.round(synth.grf((20, 40, 130), 2.0, 7 + i) * 40) / 8 for i in range(B)]).astype(np.float32)
    u = np.array([-0.8, 0.0, 0.6], np.float32)
    G = np.random.default_rng(T).standard_normal((B, T)).astype(np.float32)
    for tilted in (False, True):
        Y = np.stack([O.tilt_field(x, u, np.float32(0.03)) for x in Xb])
        tau = np.linspace(Y.min() - 0.1, Y.max() + 0.2, T).astype(np.float32)
        _case(Xb, u, np.float32(0.03), tau, np.float32(9.0), G, tilted=tilted)


def test_saved_state_3d_overflow_other_thresholds_and_reuse():
    # item 1 is white noise: its lists overflow and its grad_X comes from the grid
    shape = (30, 24, 130)
    Xb = np.stack([synth.grf(shape, 2.0, 3), np.random.default_rng(4).standard_normal(shape).astype(np.float32),
                   synth.grf(shape, 2.0, 5)])
    tau = np.linspace(-2, 3, 10).astype(np.float32)
    u = np.array([0.28, 0.0, 0.96], np.float32)
    G = np.random.default_rng(2).standard_normal((3, 10)).astype(np.float32)
    state = _case(Xb, u, np.float32(0.004), tau, np.float32(5.0), None,
                  tau_bwd=(tau[::-1] * 0.9).astype(np.float32).copy()[:7], lam_bwd=np.float32(7.0))
    gen = int(host(state[128:132]).view(np.uint32)[0])
    flags = host(state[256:256 + 12]).view(np.uint32)
    assert [int(f) == gen for f in flags] == [False, True, False]
    # the same buffer again (its generation moves on), then handed to a backward call of another shape
    _case(Xb[::-1].copy(), u, np.float32(0.004), tau, np.float32(5.0), G, state=state)
    Xc = np.stack([synth.grf((30, 24, 66), 2.0, 9 + i) for i in range(3)])
    big = torch.empty(max(state.numel(), api.ecc_soft_state_bytes((30, 24, 66), 3)), dtype=torch.uint8, device="cuda")
    big[:state.numel()] = state
    gx = host(api.ecc_soft_bwd_saved(dev(Xc), 3, dev(u), 0.004, dev(tau), 5.0, big))
    ref = O.soft_bwd_batch(Xc, u, 0.004, tau, 5.0, None)[0]
    for i in range(3):
        _close(gx[i], ref[i], 1e-3, f"grad_X[{i}]")


def test_saved_state_3d_is_deterministic_and_agrees_with_the_stateless_pass():
    Xb = np.stack([synth.grf((48, 50, 70), 1.5, 21 + i) for i in range(2)])
    u = np.array([0.48, -0.6, 0.64], np.float32)
    tau = np.linspace(Xb.min(), Xb.max(), 33).astype(np.float32)
    g, ud, td = dev(Xb), dev(u), dev(tau)
    a = api.ecc_soft_fwd_save(g, 3, ud, 0.01, td, 20.0)
    b = api.ecc_soft_fwd_save(g, 3, ud, 0.01, td, 20.0)
    for x, y in zip(a[:3], b[:3]):
        assert torch.equal(x, y)
    assert torch.equal(api.ecc_soft_bwd_saved(g, 3, ud, 0.01, td, 20.0, a[3]),
                       api.ecc_soft_bwd_saved(g, 3, ud, 0.01, td, 20.0, b[3]))
    # the stateless backward pass gives the same grad_X (same arithmetic per vertex, other kernels)
    ref = api.ecc_soft_bwd(g, 3, ud, 0.01, td, 20.0)[0]
    got = api.ecc_soft_bwd_saved(g, 3, ud, 0.01, td, 20.0, a[3])
    for i in range(2):
        _close(host(got)[i], host(ref)[i], 1e-3, "grad_X")
