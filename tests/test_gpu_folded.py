"""Launches large enough for the 3D sweep to fold its narrow last strip (several row groups
side by side in one wave): every sink and mode of the tube sweep on such shapes, bit-exact
(hard curves) or within tolerance (soft path) against the CPU oracle.  Widths are chosen for
different fold geometries: 136 -> 12 columns left over (4 folds), 70 -> 8 (6 folds),
66 -> 4 (8 folds), 20 -> a single strip of 20 (2 folds); the heights leave ragged row groups."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import ecc_oracle as O
from oracle import ecc_oracle_c as OC
from paper_2510_20271_amd import api, synth
from tests.gpu_util import dev, host
from tests.test_gpu_soft import _close, _close_sum

pytestmark = pytest.mark.gpu

# (batch, D, H, W): strips * row groups * batch * D >= 160000 turns the folding on
BIG = [(6, 200, 202, 136), (8, 200, 202, 70), (9, 190, 199, 66), (16, 200, 203, 20)]


def _smooth(batch, shape, seed):
    # one smooth field, shifted per item: cheap to make, few critical vertices, ties at the seams
    base = synth.grf(shape, 2.0, seed)
    return np.stack([np.roll(base, 7 * i, axis=2) + np.float32(0.01 * i) for i in range(batch)])


@pytest.mark.parametrize("b,D,H,W", BIG)
def test_folded_float_single_pass_and_range(b, D, H, W):
    X = _smooth(b, (D, H, W), 300 + W)
    lo, hi = float(X.min()), float(X.max())
    t = O.thresholds_equal_width(lo, hi, 300)
    want = OC.ecc_hard_batch(X, t)
    g = dev(X)
    np.testing.assert_array_equal(host(api.ecc_hard(g, 3, 300)), want)                    # list sweep
    np.testing.assert_array_equal(host(api.ecc_hard(g, 3, 300, range=(lo, hi))), want)    # histogram sweep


@pytest.mark.parametrize("dtype,levels", [(np.uint8, 200), (np.uint16, 3000)])
def test_folded_integer_levels(dtype, levels):
    b, D, H, W = BIG[1]
    rng = np.random.default_rng(7)
    X = rng.integers(0, levels, size=(b, D, H, W), dtype=dtype)  # i.i.d.: most vertices critical
    got = host(api.ecc_hard(dev(X), 3, levels))
    np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, O.thresholds_levels(levels)))


def test_folded_conventions_and_directions():
    b, D, H, W = 2, 200, 202, 136
    X = _smooth(b, (D, H, W), 411)
    # the folding depends on the whole launch: pad the batch so that it is on, check two items
    Xb = np.concatenate([X, np.repeat(X[:1], 4, axis=0)])
    lo, hi = float(Xb.min()), float(Xb.max())
    t = O.thresholds_equal_width(lo, hi, 64)
    ts = O.thresholds_lower(t, lo)
    g = dev(Xb)
    np.testing.assert_array_equal(host(api.ecc_hard(g, 3, 64, top=True))[:b], O.ecc_top_batch(X, t))
    np.testing.assert_array_equal(host(api.ecc_hard(g, 3, 64, superlevel=True))[:b], O.ecc_super_batch(X, ts))
    np.testing.assert_array_equal(host(api.ecc_hard(g, 3, 64, top=True, superlevel=True))[:b],
                                  O.ecc_super_batch(X, ts, True))
    U = np.array([[0.6, 0.0, 0.8], [-0.48, 0.64, 0.6], [0.0, -1.0, 0.0]], np.float32)
    got = host(api.ecc_hard_dir(dev(X), 3, dev(U), 0.003, 64))   # 3 directions x 2 items: folded as well
    ys = [[O.tilt_field(x, u, 0.003) for x in X] for u in U]
    lo = min(y.min() for r in ys for y in r)
    hi = max(y.max() for r in ys for y in r)
    td = O.thresholds_equal_width(lo, hi, 64)
    np.testing.assert_array_equal(got, np.stack([OC.ecc_hard_batch(np.stack(r), td) for r in ys]))


def test_folded_soft_forward_backward():
    b, D, H, W = 8, 200, 202, 70
    X = _smooth(b, (D, H, W), 512)
    T = 5
    tau = np.linspace(X.min(), X.max() + 0.5, T).astype(np.float32)
    u = np.array([0.48, -0.6, 0.64], np.float32)
    G = np.random.default_rng(2).standard_normal((b, T)).astype(np.float32)
    g, ud, td = dev(X), dev(u), dev(tau)
    chi = host(api.ecc_soft_fwd(g, 3, ud, 0.004, td, 9.0))
    gx, dt, du = (host(a) for a in api.ecc_soft_bwd(g, 3, ud, 0.004, td, 9.0, grad_chi=dev(G)))
    for i in (0, b - 1):
        _close_sum(chi[i], O.soft_fwd(X[i], u, 0.004, tau, 9.0), 1e-4, f"chi[{i}]")
        rgx, rdt, rdu = O.soft_bwd(X[i], u, 0.004, tau, 9.0, G[i])
        _close(gx[i], rgx, 1e-3, f"grad_X[{i}]")
        _close_sum(dt[i], rdt, 1e-3, f"dchi_dtau[{i}]")
        _close_sum(du[i], rdu, 1e-3, f"dchi_du[{i}]")
