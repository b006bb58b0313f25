"""GPU parity of the directional hard curves (tilted filtration) against the CPU oracle:
bit-exact int64 curves through the C ABI.  The oracle forms the tilted field in float32 with
the operation order the header fixes and takes its hard ECC."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import ecc_oracle as O
from oracle import ecc_oracle_c as OC
from paper_2510_20271_amd import api, synth
from tests.gpu_util import dev, host

pytestmark = pytest.mark.gpu

SHAPES = [(1, 1), (3, 5), (7, 64), (40, 50), (130, 257), (257, 259), (300, 1000), (2, 2, 2), (1, 9, 40), (3, 4, 5),
          (9, 17, 33), (20, 31, 65), (33, 70, 130), (4, 9, 300), (70, 9, 131)]


def _oracle(Xb, U, alpha, t):
    return np.stack([OC.ecc_hard_batch(np.stack([O.tilt_field(x, u, alpha) for x in Xb]), t) for u in U])


def _range(Xb, U, alpha):
    ys = [O.tilt_field(x, u, alpha) for x in Xb for u in U]
    return min(y.min() for y in ys), max(y.max() for y in ys)


@pytest.mark.parametrize("shape", SHAPES)
def test_directional_curves_match_the_oracle(shape, flow):
    nd = len(shape)
    rng = np.random.default_rng(41)
    B, K, bins, alpha = 2, 3, 29, 0.37
    # few distinct values plus a tilt that is often an exact float: ties survive the tilt
    Xb = (rng.integers(-4, 5, size=(B,) + shape) / 4).astype(np.float32)
    U = rng.standard_normal((K, nd)).astype(np.float32)
    U[0] = 0.0
    U[0, 0] = 1.0  # axis direction: whole columns tie
    lo, hi = _range(Xb, U, alpha)
    want = _oracle(Xb, U, alpha, O.thresholds_equal_width(lo, hi, bins))
    got = host(api.ecc_hard_dir(dev(Xb), nd, dev(U), alpha, bins))
    np.testing.assert_array_equal(got, want)
    got = host(api.ecc_hard_dir(dev(Xb), nd, dev(U), alpha, bins, range=(float(lo), float(hi))))
    np.testing.assert_array_equal(got, want)
    assert np.all(got[..., -1] == 1)


def test_zero_alpha_gives_the_plain_curves_for_every_direction(flow):
    X = np.stack([synth.grf((90, 300), 2.0, 3 + i) for i in range(2)])
    U = np.array([[1.0, 0.0], [0.6, -0.8]], np.float32)
    got = host(api.ecc_hard_dir(dev(X), 2, dev(U), 0.0, 64))
    plain = host(api.ecc_hard(dev(X), 2, 64))
    np.testing.assert_array_equal(got[0], plain)
    np.testing.assert_array_equal(got[1], plain)


@pytest.mark.parametrize("shape", [(1024, 1024), (96, 128, 160)])
def test_directional_curves_of_smooth_fields(shape, flow):
    nd = len(shape)
    X = synth.grf(shape, 3.0, 77)[None]
    th = np.linspace(0.0, np.pi, 5, endpoint=False)
    U = (np.stack([np.cos(th), np.sin(th)], 1) if nd == 2 else
         np.stack([np.cos(th) * 0.8, np.sin(th) * 0.8, np.full_like(th, 0.6)], 1)).astype(np.float32)
    alpha = 0.002
    lo, hi = _range(X, U, alpha)
    want = _oracle(X, U, alpha, O.thresholds_equal_width(lo, hi, 256))
    got = host(api.ecc_hard_dir(dev(X), nd, dev(U), alpha, 256))
    np.testing.assert_array_equal(got, want)
