"""GPU parity of the superlevel curves (ecc_hard_ex) against the CPU oracle: bit-exact int64
curves through the C ABI, both constructions, on both sides of the line between the
one-thread-per-vertex sweep and the strip / tube sweeps, with ties, for every dtype and
threshold mode; and the sublevel combinations of ecc_hard_ex against ecc_hard / ecc_hard_top."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import ecc_oracle as O
from paper_2510_20271_amd import api, synth
from tests.gpu_util import dev, host

pytestmark = pytest.mark.gpu

SHAPES = [(1, 1), (1, 9), (9, 1), (3, 3), (17, 65), (130, 257), (257, 259), (9, 7300), (300, 1000),
          (2, 2, 2), (1, 5, 9), (5, 1, 9), (5, 9, 1), (9, 17, 33), (20, 31, 65), (33, 70, 130), (4, 9, 300),
          (67, 9, 131)]


@pytest.mark.parametrize("top", [False, True])
@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("dtype", [np.uint8, np.uint16])
def test_super_levels(shape, dtype, top, flow):
    rng = np.random.default_rng(31)
    X = rng.integers(0, 13, size=(2,) + shape, dtype=dtype)
    got = host(api.ecc_hard(dev(X), len(shape), 11, top=top, superlevel=True))  # levels 11, 12 count as X >= 10
    want = O.ecc_super_batch(X, O.thresholds_levels_super(11), top)
    np.testing.assert_array_equal(got, want)
    assert np.all(want[:, 0] == 1)  # X >= 0: the whole grid
    # with a range: lower edges of 7 bins over [2, 9.5], values outside on both sides
    t = O.thresholds_lower(O.thresholds_equal_width(2.0, 9.5, 7), 2.0)
    got = host(api.ecc_hard(dev(X), len(shape), 7, range=(2.0, 9.5), top=top, superlevel=True))
    np.testing.assert_array_equal(got, O.ecc_super_batch(X, t, top))


@pytest.mark.parametrize("top", [False, True])
@pytest.mark.parametrize("shape", SHAPES)
def test_super_float(shape, top, flow):
    rng = np.random.default_rng(37)
    X = (rng.integers(-6, 7, size=(2,) + shape) / 4).astype(np.float32)
    X[X == 0] = rng.choice([0.0, -0.0], size=int((X == 0).sum())).astype(np.float32)
    lo, hi = float(X.min()), float(X.max())
    t = O.thresholds_lower(O.thresholds_equal_width(lo, hi, 23), lo)
    want = O.ecc_super_batch(X, t, top)
    np.testing.assert_array_equal(host(api.ecc_hard(dev(X), len(shape), 23, top=top, superlevel=True)), want)
    np.testing.assert_array_equal(
        host(api.ecc_hard(dev(X), len(shape), 23, range=(lo, hi), top=top, superlevel=True)), want)
    assert np.all(want[:, 0] == 1)


@pytest.mark.parametrize("top", [False, True])
def test_super_smooth_fields(top, flow):
    X = np.stack([synth.grf((200, 520), 3.0, 5 + i) for i in range(2)])
    lo, hi = float(X.min()), float(X.max())
    t = O.thresholds_lower(O.thresholds_equal_width(lo, hi, 200), lo)
    want = O.ecc_super_batch(X, t, top)
    np.testing.assert_array_equal(host(api.ecc_hard(dev(X), 2, 200, top=top, superlevel=True)), want)
    if top:  # one layer of cubes is the same complex as the squares
        np.testing.assert_array_equal(host(api.ecc_hard(dev(X[:, None]), 3, 200, top=True, superlevel=True)), want)
    V = synth.grf((40, 72, 130), 2.0, 8)[None]
    lo, hi = float(V.min()), float(V.max())
    t = O.thresholds_lower(O.thresholds_equal_width(lo, hi, 100), lo)
    np.testing.assert_array_equal(host(api.ecc_hard(dev(V), 3, 100, top=top, superlevel=True)),
                                  O.ecc_super_batch(V, t, top))
    # a range that cuts both tails, 1 bin and many bins
    for bins in (1, 4000):
        t = O.thresholds_lower(O.thresholds_equal_width(-1.0, 0.5, bins), -1.0)
        np.testing.assert_array_equal(
            host(api.ecc_hard(dev(V), 3, bins, range=(-1.0, 0.5), top=top, superlevel=True)),
            O.ecc_super_batch(V, t, top))


def test_super_overflowing_lists_fall_back(flow):
    # i.i.d. float grids: most vertices are critical, the single-pass lists overflow
    rng = np.random.default_rng(41)
    for shape in ((300, 700), (30, 64, 130)):
        X = rng.standard_normal((1,) + shape).astype(np.float32)
        lo, hi = float(X.min()), float(X.max())
        t = O.thresholds_lower(O.thresholds_equal_width(lo, hi, 64), lo)
        for top in (False, True):
            np.testing.assert_array_equal(host(api.ecc_hard(dev(X), len(shape), 64, top=top, superlevel=True)),
                                          O.ecc_super_batch(X, t, top))


def test_ex_sublevel_is_ecc_hard_and_ecc_hard_top():
    X = np.stack([synth.grf((130, 300), 2.0, 3 + i) for i in range(2)])
    a = host(api.ecc_hard_ex(dev(X), 2, api.ECC_VERTEX, api.ECC_SUBLEVEL, 50))
    np.testing.assert_array_equal(a, host(api.ecc_hard(dev(X), 2, 50)))
    b = host(api.ecc_hard_ex(dev(X), 2, api.ECC_TOPCELL, api.ECC_SUBLEVEL, 50))
    np.testing.assert_array_equal(b, host(api.ecc_hard_top(dev(X), 2, 50)))


def test_super_peaks(flow):
    # three isolated peaks: the superlevel curve counts them, the sublevel curve never does
    X = np.zeros((1, 5, 5), np.uint8)
    X[0, 1, 1] = X[0, 3, 3] = 5
    X[0, 1, 3] = 4
    got = host(api.ecc_hard(dev(X), 2, 6, superlevel=True))
    assert got.tolist() == [[1, 3, 3, 3, 3, 2]]
