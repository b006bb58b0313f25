"""GPU parity of the top-cell construction (ecc_hard_top) against the CPU oracle: bit-exact
int64 curves through the C ABI, on both sides of the line between the one-thread-per-vertex
sweep and the strip / tube sweeps, with ties, for every dtype and threshold mode."""
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


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("dtype", [np.uint8, np.uint16])
def test_top_levels(shape, dtype, flow):
    rng = np.random.default_rng(23)
    X = rng.integers(0, 13, size=(2,) + shape, dtype=dtype)
    got = host(api.ecc_hard_top(dev(X), len(shape), 11))  # the two top levels fall above the last threshold
    np.testing.assert_array_equal(got, O.ecc_top_batch(X, O.thresholds_levels(11)))


@pytest.mark.parametrize("shape", SHAPES)
def test_top_float(shape, flow):
    rng = np.random.default_rng(29)
    X = (rng.integers(-6, 7, size=(2,) + shape) / 4).astype(np.float32)
    X[X == 0] = rng.choice([0.0, -0.0], size=int((X == 0).sum())).astype(np.float32)
    t = O.thresholds_equal_width(X.min(), X.max(), 23)
    want = O.ecc_top_batch(X, t)
    np.testing.assert_array_equal(host(api.ecc_hard_top(dev(X), len(shape), 23)), want)
    np.testing.assert_array_equal(
        host(api.ecc_hard_top(dev(X), len(shape), 23, range=(float(X.min()), float(X.max())))), want)
    assert np.all(want[:, -1] == 1)


def test_top_smooth_fields_and_depth_one(flow):
    X = np.stack([synth.grf((200, 520), 3.0, 5 + i) for i in range(2)])
    t = O.thresholds_equal_width(X.min(), X.max(), 200)
    want = O.ecc_top_batch(X, t)
    np.testing.assert_array_equal(host(api.ecc_hard_top(dev(X), 2, 200)), want)
    np.testing.assert_array_equal(host(api.ecc_hard_top(dev(X[:, None]), 3, 200)), want)  # one layer of cubes
    V = synth.grf((40, 72, 130), 2.0, 8)[None]
    t = O.thresholds_equal_width(V.min(), V.max(), 100)
    np.testing.assert_array_equal(host(api.ecc_hard_top(dev(V), 3, 100)), O.ecc_top_batch(V, t))


def test_top_differs_from_the_vertex_construction_where_it_should():
    # two squares touching in a corner: one component here, two for ecc_hard
    X = np.array([[[0, 1], [1, 0]]], np.uint8)
    assert host(api.ecc_hard_top(dev(X), 2, 2)).tolist() == [[1, 1]]
    assert host(api.ecc_hard(dev(X), 2, 2)).tolist() == [[2, 1]]
