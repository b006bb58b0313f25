"""Randomised parity sweep: random shapes, dtypes, batch sizes, bin counts and threshold modes
through every hard entry point and convention, each compared bit for bit with the CPU oracle.  The cases are
drawn from a fixed seed, so a failure names its case."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import ecc_oracle as O
from oracle import ecc_oracle_c as OC
from paper_2510_20271_amd import api
from tests.gpu_util import dev, host

pytestmark = pytest.mark.gpu


def _case(seed):
    rng = np.random.default_rng(seed)
    nd = int(rng.integers(2, 4))
    if nd == 2:
        shape = (int(rng.integers(1, 400)), int(rng.choice([1, 3, 7, 8, 9, 63, 64, 65, 247, 248, 249, 256, 500, 1000, 1303])))
    else:
        shape = (int(rng.integers(1, 40)), int(rng.integers(1, 90)), int(rng.choice([1, 5, 8, 9, 61, 62, 63, 64, 124, 130, 257])))
    batch = int(rng.integers(1, 4))
    dtype = [np.uint8, np.uint16, np.float32][int(rng.integers(0, 3))]
    levels = int(rng.choice([2, 5, 40, 250]))
    bins = int(rng.choice([1, 2, 17, 300, 5000]))
    smooth = bool(rng.integers(0, 2))
    if dtype == np.float32:
        X = rng.standard_normal((batch,) + shape).astype(np.float32)
        if smooth:  # cumulative sums: long monotone runs, few critical vertices
            X = np.cumsum(X, axis=-1).astype(np.float32) / 8
        else:      # few distinct values: ties everywhere, signed zeros
            X = np.round(X * 2).astype(np.float32) / 2
            X[X == 0] = rng.choice([0.0, -0.0], size=int((X == 0).sum())).astype(np.float32)
    else:
        X = rng.integers(0, levels, size=(batch,) + shape, dtype=dtype)
    mode = ["auto", "range"][int(rng.integers(0, 2))]
    return nd, shape, batch, X, bins, mode, rng


@pytest.mark.parametrize("seed", range(60))
def test_random_case(seed):
    nd, shape, batch, X, bins, mode, rng = _case(seed)
    is_float = X.dtype == np.float32
    if mode == "range" or is_float:
        lo, hi = float(X.min()), float(X.max())
        if mode == "range" and rng.integers(0, 2):
            lo, hi = lo + 0.25 * (hi - lo), hi - 0.1 * (hi - lo)  # values fall outside on both sides
        t = O.thresholds_equal_width(lo, hi, bins)
        rng_arg = (lo, hi) if mode == "range" else None
    else:
        t, rng_arg = O.thresholds_levels(bins), None
    info = f"seed {seed} shape {shape} batch {batch} dtype {X.dtype} bins {bins} mode {mode}"
    got = host(api.ecc_hard(dev(X), nd, bins, range=rng_arg))
    np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, t), err_msg=info)
    got = host(api.ecc_hard_top(dev(X), nd, bins, range=rng_arg))
    np.testing.assert_array_equal(got, O.ecc_top_batch(X, t), err_msg="top " + info)
    # superlevel sets, both constructions: lower edges of the same bins
    if mode == "range" or is_float:
        ts = O.thresholds_lower(t, lo)
    else:
        ts = O.thresholds_levels_super(bins)
    for top in (False, True):
        got = host(api.ecc_hard(dev(X), nd, bins, range=rng_arg, top=top, superlevel=True))
        np.testing.assert_array_equal(got, O.ecc_super_batch(X, ts, top), err_msg=f"super top={top} " + info)
    if is_float:
        U = rng.standard_normal((2, nd)).astype(np.float32)
        alpha = float(rng.choice([0.0, 0.01, 0.5]))
        ys = [[O.tilt_field(x, u, alpha) for x in X] for u in U]
        if mode == "range":
            td, ra = t, rng_arg
        else:
            lo = min(y.min() for r in ys for y in r)
            hi = max(y.max() for r in ys for y in r)
            td, ra = O.thresholds_equal_width(lo, hi, bins), None
        want = np.stack([OC.ecc_hard_batch(np.stack(r), td) for r in ys])
        got = host(api.ecc_hard_dir(dev(X), nd, dev(U), alpha, bins, range=ra))
        np.testing.assert_array_equal(got, want, err_msg="dir " + info)
