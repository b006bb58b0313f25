"""The flow for small float grids without a range (stage: per-block lists of critical vertices and
value ranges; finish: range, thresholds, histogram and prefix sum in one block per item, or, for
items above 2^16 vertices, several blocks per item and the scan as a third launch) at the edges of
what it takes -- items of 2^16 vertices, 2^18 in the batch, 64 items, 4096 bins, one or two
vertices per thread, lists that are nearly full -- and just beyond them, with the same calls
repeated with the flow switched off."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import ecc_oracle as O
from oracle import ecc_oracle_c as OC
from paper_2510_20271_amd import api, synth
from tests.gpu_util import dev, host

pytestmark = pytest.mark.gpu


def _both(fn):
    a = fn()
    prev = api.ecc_debug_force(api.ECC_FORCE_NO_SMALL)
    try:
        b = fn()
    finally:
        api.ecc_debug_force(prev)
    assert torch.equal(a, b)
    return host(a)


# items of 2^16 vertices and just above (three launches), 2^17 vertices in all (one vertex per thread) and
# more (two), 2^18 in all and just above (not taken), larger items (three launches, 16 blocks per
# item), the largest batch and beyond, 3D
@pytest.mark.parametrize("B,shape", [(1, (256, 256)), (1, (257, 256)), (2, (200, 300)), (3, (256, 255)), (4, (256, 256)),
                                      (5, (230, 230)), (1, (512, 512)), (2, (300, 400)), (1, (500, 524)), (1, (3, 87381)),
                                      (64, (64, 64)), (65, (60, 60)), (64, (1, 1)), (2, (40, 40, 40)),
                                      (1, (64, 64, 64)), (7, (3, 70, 150))])
def test_small_flow_sizes(B, shape):
    nd = len(shape)
    rng = np.random.default_rng(B + shape[-1])
    X = rng.standard_normal((B,) + shape).astype(np.float32)  # white noise: long lists
    got = _both(lambda: api.ecc_hard(dev(X), nd, 100))
    np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, O.thresholds_equal_width(X.min(), X.max(), 100)))
    U = rng.integers(0, 256, size=(B,) + shape, dtype=np.uint8)
    got = _both(lambda: api.ecc_hard(dev(U), nd, 256))
    np.testing.assert_array_equal(got, OC.ecc_hard_batch(U, O.thresholds_levels(256)))


def test_small_flow_nearly_every_vertex_critical():
    # a checkerboard: a vertex is a local minimum (c = 1) or closes cells, except on the border;
    # the stage blocks' lists are full to the last few entries
    y, x = np.mgrid[0:256, 0:256]
    X = ((x + y) % 2).astype(np.float32)[None]
    assert np.mean(OC.coeff(X[0]) != 0) > 0.99
    got = _both(lambda: api.ecc_hard(dev(X), 2, 2))
    np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, O.thresholds_equal_width(0.0, 1.0, 2)))


@pytest.mark.parametrize("shape", [(100, 130), (270, 300)])
@pytest.mark.parametrize("bins", [1, 2, 1023, 1024, 1025, 4096, 4097])
def test_small_flow_bin_counts_and_scan(bins, shape):
    X = np.stack([synth.grf(shape, 1.0, 60 + i) for i in range(3)])
    lo, hi = float(X.min()), float(X.max())
    got = _both(lambda: api.ecc_hard(dev(X), 2, bins))
    np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, O.thresholds_equal_width(lo, hi, bins)))
    got = _both(lambda: api.ecc_hard(dev(X), 2, bins, range=(lo / 2, hi / 2)))
    np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, O.thresholds_equal_width(lo / 2, hi / 2, bins)))
    t = O.thresholds_lower(O.thresholds_equal_width(lo, hi, bins), lo)
    got = _both(lambda: api.ecc_hard(dev(X), 2, bins, superlevel=True))
    np.testing.assert_array_equal(got, O.ecc_super_batch(X, t, False))


def test_small_flow_range_is_the_batch_range():
    # the extremes sit in different items, in vertices that are not critical
    X = np.stack([synth.grf((90, 70), 2.0, 5 + i) for i in range(4)])
    X[1, 40, 30] = X.max() + 3.0   # a peak: enters last, closes cells (critical) ...
    X[3, 0, 0] = X.min() - 2.0     # ... a pit: critical as well
    X[2, 10:13, 10:13] = X.max() + 1.0  # a plateau: its later vertices are not all critical
    got = _both(lambda: api.ecc_hard(dev(X), 2, 77))
    np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, O.thresholds_equal_width(X.min(), X.max(), 77)))


def test_small_flow_static_scratch_and_workspace_reuse():
    X = np.stack([synth.grf((128, 128), 2.0, 15 + i) for i in range(2)])
    want = OC.ecc_hard_batch(X, O.thresholds_equal_width(X.min(), X.max(), 64))
    np.testing.assert_array_equal(host(api.ecc_hard_static(dev(X), 2, 64)), want)
    ws = torch.full((api.ecc_workspace_bytes((128, 128), 2, 64),), 0xff, dtype=torch.uint8, device="cuda")  # garbage
    for _ in range(3):
        np.testing.assert_array_equal(host(api.ecc_hard(dev(X), 2, 64, workspace=ws)), want)


# ---- mid-sized grids: the strip / tube sweep with a list per block, the same finishing kernel --------


@pytest.mark.parametrize("B,shape", [(1, (1024, 1024)), (3, (700, 1300)), (64, (100, 650)), (65, (100, 650)),
                                      (4096, (8, 16)), (4097, (8, 16)), (300, (64, 64)), (1024, (28, 28)), (70, (64, 65)),
                                      (1, (4096, 8192)), (1, (4096, 8200)),
                                      (1, (128, 128, 128)), (2, (60, 200, 300)), (1, (9, 1000, 1000)),
                                      (1, (256, 256, 512)), (1, (256, 256, 520))])
def test_mid_flow_sizes(B, shape):
    nd = len(shape)
    X = np.stack([synth.grf(shape, 2.0, 70 + i) if np.prod(shape) < (1 << 24) else
                  np.tile(synth.grf(tuple(n // 2 for n in shape), 2.0, 70 + i), (2,) * nd) for i in range(min(B, 3))])
    X = X[np.arange(B) % X.shape[0]] + (np.arange(B, dtype=np.float32) * 0.01).reshape((B,) + (1,) * nd)
    X = np.ascontiguousarray(X, dtype=np.float32)
    got = _both(lambda: api.ecc_hard(dev(X), nd, 300))
    np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, O.thresholds_equal_width(X.min(), X.max(), 300)))
    assert np.all(got[:, -1] == 1)


@pytest.mark.parametrize("B,shape", [(2, (1500, 1500)), (2, (100, 120, 250)), (70, (200, 300)), (200, (60, 60))])
def test_mid_flow_white_noise_fills_the_lists(B, shape):
    # 60 % of the vertices are critical: far beyond the room of the shared lists of the large-input flow
    # (the two batches of many small items are finished by one block per item, prefix sum included)
    X = np.random.default_rng(9).standard_normal((B,) + shape).astype(np.float32)
    for kw in ({}, {"top": True}, {"superlevel": True}):
        got = _both(lambda: api.ecc_hard(dev(X), len(shape), 129, **kw))
        lo, hi = float(X.min()), float(X.max())
        if kw.get("superlevel"):
            want = O.ecc_super_batch(X, O.thresholds_lower(O.thresholds_equal_width(lo, hi, 129), lo), False)
        elif kw.get("top"):
            want = np.stack([O.ecc_top(x, O.thresholds_equal_width(lo, hi, 129)) for x in X])
        else:
            want = OC.ecc_hard_batch(X, O.thresholds_equal_width(lo, hi, 129))
        np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("bins", [1, 4096, 4097])
def test_mid_flow_bins_half_precision_and_static_scratch(bins):
    X = np.stack([synth.grf((900, 1100), 2.0, 80 + i) for i in range(2)])
    H = X.astype(np.float16)
    want = OC.ecc_hard_batch(H.astype(np.float32), O.thresholds_equal_width(float(H.min()), float(H.max()), bins))
    got = _both(lambda: api.ecc_hard(dev(H), 2, bins))
    np.testing.assert_array_equal(got, want)
    want = OC.ecc_hard_batch(X, O.thresholds_equal_width(X.min(), X.max(), bins))
    np.testing.assert_array_equal(host(api.ecc_hard_static(dev(X), 2, bins)), want)
    # a batch whose lists per block do not fit the static scratch goes through the shared lists there
    Y = np.stack([synth.grf((1500, 2000), 2.0, 90 + i) for i in range(2)])
    assert api.ecc_workspace_bytes((1500, 2000), 2, bins) > 32 << 20
    np.testing.assert_array_equal(host(api.ecc_hard_static(dev(Y), 2, bins)),
                                  OC.ecc_hard_batch(Y, O.thresholds_equal_width(Y.min(), Y.max(), bins)))
