"""GPU parity of the hard ECC path against the CPU oracle: bit-exact int64
curves and coefficient maps, through the C ABI (ctypes binding)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import ecc_oracle as O
from oracle import ecc_oracle_c as OC
from paper_2510_20271_amd import api, synth
from tests.gpu_util import dev, host

pytestmark = pytest.mark.gpu

# (small inputs take a two-launch flow of their own, see the `flow` fixture; with that flow off and
# the thresholds known up front, inputs of up to 2^16 vertices take the one-thread-per-vertex sweep,
# larger ones the strip / tube sweeps: both sides of either line are covered)
SHAPES_2D = [(1, 1), (1, 7), (7, 1), (2, 2), (3, 3), (5, 64), (64, 5), (17, 65), (63, 129), (130, 257),
             (256, 256), (257, 259), (9, 7300), (300, 1000)]
SHAPES_3D = [(1, 1, 1), (2, 2, 2), (1, 5, 9), (5, 1, 9), (5, 9, 1), (3, 4, 5), (9, 17, 33), (8, 64, 64),
             (20, 31, 65), (33, 70, 130), (4, 9, 300), (2, 129, 257), (67, 9, 131), (31, 300, 9)]


def _rand(shape, dtype, seed, levels=6):
    rng = np.random.default_rng(seed)
    if dtype == np.float32:
        # few distinct values -> many exact ties, plus signed zeros
        v = rng.integers(-levels, levels, size=shape).astype(np.float32) / 4
        v[v == 0] = rng.choice([0.0, -0.0], size=int((v == 0).sum())).astype(np.float32)
        return v
    return rng.integers(0, levels, size=shape, dtype=dtype)


@pytest.mark.parametrize("shape", SHAPES_2D + SHAPES_3D)
@pytest.mark.parametrize("dtype", [np.uint8, np.uint16, np.float32])
def test_coeff_map_matches_oracle(shape, dtype):
    B = 2
    X = np.stack([_rand(shape, dtype, 100 + i) for i in range(B)])
    got = host(api.ecc_coeff(dev(X), len(shape)))
    for i in range(B):
        np.testing.assert_array_equal(got[i], OC.coeff(X[i]), err_msg=f"{shape} {dtype}")


@pytest.mark.parametrize("shape", SHAPES_2D + SHAPES_3D)
@pytest.mark.parametrize("dtype", [np.uint8, np.uint16])
def test_hard_levels(shape, dtype, flow):
    B, bins = 3, 11  # levels 0..12 -> the top two are above the last threshold and dropped
    X = np.stack([_rand(shape, dtype, 7 + i, levels=13) for i in range(B)])
    got = host(api.ecc_hard(dev(X), len(shape), bins))
    np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, O.thresholds_levels(bins)))


@pytest.mark.parametrize("shape", SHAPES_2D + SHAPES_3D)
def test_hard_float_auto_range(shape, flow):
    B, bins = 2, 37
    rng = np.random.default_rng(5)
    X = rng.standard_normal((B,) + shape).astype(np.float32)
    got = host(api.ecc_hard(dev(X), len(shape), bins))
    t = O.thresholds_equal_width(X.min(), X.max(), bins)
    np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, t))
    assert np.all(got[:, -1] == 1)


@pytest.mark.parametrize("dtype", [np.uint8, np.uint16, np.float32])
@pytest.mark.parametrize("shape", [(40, 50), (6, 20, 30)])
def test_hard_supplied_range(shape, dtype, flow):
    X = np.stack([_rand(shape, dtype, 3 + i, levels=40) for i in range(2)])
    for lo, hi, bins in [(-1.5, 7.25, 16), (2.0, 2.0, 4), (0.0, 39.0, 40), (-100.0, 100.0, 1000)]:
        got = host(api.ecc_hard(dev(X), len(shape), bins, range=(lo, hi)))
        t = O.thresholds_equal_width(lo, hi, bins)
        np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, t), err_msg=f"{lo} {hi} {bins}")


def test_hard_many_bins_and_ties_on_edges(flow):
    # values exactly on thresholds; bins up to the maximum
    X = (np.arange(64 * 64, dtype=np.float32).reshape(64, 64) % 97) / 8
    X = X[None]
    for bins in (1, 2, 96, 4096, 16384):
        got = host(api.ecc_hard(dev(X), 2, bins, range=(0.0, 12.0)))
        np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, O.thresholds_equal_width(0.0, 12.0, bins)))


def test_constant_and_ramp(flow):
    X = np.full((1, 9, 10, 11), 3, np.uint8)
    got = host(api.ecc_hard(dev(X), 3, 5))
    np.testing.assert_array_equal(got[0], [0, 0, 0, 1, 1])
    X = np.full((1, 33, 65), 0.5, np.float32)
    got = host(api.ecc_hard(dev(X), 2, 8))  # degenerate auto range lo == hi
    np.testing.assert_array_equal(got[0], 1)
    X = np.arange(40 * 50, dtype=np.uint16).reshape(1, 40, 50)
    got = host(api.ecc_hard(dev(X), 2, 2000))
    np.testing.assert_array_equal(got[0], 1)


def test_depth_one_equals_2d_and_batch_equals_singles(flow):
    rng = np.random.default_rng(12)
    X = rng.integers(0, 32, size=(4, 37, 41), dtype=np.uint8)
    a = host(api.ecc_hard(dev(X), 2, 32))
    b = host(api.ecc_hard(dev(X[:, None]), 3, 32))
    np.testing.assert_array_equal(a, b)
    for i in range(4):
        np.testing.assert_array_equal(host(api.ecc_hard(dev(X[i:i + 1]), 2, 32))[0], a[i])


def test_repeated_calls_are_identical_and_workspace_reusable(flow):
    X = synth.grf((3, 48, 52), 1.5, 77)[None]
    g = dev(X)
    ws = torch.empty(api.ecc_workspace_bytes((3, 48, 52), 1, 128), dtype=torch.uint8, device="cuda")
    a = host(api.ecc_hard(g, 3, 128, workspace=ws))
    for _ in range(3):
        np.testing.assert_array_equal(host(api.ecc_hard(g, 3, 128, workspace=ws)), a)


def _overflow_flag(ws):
    # fifth 32-bit word of the workspace header: set by the single-pass sweep when a
    # critical-vertex list ran out of room (the histogram-mode sweep then redid the work)
    return int(ws[16:20].cpu().numpy().view(np.uint32)[0])


@pytest.mark.parametrize("shape", [(256, 256), (300, 1000), (33, 70, 130), (64, 64, 64)])
def test_single_pass_overflow_fallback(shape):
    bins = 100
    rng = np.random.default_rng(21)
    rough = rng.standard_normal((2,) + shape).astype(np.float32)   # ~58 % of the vertices critical
    smooth = np.stack([synth.grf(shape, 3.0, 500 + i) for i in range(2)])  # ~1 %
    ws = torch.empty(api.ecc_workspace_bytes(shape, 2, bins), dtype=torch.uint8, device="cuda")
    prev = api.ecc_debug_force(api.ECC_FORCE_NO_SMALL)  # the lists of the sweeps, also for the smaller shapes
    try:
        for X, want_flag in ((rough, 1), (smooth, 0), (rough, 1)):
            got = host(api.ecc_hard(dev(X), len(shape), bins, workspace=ws))
            assert _overflow_flag(ws) == want_flag
            t = O.thresholds_equal_width(X.min(), X.max(), bins)
            np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, t))
    finally:
        api.ecc_debug_force(prev)


@pytest.mark.parametrize("shape", [(70, 300), (9, 40, 130)])
def test_float_extremes_denormals_and_neighbouring_floats(shape, flow):
    # the fast sweeps decide "q before p" from the sign of a float difference: that is
    # exact only with gradual underflow, and must survive overflow of the difference
    tiny = np.float32(1e-45)  # smallest denormal
    pool = np.array([0.0, -0.0, tiny, -tiny, 3 * tiny, np.finfo(np.float32).tiny,
                     np.finfo(np.float32).tiny - tiny, 1.0, np.nextafter(np.float32(1), np.float32(2)),
                     np.nextafter(np.float32(1), np.float32(0)), -1.0, np.finfo(np.float32).max,
                     -np.finfo(np.float32).max, 1e38, -1e38], dtype=np.float32)
    rng = np.random.default_rng(33)
    X = pool[rng.integers(0, len(pool), size=(2,) + shape)]
    got = host(api.ecc_coeff(dev(X), len(shape)))
    for i in range(2):
        np.testing.assert_array_equal(got[i], OC.coeff(X[i]))
    for rng_arg in (None, (-2.0, 2.0), (-1e-44, 1e-44)):
        bins = 64
        got = host(api.ecc_hard(dev(X), len(shape), bins, range=rng_arg))
        lo, hi = (X.min(), X.max()) if rng_arg is None else rng_arg
        t = O.thresholds_equal_width(lo, hi, bins)
        np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, t), err_msg=str(rng_arg))


def test_3d_planes_beyond_the_32_bit_segment_window():
    # nine planes of 243 MB: byte offsets inside the one z segment pass 2^31, so the
    # sweep has to rebase its buffer resource as it marches
    D, H, W = 9, 7800, 7800
    rng = np.random.default_rng(8)
    y = np.sin(np.arange(H, dtype=np.float32) * 0.05)[:, None]
    x = np.cos(np.arange(W, dtype=np.float32) * 0.03)[None, :]
    X = np.empty((1, D, H, W), np.float32)
    for z in range(D):
        X[0, z] = y * x * np.float32(np.cos(0.7 * z)) + np.float32(0.004) * rng.random((H, W), dtype=np.float32)
    bins = 300
    lo, hi = float(X.min()), float(X.max())
    want = OC.ecc_hard_batch(X, O.thresholds_equal_width(lo, hi, bins))
    g = dev(X)
    np.testing.assert_array_equal(host(api.ecc_hard(g, 3, bins)), want)                    # single pass (lists)
    np.testing.assert_array_equal(host(api.ecc_hard(g, 3, bins, range=(lo, hi))), want)    # histogram mode
    assert want[0, -1] == 1


@pytest.mark.parametrize("shape", [(3, 5), (4, 8), (2, 3, 9)])
def test_largest_batch(shape):
    # 65535 items (the batch rides on the grid's y dimension), tiny grids: one curve each
    rng = np.random.default_rng(19)
    X = rng.integers(0, 7, size=(65535,) + shape, dtype=np.uint8)
    got = host(api.ecc_hard(dev(X), len(shape), 7))
    np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, O.thresholds_levels(7)))
    Xf = (X.astype(np.float32) - 3) / 2
    gotf = host(api.ecc_hard(dev(Xf), len(shape), 5))  # batch-global range
    np.testing.assert_array_equal(gotf, OC.ecc_hard_batch(Xf, O.thresholds_equal_width(Xf.min(), Xf.max(), 5)))


def test_one_bin_and_most_bins(flow):
    X = synth.grf((70, 90), 2.0, 31)[None]
    for bins in (1, 16384):
        got = host(api.ecc_hard(dev(X), 2, bins))
        np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, O.thresholds_equal_width(X.min(), X.max(), bins)))
        assert got[0, -1] == 1


# ---- the workloads the benchmark times, at full size -------------------------


def test_config_c1_full():
    X = synth.config_c1()[None]
    got = host(api.ecc_hard(dev(X), 2, 256))
    np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, O.thresholds_levels(256)))
    assert got[0, -1] == 1


def test_config_c3_full():
    X = synth.config_c3()[None]
    got = host(api.ecc_hard(dev(X), 3, 4096))
    np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, O.thresholds_levels(4096)))


def test_config_c2_full():
    X = synth.config_c2()
    got = host(api.ecc_hard(dev(X), 2, 1024))
    t = O.thresholds_equal_width(X.min(), X.max(), 1024)
    np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, t))
    assert np.all(got[:, -1] == 1)
    # supplied range gives the same curve in one pass
    got2 = host(api.ecc_hard(dev(X), 2, 1024, range=(float(X.min()), float(X.max()))))
    np.testing.assert_array_equal(got2, got)


def test_config_c4_full():
    X = synth.config_c4()[None]
    got = host(api.ecc_hard(dev(X), 3, 1024))
    t = O.thresholds_equal_width(X.min(), X.max(), 1024)
    np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, t))
    assert got[0, -1] == 1


# ---- the largest sizes of the paper's Tables 1-2, as the benchmark's size sweep builds them ----


def test_table_size_8192_squared():
    X = np.tile(synth.grf((4096, 4096), 4.0, 4242), (2, 2))[None]   # periodic field: the tiling is seamless
    got = host(api.ecc_hard(dev(X), 2, 1024))
    t = O.thresholds_equal_width(X.min(), X.max(), 1024)
    np.testing.assert_array_equal(got, OC.ecc_hard_batch(X, t))
    assert got[0, -1] == 1


def test_table_size_1024_cubed():
    # 4 GiB of float32: element offsets pass 2^31, the sweep runs in many z segments
    X = np.tile(synth.grf((512, 512, 512), 3.0, 4242), (2, 2, 2))[None]
    lo, hi = float(X.min()), float(X.max())
    g = dev(X)
    got = host(api.ecc_hard(g, 3, 1024))
    got_r = host(api.ecc_hard(g, 3, 1024, range=(lo, hi)))
    del g
    torch.cuda.empty_cache()
    want = OC.ecc_hard_batch(X, O.thresholds_equal_width(lo, hi, 1024))
    np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(got_r, want)
    assert got[0, -1] == 1
