"""The hard curves on the further element types (float16, bfloat16, int16: loaded directly by the
strip / tube sweeps, or rounded to float32 first on the shapes the plain kernels take; int32,
float64: always rounded first): bit-exact against the oracle's curve of the float32 grid, for the
sublevel and superlevel sets of both constructions and every threshold mode."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import ecc_oracle as O
from paper_2510_20271_amd import api
from tests.gpu_util import host

pytestmark = pytest.mark.gpu

SHAPES = [(1, 9), (33, 70), (130, 300), (5, 9, 33), (20, 40, 131)]


def _grid(kind, shape, rng):
    """(device tensor, float32 numpy array it rounds to)"""
    size = (2,) + shape
    if kind == "f16":
        t = torch.from_numpy((rng.standard_normal(size) * 3).astype(np.float16))
    elif kind == "bf16":
        t = torch.from_numpy((rng.standard_normal(size) * 3).astype(np.float32)).to(torch.bfloat16)
    elif kind == "i16":
        t = torch.from_numpy(rng.integers(-20, 60, size=size).astype(np.int16))
    elif kind == "i32":
        # small levels and, in places, values beyond 2^24 that differ by less than a float32 step
        a = rng.integers(-5, 40, size=size).astype(np.int32)
        big = rng.random(size) < 0.05
        a[big] = (1 << 24) + rng.integers(0, 9, size=int(big.sum())).astype(np.int32)
        t = torch.from_numpy(a)
    else:
        # float64 values that collide in float32 and values that do not
        a = 1.0 + rng.integers(0, 50, size=size) * 1e-9 + rng.integers(0, 6, size=size) * 0.25
        t = torch.from_numpy(a.astype(np.float64))
    return t.cuda(), t.float().numpy()


@pytest.mark.parametrize("kind", ["f16", "bf16", "i16", "i32", "f64"])
@pytest.mark.parametrize("shape", SHAPES)
def test_converted_dtypes(kind, shape, flow):
    rng = np.random.default_rng(len(shape) * 100 + shape[-1])
    g, Y = _grid(kind, shape, rng)
    assert Y.dtype == np.float32
    nd = len(shape)
    bins = 37
    if kind in ("i16", "i32"):  # one bin per level when no range is given
        t, ts = O.thresholds_levels(bins), O.thresholds_levels_super(bins)
    else:
        lo, hi = float(Y.min()), float(Y.max())
        t = O.thresholds_equal_width(lo, hi, bins)
        ts = O.thresholds_lower(t, lo)
    np.testing.assert_array_equal(host(api.ecc_hard(g, nd, bins)), O.ecc_hard_batch(Y, t))
    np.testing.assert_array_equal(host(api.ecc_hard(g, nd, bins, top=True)), O.ecc_top_batch(Y, t))
    np.testing.assert_array_equal(host(api.ecc_hard(g, nd, bins, superlevel=True)), O.ecc_super_batch(Y, ts))
    np.testing.assert_array_equal(host(api.ecc_hard(g, nd, bins, top=True, superlevel=True)),
                                  O.ecc_super_batch(Y, ts, True))
    # a supplied range that leaves values out on both sides
    lo, hi = float(np.quantile(Y, 0.1)), float(np.quantile(Y, 0.9))
    t = O.thresholds_equal_width(lo, hi, bins)
    np.testing.assert_array_equal(host(api.ecc_hard(g, nd, bins, range=(lo, hi))), O.ecc_hard_batch(Y, t))
    np.testing.assert_array_equal(host(api.ecc_hard(g, nd, bins, range=(lo, hi), superlevel=True)),
                                  O.ecc_super_batch(Y, O.thresholds_lower(t, lo)))


def test_int32_levels_equal_the_uint16_path(flow):
    rng = np.random.default_rng(3)
    a = rng.integers(0, 300, size=(2, 70, 131))
    want = host(api.ecc_hard(torch.from_numpy(a.astype(np.int16)).cuda().view(torch.uint16), 2, 256))
    np.testing.assert_array_equal(host(api.ecc_hard(torch.from_numpy(a.astype(np.int32)).cuda(), 2, 256)), want)
    np.testing.assert_array_equal(host(api.ecc_hard(torch.from_numpy(a.astype(np.int16)).cuda(), 2, 256)), want)


# ---- float16 / bfloat16 / int16 read directly by the strip / tube sweeps ----------------------
def _tied16(kind, shape, seed):
    """Few levels (ties everywhere) with signed zeros; (device tensor, float32 numpy view)."""
    rng = np.random.default_rng(seed)
    a = rng.integers(-6, 6, size=shape).astype(np.float32) / 4
    if kind == "i16":
        t = torch.from_numpy((a * 4).astype(np.int16))
        return t.cuda(), t.float().numpy()
    a[a == 0] = rng.choice([0.0, -0.0], size=int((a == 0).sum())).astype(np.float32)
    t = torch.from_numpy(a)
    t = t.half() if kind == "f16" else t.to(torch.bfloat16)
    return t.cuda(), t.float().numpy()


@pytest.mark.parametrize("kind", ["f16", "bf16", "i16"])
@pytest.mark.parametrize("shape", [(300, 1000), (70, 1024), (129, 503), (40, 70, 130), (35, 9, 200)])
def test_two_byte_types_through_the_sweeps(kind, shape):
    nd, bins = len(shape), 23
    g, Y = _tied16(kind, (2,) + shape, 11 + len(shape))
    lo, hi = float(Y.min()), float(Y.max())
    t = O.thresholds_equal_width(lo, hi, bins)
    ts = O.thresholds_lower(t, lo)
    want = O.ecc_hard_batch(Y, t)
    np.testing.assert_array_equal(host(api.ecc_hard(g, nd, bins, range=(lo, hi))), want)  # histogram-mode sweep
    if kind != "i16":
        np.testing.assert_array_equal(host(api.ecc_hard(g, nd, bins)), want)              # single pass, range on the device
        prev = api.ecc_debug_force(api.ECC_FORCE_TWO_PASS)                                 # float32 copy + range pass
        try:
            np.testing.assert_array_equal(host(api.ecc_hard(g, nd, bins)), want)
        finally:
            api.ecc_debug_force(prev)
    np.testing.assert_array_equal(host(api.ecc_hard(g, nd, bins, range=(lo, hi), top=True)), O.ecc_top_batch(Y, t))
    np.testing.assert_array_equal(host(api.ecc_hard(g, nd, bins, range=(lo, hi), superlevel=True)),
                                  O.ecc_super_batch(Y, ts))
    np.testing.assert_array_equal(host(api.ecc_hard(g, nd, bins, range=(lo, hi), top=True, superlevel=True)),
                                  O.ecc_super_batch(Y, ts, True))
    prev = api.ecc_debug_force(api.ECC_FORCE_GENERIC)  # the one-thread-per-vertex kernels on the float32 copy
    try:
        np.testing.assert_array_equal(host(api.ecc_hard(g, nd, bins, range=(lo, hi))), want)
    finally:
        api.ecc_debug_force(prev)


@pytest.mark.parametrize("off", [1, 2, 3])
def test_two_byte_rows_not_aligned_to_eight_bytes(off):
    shape = (40, 512)
    g0, Y = _tied16("f16", (1,) + shape, 5)
    buf = torch.zeros(Y.size + 8, dtype=torch.float16, device="cuda")
    buf[off:off + Y.size] = g0.reshape(-1)
    g = buf[off:off + Y.size].view((1,) + shape)
    t = O.thresholds_equal_width(-1.5, 1.5, 12)
    np.testing.assert_array_equal(host(api.ecc_hard(g, 2, 12, range=(-1.5, 1.5))), O.ecc_hard_batch(Y, t))
