"""The tie-break of Eq. 3 (equal values: the smaller C-order index comes first; -0 equals +0)
observed vertex by vertex on the kernels that run in every timed call.

ecc_coeff goes through the bit-sliced strip (2D) / tube (3D) sweeps for every shape they take, so
its map is the stencil of the hard and the soft path made visible.  The grids here are tied
almost everywhere (a handful of levels, signed zeros, plateaus of a quantised smooth field), on
shapes that span several strips, row groups, segments and chunks, with ragged tails, unaligned
base pointers and folded 3D launches.  The soft path is checked on quantised fields as well: its
grad_X is -lambda c(p) (...) per vertex, so a coefficient that sits on the wrong one of two equal
neighbours shows up directly.  The fall-back kernels (one thread per vertex, two-pass range, soft
tile kernels) are forced on the same inputs through ecc_debug_force.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import ecc_oracle as O
from oracle import ecc_oracle_c as OC
from paper_2510_20271_amd import api, synth
from tests.gpu_util import dev, host
from tests.test_gpu_soft import _close, _close_sum

pytestmark = pytest.mark.gpu


def _tied(shape, dtype, seed, levels=3):
    rng = np.random.default_rng(seed)
    if dtype == np.float32:
        v = rng.integers(-levels, levels, size=shape).astype(np.float32) / 4
        v[v == 0] = rng.choice([0.0, -0.0], size=int((v == 0).sum())).astype(np.float32)
        return v
    return rng.integers(0, levels, size=shape, dtype=dtype)


def _quantised(shape, seed, steps=8.0, sigma=2.0):
    """A smooth field rounded to a few levels: plateaus of equal values with signed zeros."""
    x = np.round(synth.grf(shape, sigma, seed) * np.float32(steps * 10)) / np.float32(steps)
    x = x.astype(np.float32)
    z = x == 0
    x[z] = np.where(np.random.default_rng(seed).random(int(z.sum())) < 0.5, np.float32(-0.0), np.float32(0.0))
    return x


# 2D: several strips of 248 columns (aligned interior strips need W % 4 == 0), several 8-row
# chunks and segments, ragged last strip / chunk; 3D: several strips of 62 columns, row groups
# of 4 with a ragged last one, more than one 30-plane chunk and more than one segment
# (widths 256, 260, 500, 512: the first and the last strip start / end at the grid's own edge)
SHAPES = [(70, 1024), (33, 1000), (129, 503), (300, 250), (16, 249), (1, 600), (600, 8), (40, 256), (24, 260),
          (18, 500), (20, 512),
          (70, 70, 130), (35, 9, 200), (2, 131, 64), (64, 6, 63), (31, 5, 8)]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("dtype", [np.uint8, np.uint16, np.float32])
def test_coeff_map_of_the_sweeps_on_tied_grids(shape, dtype):
    B = 2
    X = np.stack([_tied(shape, dtype, 900 + i) for i in range(B)])
    got = host(api.ecc_coeff(dev(X), len(shape)))
    for i in range(B):
        np.testing.assert_array_equal(got[i], OC.coeff(X[i]), err_msg=f"{shape} {dtype}")


@pytest.mark.parametrize("shape", [(40, 1024), (50, 70, 130)])
def test_coeff_map_quantised_fields_and_constant_grid(shape):
    X = np.stack([_quantised(shape, 31), np.full(shape, -0.0, np.float32), _quantised(shape, 32, steps=2.0)])
    got = host(api.ecc_coeff(dev(X), len(shape)))
    for i in range(3):
        np.testing.assert_array_equal(got[i], OC.coeff(X[i]))
    # a constant grid: the one vertex that is charged is the first in C order
    assert got[1].ravel()[0] == 1 and np.count_nonzero(got[1]) == 1


@pytest.mark.parametrize("off", [1, 2, 3])
def test_coeff_map_unaligned_rows(off):
    # the grid starts 4, 8, 12 bytes past a 16-byte boundary: the strips load element by element
    shape = (20, 512)
    X = _tied(shape, np.float32, 77)
    buf = torch.zeros(X.size + 8, dtype=torch.float32, device="cuda")
    buf[off:off + X.size] = dev(X).reshape(-1)
    g = buf[off:off + X.size].view((1,) + shape)
    np.testing.assert_array_equal(host(api.ecc_coeff(g, 2))[0], OC.coeff(X))


@pytest.mark.parametrize("b,D,H,W", [(8, 200, 202, 70), (16, 200, 203, 20)])
def test_coeff_map_folded_3d_launch(b, D, H, W):
    # large enough for the tube sweep to fold its narrow last strip (several row groups in one wave)
    base = _quantised((D, H, W), 5, steps=4.0)
    X = np.stack([np.roll(base, 3 * i, axis=2) for i in range(b)])
    got = host(api.ecc_coeff(dev(X), 3))
    for i in (0, b - 1):
        np.testing.assert_array_equal(got[i], OC.coeff(X[i]))


@pytest.mark.parametrize("shape", [(33, 1000), (70, 70, 130)])
@pytest.mark.parametrize("dtype", [np.uint8, np.float32])
def test_forced_generic_kernels_agree(shape, dtype):
    X = np.stack([_tied(shape, dtype, 40 + i, levels=5) for i in range(2)])
    prev = api.ecc_debug_force(api.ECC_FORCE_GENERIC)
    try:
        c = host(api.ecc_coeff(dev(X), len(shape)))
        curve = host(api.ecc_hard(dev(X), len(shape), 9, range=(-1.5, 1.5) if dtype == np.float32 else None))
    finally:
        api.ecc_debug_force(prev)
    for i in range(2):
        np.testing.assert_array_equal(c[i], OC.coeff(X[i]))
    t = O.thresholds_equal_width(-1.5, 1.5, 9) if dtype == np.float32 else O.thresholds_levels(9)
    np.testing.assert_array_equal(curve, OC.ecc_hard_batch(X, t))
    assert api.ecc_debug_force(0) == 0  # and the switch is off again


@pytest.mark.parametrize("shape", [(300, 1000), (33, 70, 130)])
def test_forced_two_pass_range(shape):
    # separate min / max pass + histogram-mode strip / tube sweep
    X = np.stack([_quantised(shape, 60 + i) for i in range(2)])
    t = O.thresholds_equal_width(X.min(), X.max(), 50)
    want = OC.ecc_hard_batch(X, t)
    prev = api.ecc_debug_force(api.ECC_FORCE_TWO_PASS)
    try:
        got = host(api.ecc_hard(dev(X), len(shape), 50))
    finally:
        api.ecc_debug_force(prev)
    np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(host(api.ecc_hard(dev(X), len(shape), 50)), want)  # single pass


def _soft_case(Xb, u, alpha, tau, lam, G, tilted=False):
    nd = Xb.ndim - 1
    g, ud, td = dev(Xb), dev(u), dev(tau)
    chi = host(api.ecc_soft_fwd(g, nd, ud, alpha, td, lam, tilted_c=tilted))
    gx, dt, du = (host(a) for a in api.ecc_soft_bwd(g, nd, ud, alpha, td, lam, grad_chi=dev(G), tilted_c=tilted))
    for i, X in enumerate(Xb):
        c = O.coeff_tilted(X, u, alpha) if tilted else O.coeff(X)
        _close_sum(chi[i], O.soft_fwd(X, u, alpha, tau, lam, c=c), 1e-4, f"chi[{i}]")
        rgx, rdt, rdu = O.soft_bwd(X, u, alpha, tau, lam, G[i], c=c)
        _close(gx[i], rgx, 1e-3, f"grad_X[{i}]")
        _close_sum(dt[i], rdt, 1e-3, f"dchi_dtau[{i}]")
        _close_sum(du[i], rdu, 1e-3, f"dchi_du[{i}]")
        # grad_X is non-zero exactly where the oracle's coefficient is (up to underflow of sigma')
        assert not np.any((gx[i] != 0) & (c == 0)), "grad_X at a vertex with c = 0"


SOFT_SHAPES = [(64, 64), (100, 259), (45, 1024), (9, 30, 70), (40, 33, 129)]


@pytest.mark.parametrize("shape", SOFT_SHAPES)
@pytest.mark.parametrize("alpha", [0.0, 0.01])
def test_soft_fused_paths_on_quantised_fields(shape, alpha):
    nd, B, T = len(shape), 2, 9
    Xb = np.stack([_quantised(shape, 70 + i) for i in range(B)])
    tau = np.linspace(Xb.min() - 0.1, Xb.max() + 0.3, T).astype(np.float32)
    u = np.array([np.cos(0.3), np.sin(0.3)] if nd == 2 else [0.48, -0.6, 0.64], np.float32)
    G = np.random.default_rng(1).standard_normal((B, T)).astype(np.float32)
    _soft_case(Xb, u, np.float32(alpha), tau, np.float32(20.0), G)


@pytest.mark.parametrize("shape", [(100, 259), (9, 30, 70)])
def test_soft_tile_kernels_on_quantised_fields(shape):
    nd, B = len(shape), 2
    Xb = np.stack([_quantised(shape, 80 + i) for i in range(B)])
    u = np.array([np.cos(0.3), np.sin(0.3)] if nd == 2 else [0.48, -0.6, 0.64], np.float32)
    # more thresholds than the fused paths take: the tile kernels by themselves
    T = 300
    tau = np.linspace(Xb.min() - 0.1, Xb.max() + 0.3, T).astype(np.float32)
    G = np.random.default_rng(2).standard_normal((B, T)).astype(np.float32)
    _soft_case(Xb, u, np.float32(0.01), tau, np.float32(20.0), G)
    # and forced, with few thresholds
    T = 7
    tau = np.linspace(Xb.min() - 0.1, Xb.max() + 0.3, T).astype(np.float32)
    G = G[:, :T].copy()
    prev = api.ecc_debug_force(api.ECC_FORCE_SOFT_TILES)
    try:
        _soft_case(Xb, u, np.float32(0.01), tau, np.float32(20.0), G)
    finally:
        api.ecc_debug_force(prev)


@pytest.mark.parametrize("shape", [(100, 259), (9, 30, 70)])
def test_soft_tilted_coefficient_on_quantised_fields(shape):
    # c of the tilted field: the tilt breaks most ties, a tilt along one axis keeps those of the others
    nd, B, T = len(shape), 2, 9
    Xb = np.stack([_quantised(shape, 90 + i) for i in range(B)])
    G = np.random.default_rng(3).standard_normal((B, T)).astype(np.float32)
    for u in ([1.0, 0.0], [0.0, -1.0], [0.6, 0.8]) if nd == 2 else ([0.0, 0.0, 1.0], [0.48, -0.6, 0.64]):
        u = np.array(u, np.float32)
        alpha = np.float32(0.125)  # a power of two: tilted values of different vertices collide exactly
        Y = np.stack([O.tilt_field(x, u, alpha) for x in Xb])
        tau = np.linspace(Y.min() - 0.1, Y.max() + 0.3, T).astype(np.float32)
        _soft_case(Xb, u, alpha, tau, np.float32(6.0), G, tilted=True)
