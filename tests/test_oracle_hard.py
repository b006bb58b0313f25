"""Pins for the hard-ECC CPU oracle (no GPU).

The oracle has three independent derivations of the curve (literal Eq. 1-2
count, cell-maximum histogram, per-vertex coefficient of Eq. 3) in numpy and
one in plain C.  They are pinned to hand-worked examples, closed forms,
invariants and each other, so that a dropped term, a wrong sign, a wrong
tie-break or a transposed axis fails at least one test.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import ecc_oracle as O
from oracle import ecc_oracle_c as OC


def _read_golden(path):
    blocks, cur = [], []
    for line in open(path):
        line = line.strip()
        if line.startswith("#"):
            if cur:
                blocks.append(cur)
                cur = []
            continue
        if line:
            cur.append([int(v) for v in line.split()])
    if cur:
        blocks.append(cur)
    return [np.array(b) for b in blocks]


def _all_curves(X, t):
    """Curves from the four derivations."""
    return {
        "brute": O.ecc_bruteforce(X, t),
        "cellmax": O.ecc_cellmax(X, t),
        "coeff": O.ecc_hard(X, t),
        "c": OC.ecc_hard(X, t),
    }


@pytest.mark.parametrize("name", ["worked_3x3.txt", "frame_4x4.txt"])
def test_golden_examples(golden_dir, name):
    X, c, curve = _read_golden(os.path.join(golden_dir, name))
    curve = curve.ravel()
    t = O.thresholds_levels(len(curve))
    X8 = X.astype(np.uint8)
    np.testing.assert_array_equal(O.coeff(X8), c)
    np.testing.assert_array_equal(OC.coeff(X8), c)
    for k, v in _all_curves(X8, t).items():
        np.testing.assert_array_equal(v, curve, err_msg=k)
    # float input gives the same map and curve
    np.testing.assert_array_equal(OC.coeff(X.astype(np.float32)), c)


def test_exhaustive_three_level_3x3():
    """All 3^9 grids over {0,1,2}: ties everywhere; every derivation agrees at
    every level and sum c = 1."""
    t = O.thresholds_levels(3)
    for vals in itertools.product(range(3), repeat=9):
        X = np.array(vals, dtype=np.uint8).reshape(3, 3)
        ref = O.ecc_bruteforce(X, t)
        c = O.coeff(X)
        assert c.sum() == 1
        np.testing.assert_array_equal(O.ecc_from_coeff(X, c, t), ref)
        np.testing.assert_array_equal(O.ecc_cellmax(X, t), ref)
        assert ref[-1] == 1


def test_exhaustive_3x3_c_oracle_matches_numpy_coeff():
    grids = np.array(list(itertools.product(range(3), repeat=9)), dtype=np.uint8).reshape(-1, 3, 3)
    for X in grids[::7]:
        np.testing.assert_array_equal(OC.coeff(X), O.coeff(X))


def test_coefficient_range_extremes():
    """The exact coefficient leaves {-1,0,1}: -3 in 2D when the four edge
    neighbours are lower and the diagonals higher; -5 and +7 in 3D."""
    X = np.array([[9, 0, 9], [0, 5, 0], [9, 0, 9]], dtype=np.uint8)
    assert O.coeff(X)[1, 1] == -3 and OC.coeff(X)[1, 1] == -3
    X3 = np.full((3, 3, 3), 9, dtype=np.uint8)
    X3[1, 1, 1] = 5
    for ax in range(3):
        for d in (0, 2):
            idx = [1, 1, 1]
            idx[ax] = d
            X3[tuple(idx)] = 0
    assert O.coeff(X3)[1, 1, 1] == -5 and OC.coeff(X3)[1, 1, 1] == -5
    # faces and edges lower, corners higher: 1 - 6 + 12 - 0 = 7
    X3 = np.zeros((3, 3, 3), dtype=np.uint8)
    X3[1, 1, 1] = 5
    for cz, cy, cx in itertools.product((0, 2), repeat=3):
        X3[cz, cy, cx] = 9
    assert O.coeff(X3)[1, 1, 1] == 7 and OC.coeff(X3)[1, 1, 1] == 7


@pytest.mark.parametrize("shape", [(2, 2, 2), (3, 4, 2), (4, 4, 4), (1, 5, 3), (2, 1, 4)])
def test_random_small_3d_with_ties(shape):
    rng = np.random.default_rng(7)
    t = O.thresholds_levels(4)
    for _ in range(40):
        X = rng.integers(0, 4, size=shape, dtype=np.uint8)
        cur = _all_curves(X, t)
        for k, v in cur.items():
            np.testing.assert_array_equal(v, cur["brute"], err_msg=k)
        assert O.coeff(X).sum() == 1
        np.testing.assert_array_equal(OC.coeff(X), O.coeff(X))


@pytest.mark.parametrize("shape", [(1, 1), (1, 7), (7, 1), (2, 2), (5, 9), (13, 6)])
def test_random_small_2d_with_ties(shape):
    rng = np.random.default_rng(11)
    t = O.thresholds_levels(5)
    for _ in range(40):
        X = rng.integers(0, 5, size=shape, dtype=np.uint16)
        cur = _all_curves(X, t)
        for k, v in cur.items():
            np.testing.assert_array_equal(v, cur["brute"], err_msg=k)
        np.testing.assert_array_equal(OC.coeff(X), O.coeff(X))


def test_constant_grid_tie_break():
    for shape in [(4, 5), (3, 4, 5)]:
        X = np.full(shape, 3, dtype=np.uint8)
        expect = np.zeros(shape, dtype=np.int8)
        expect.flat[0] = 1
        np.testing.assert_array_equal(O.coeff(X), expect)
        np.testing.assert_array_equal(OC.coeff(X), expect)
        np.testing.assert_array_equal(OC.ecc_hard(X, O.thresholds_levels(5)), [0, 0, 0, 1, 1])


def test_ramps_are_regular():
    """Monotone ramps: only the first vertex is critical; ECC = 1 from the minimum up."""
    X = np.arange(4 * 5 * 6, dtype=np.uint16).reshape(4, 5, 6)
    for c in (O.coeff(X), OC.coeff(X)):
        assert c.flat[0] == 1 and np.count_nonzero(c) == 1
    z, y, x = np.meshgrid(np.arange(4), np.arange(5), np.arange(6), indexing="ij")
    X = (x + y + z).astype(np.uint8)  # index ties on every anti-diagonal plane
    for c in (O.coeff(X), OC.coeff(X)):
        assert c.flat[0] == 1 and np.count_nonzero(c) == 1
    # reversed ramp: the last vertex enters first
    X = (200 - np.arange(4 * 5, dtype=np.int64)).astype(np.uint8).reshape(4, 5)
    for c in (O.coeff(X), OC.coeff(X)):
        assert c.flat[-1] == 1 and np.count_nonzero(c) == 1
    np.testing.assert_array_equal(OC.ecc_hard(X, O.thresholds_levels(201))[181:], 1)


def test_checkerboard():
    y, x = np.meshgrid(np.arange(6), np.arange(7), indexing="ij")
    X = ((x + y) % 2).astype(np.uint8)
    t = O.thresholds_levels(2)
    for k, v in _all_curves(X, t).items():
        np.testing.assert_array_equal(v, [int((X == 0).sum()), 1], err_msg=k)


def _shape_curve(mask):
    """low (0) on the shape, high (1) elsewhere: ECC(0) = chi(shape)."""
    X = np.where(mask, 0, 1).astype(np.uint8)
    t = O.thresholds_levels(2)
    cur = _all_curves(X, t)
    for k, v in cur.items():
        np.testing.assert_array_equal(v, cur["brute"], err_msg=k)
    return cur["c"]


def test_solid_shapes_known_euler_characteristic():
    # filled box
    m = np.zeros((7, 8), bool); m[2:5, 1:6] = True
    np.testing.assert_array_equal(_shape_curve(m), [1, 1])
    # square annulus
    m = np.zeros((7, 8), bool); m[1:6, 1:7] = True; m[3, 3:5] = False
    np.testing.assert_array_equal(_shape_curve(m), [0, 1])
    # two boxes
    m = np.zeros((7, 9), bool); m[1:3, 1:3] = True; m[4:6, 5:8] = True
    np.testing.assert_array_equal(_shape_curve(m), [2, 1])
    # 3D hollow shell: chi = 2
    m = np.zeros((7, 7, 7), bool); m[1:6, 1:6, 1:6] = True; m[3, 3, 3] = False
    np.testing.assert_array_equal(_shape_curve(m), [2, 1])
    # 3D solid torus (a square ring extruded): chi = 0
    m = np.zeros((5, 8, 8), bool); m[1:4, 1:7, 1:7] = True; m[1:4, 3:5, 3:5] = False
    np.testing.assert_array_equal(_shape_curve(m), [0, 1])
    # 3D solid ball-like box: chi = 1
    m = np.zeros((5, 6, 7), bool); m[1:4, 1:5, 2:6] = True
    np.testing.assert_array_equal(_shape_curve(m), [1, 1])


def test_invariants_below_min_and_at_max():
    rng = np.random.default_rng(3)
    X = rng.standard_normal((9, 10, 11)).astype(np.float32)
    lo, hi = float(X.min()), float(X.max())
    t = np.array([lo - 1.0, np.nextafter(np.float32(lo), np.float32(-9)), lo, hi, hi + 1], dtype=np.float64)
    cur = OC.ecc_hard(X, t)
    assert cur[0] == 0 and cur[1] == 0 and cur[2] == 1 and cur[3] == 1 and cur[4] == 1
    np.testing.assert_array_equal(O.ecc_cellmax(X, t), cur)


def test_geometry_invariance_and_depth_one():
    rng = np.random.default_rng(5)
    X = rng.integers(0, 16, size=(6, 7, 8), dtype=np.uint8)
    t = O.thresholds_levels(16)
    ref = OC.ecc_hard(X, t)
    np.testing.assert_array_equal(OC.ecc_hard(np.ascontiguousarray(X[::-1]), t), ref)
    np.testing.assert_array_equal(OC.ecc_hard(np.ascontiguousarray(X[:, :, ::-1]), t), ref)
    np.testing.assert_array_equal(OC.ecc_hard(np.ascontiguousarray(X.transpose(2, 0, 1)), t), ref)
    X2 = X[0]
    np.testing.assert_array_equal(OC.ecc_hard(X2[None], t), OC.ecc_hard(X2, t))
    np.testing.assert_array_equal(OC.coeff(X2[None])[0], OC.coeff(X2))


def test_iid_expectation_formula():
    """For i.i.d. values each k-vertex cell is present with probability q^k:
    E[ECC] = V q - E q^2 + F q^4 - C q^8 (cell counts of the full grid)."""
    n, L = 48, 16
    rng = np.random.default_rng(2024)
    reps = 6
    acc = np.zeros(L)
    for _ in range(reps):
        X = rng.integers(0, L, size=(n, n, n), dtype=np.uint16)
        acc += OC.ecc_hard(X, O.thresholds_levels(L))
    mean = acc / reps
    q = (np.arange(L) + 1) / L
    V, E, F, C = n ** 3, 3 * n * n * (n - 1), 3 * n * (n - 1) ** 2, (n - 1) ** 3
    expect = V * q - E * q ** 2 + F * q ** 4 - C * q ** 8
    # fluctuations of the mean are O(sqrt(V / reps)); sqrt(V) is ~3 % of the curve's scale
    assert np.max(np.abs(mean - expect)) < np.sqrt(V)
    assert np.max(np.abs(expect)) > 30 * np.sqrt(V)
    n2 = 200
    acc = np.zeros(L)
    for _ in range(reps):
        X = rng.integers(0, L, size=(n2, n2), dtype=np.uint8)
        acc += OC.ecc_hard(X, O.thresholds_levels(L))
    V, E, F = n2 * n2, 2 * n2 * (n2 - 1), (n2 - 1) ** 2
    expect = V * q - E * q ** 2 + F * q ** 4
    assert np.max(np.abs(acc / reps - expect)) < np.sqrt(V)


def test_float_thresholds_and_binning():
    t = O.thresholds_equal_width(-1.0, 3.0, 8)
    np.testing.assert_allclose(t, np.linspace(-0.5, 3.0, 8))
    assert t[-1] == 3.0
    x = np.array([-2.0, -1.0, -0.5, -0.49, 3.0, 3.1])
    np.testing.assert_array_equal(O.bin_index(x, t), [0, 0, 0, 1, 7, 8])
    # degenerate range
    t = O.thresholds_equal_width(2.0, 2.0, 4)
    np.testing.assert_array_equal(t, 2.0)
    # mid-size float field: curve ends at 1, starts with c of the minimum
    rng = np.random.default_rng(9)
    X = rng.standard_normal((37, 53)).astype(np.float32)
    t = O.thresholds_equal_width(X.min(), X.max(), 64)
    cur = _all_curves(X, t)
    for k, v in cur.items():
        np.testing.assert_array_equal(v, cur["brute"], err_msg=k)
    assert cur["c"][-1] == 1


def test_values_above_last_threshold_are_dropped():
    X = np.array([[0, 9], [9, 1]], dtype=np.uint8)
    t = O.thresholds_levels(2)
    for k, v in _all_curves(X, t).items():
        np.testing.assert_array_equal(v, [1, 2], err_msg=k)


def test_mid_size_dtypes_and_batch():
    rng = np.random.default_rng(17)
    Xb = rng.integers(0, 300, size=(3, 19, 23, 29), dtype=np.uint16)
    t = O.thresholds_levels(300)
    got = OC.ecc_hard_batch(Xb, t)
    for i in range(3):
        np.testing.assert_array_equal(got[i], O.ecc_cellmax(Xb[i], t))
    Xf = rng.standard_normal((2, 31, 17)).astype(np.float32)
    Xf[0, 3:9, 4:8] = Xf[0, 3, 4]  # a plateau of exact ties
    t = O.thresholds_equal_width(Xf.min(), Xf.max(), 50)
    got = OC.ecc_hard_batch(Xf, t)
    for i in range(2):
        np.testing.assert_array_equal(got[i], O.ecc_cellmax(Xf[i], t))
        np.testing.assert_array_equal(got[i], O.ecc_hard(Xf[i], t))


# ---- directional curves (tilted filtration) ----------------------------------


def test_tilt_zero_alpha_is_the_plain_curve_and_rounding_is_float32():
    rng = np.random.default_rng(5)
    X = rng.standard_normal((6, 7)).astype(np.float32)
    assert np.array_equal(O.tilt_field(X, [0.6, 0.8], 0.0), X)
    Y = O.tilt_field(X, [0.6, 0.8], 0.25)
    assert Y.dtype == np.float32
    # one vertex by hand, every operation rounded to float32
    a = np.float32(0.25) * np.array([0.6, 0.8], np.float32)
    want = np.float32(X[4, 5] + np.float32(np.float32(a[0] * np.float32(5)) + np.float32(a[1] * np.float32(4))))
    assert Y[4, 5] == want
    Z = rng.standard_normal((3, 4, 5)).astype(np.float32)
    W = O.tilt_field(Z, [0.1, 0.2, 0.3], 2.0)
    a = np.float32(2.0) * np.array([0.1, 0.2, 0.3], np.float32)
    t = np.float32(np.float32(np.float32(a[0] * np.float32(4)) + np.float32(a[1] * np.float32(3))) + np.float32(a[2] * np.float32(2)))
    assert W[2, 3, 4] == np.float32(Z[2, 3, 4] + t)


def test_directional_curve_of_a_flat_grid_is_a_ramp():
    # X = 0: the tilted field is strictly monotone along every axis, so one vertex
    # (the corner the direction points away from) carries c = 1 and the curve is 1
    # from the smallest value on -- for any direction without a zero component
    for shape, u in (((5, 6), [0.6, -0.8]), ((3, 4, 5), [-0.3, 0.5, 0.8])):
        X = np.zeros(shape, np.float32)
        Y = O.tilt_field(X, u, 1.0)
        c = O.coeff(Y)
        assert c.sum() == 1 and np.count_nonzero(c) == 1 and c.ravel()[np.argmin(Y)] == 1
        t = O.thresholds_equal_width(Y.min(), Y.max(), 9)
        assert np.array_equal(O.ecc_hard_dir(X[None], [u], 1.0, t)[0, 0], np.ones(9, np.int64))


def test_directional_curves_match_the_brute_force_count_on_the_tilted_field():
    rng = np.random.default_rng(11)
    for shape in ((5, 7), (3, 4, 5)):
        nd = len(shape)
        Xb = rng.integers(0, 4, size=(2,) + shape).astype(np.float32)
        U = rng.standard_normal((3, nd)).astype(np.float32)
        lo = min(O.tilt_field(x, u, 0.5).min() for x in Xb for u in U)
        hi = max(O.tilt_field(x, u, 0.5).max() for x in Xb for u in U)
        t = O.thresholds_equal_width(lo, hi, 13)
        got = O.ecc_hard_dir(Xb, U, 0.5, t)
        assert got.shape == (3, 2, 13)
        for k, u in enumerate(U):
            for i, x in enumerate(Xb):
                Y = O.tilt_field(x, u, 0.5)
                assert np.array_equal(got[k, i], O.ecc_bruteforce(Y, t))
                assert np.array_equal(got[k, i], O.ecc_cellmax(Y, t))


# ---- top-cell construction ------------------------------------------------------


def test_topcell_closed_forms():
    one = np.ones((1, 1), bool)
    assert O.euler_characteristic_topcells(one) == 1                    # a closed square
    assert O.euler_characteristic_topcells(np.ones((3, 4, 5), bool)) == 1
    ring = np.ones((3, 3), bool)
    ring[1, 1] = False
    assert O.euler_characteristic_topcells(ring) == 0                   # annulus
    diag = np.eye(2, dtype=bool)
    assert O.euler_characteristic_topcells(diag) == 1                   # corner contact joins (8-connectivity)
    assert O.euler_characteristic_mask(diag) == 2                       # ... where the vertex construction has two
    shell = np.ones((3, 3, 3), bool)
    shell[1, 1, 1] = False
    assert O.euler_characteristic_topcells(shell) == 2
    assert O.euler_characteristic_topcells(np.zeros((4, 4), bool)) == 0


@pytest.mark.parametrize("shape", [(1, 1), (1, 5), (4, 1), (3, 3), (5, 6), (2, 2, 2), (1, 3, 4), (3, 4, 5)])
def test_topcell_coefficients_reproduce_the_brute_force_curve(shape):
    rng = np.random.default_rng(sum(shape))
    for levels in (2, 3, 50):
        for _ in range(10):
            X = rng.integers(0, levels, size=shape).astype(np.float32)
            t = O.thresholds_levels(levels)
            c = O.coeff_top(X)
            assert c.sum() == 1                                         # the full box is contractible
            assert np.array_equal(O.ecc_top(X, t), O.ecc_top_bruteforce(X, t))


def test_topcell_coefficient_is_the_reversed_vertex_coefficient_in_the_interior():
    # away from the boundary: c_top(X) = (-1)^d c_vertex(-X) up to the tie-break, so on
    # grids without ties the two agree exactly there
    rng = np.random.default_rng(3)
    for shape in ((7, 8), (5, 6, 7)):
        X = rng.permutation(int(np.prod(shape))).reshape(shape).astype(np.float32)
        a = O.coeff_top(X)
        b = (-1) ** len(shape) * O.coeff(-X)
        inner = tuple(slice(1, -1) for _ in shape)
        assert np.array_equal(a[inner], b[inner])


# ---- superlevel filtration --------------------------------------------------------


def test_superlevel_closed_forms():
    t = np.array([0.0, 1.0, 2.0, 3.0])
    const = np.full((4, 5), 2.0)
    assert O.ecc_super_bruteforce(const, t).tolist() == [1, 1, 1, 0]        # one box until tau passes the value
    ramp = np.arange(12, dtype=np.float64).reshape(3, 4)
    tt = np.arange(13, dtype=np.float64)
    assert O.ecc_super_bruteforce(ramp, tt).tolist() == [1] * 12 + [0]      # a shrinking staircase, then nothing
    peaks = np.zeros((5, 5))
    peaks[1, 1] = peaks[3, 3] = 5.0
    peaks[1, 3] = 4.0
    assert O.ecc_super_bruteforce(peaks, np.array([0.0, 4.0, 5.0])).tolist() == [1, 3, 2]
    pit = np.ones((3, 3))
    pit[1, 1] = 0.0
    assert O.ecc_super_bruteforce(pit, np.array([0.0, 1.0])).tolist() == [1, 0]          # box, then a ring
    assert O.ecc_super_bruteforce(pit, np.array([0.0, 1.0]), top=True).tolist() == [1, 0]
    diag = np.eye(2)
    assert O.ecc_super_bruteforce(diag, np.array([1.0])).tolist() == [2]                 # two vertices
    assert O.ecc_super_bruteforce(diag, np.array([1.0]), top=True).tolist() == [1]       # two squares sharing a corner


@pytest.mark.parametrize("top", [False, True])
@pytest.mark.parametrize("shape", [(1, 1), (1, 5), (4, 1), (3, 3), (5, 6), (2, 2, 2), (1, 3, 4), (3, 4, 5)])
def test_superlevel_coefficients_reproduce_the_brute_force_curve(shape, top):
    rng = np.random.default_rng(sum(shape) + 100 * top)
    for levels in (2, 3, 50):
        for _ in range(8):
            X = rng.integers(0, levels, size=shape).astype(np.float32)
            t = O.thresholds_levels_super(levels)
            c = O.coeff_top(X, descending=True) if top else O.coeff(X, descending=True)
            assert c.sum() == 1
            got = O.ecc_super(X, t, top)
            assert got[0] == 1                                              # X >= 0 is the whole grid
            assert np.array_equal(got, O.ecc_super_bruteforce(X, t, top))
            # thresholds that leave points out on both sides
            t2 = np.array([1.0, levels / 2, levels - 1.5])
            assert np.array_equal(O.ecc_super(X, t2, top), O.ecc_super_bruteforce(X, t2, top))


@pytest.mark.parametrize("top", [False, True])
def test_superlevel_is_the_sublevel_curve_of_the_negated_grid(top):
    # {X >= tau} = {-X <= -tau}: the sublevel functions, pinned on their own, give the same numbers
    rng = np.random.default_rng(8)
    for shape in ((6, 7), (4, 5, 6)):
        X = rng.integers(-4, 5, size=shape).astype(np.float64)
        t = np.array([-3.0, -1.0, 0.0, 0.5, 2.0, 4.0])
        sub = (O.ecc_top_bruteforce if top else O.ecc_bruteforce)(-X, -t[::-1])[::-1]
        assert np.array_equal(O.ecc_super(X, t, top), sub)
        sub3 = (O.ecc_top if top else O.ecc_hard)(-X, -t[::-1])[::-1]
        assert np.array_equal(O.ecc_super(X, t, top), sub3)


def test_lower_thresholds_are_the_upper_ones_shifted_by_a_bin():
    up = O.thresholds_equal_width(-1.5, 2.25, 7)
    lowr = O.thresholds_lower(up, -1.5)
    assert lowr[0] == np.float32(-1.5) and np.array_equal(lowr[1:], up[:-1])
    x = np.array([-2.0, -1.5, -1.4, 2.25, 3.0, up[2], np.nextafter(up[2], -np.inf)])
    b = O.bin_index_super(x, lowr)
    assert b.tolist() == [-1, 0, 0, 6, 6, 3, 2]
