"""CPU oracle for the Euler Characteristic Curve path.  TEST INFRASTRUCTURE ONLY.

Plain, slow, float64/integer numpy written from the paper's definitions; it
shares no code with the HIP library and must never be imported by the product
package.  Only tests, the smoke check and the benchmark's CPU-baseline leg use
it.

Convention (the paper's Background section only says "cubical complex:
vertices, edges, faces, cubes"; this build fixes the rest):
  * grid points are the vertices of the complex;
  * an elementary cell (edge = 2 axis-adjacent points, square = 2x2 points,
    cube = 2x2x2 points, entirely inside the grid, no wrap-around) is present
    at threshold tau iff ALL its vertices have X <= tau  (Eq. 1);
  * ECC(tau) = V - E + F - C of the present cells  (Eq. 2);
  * per-vertex form (Eq. 3): ECC(tau) = sum_p c(p) 1[X(p) <= tau], where each
    cell is charged to its last-entering vertex under the total order
    q < p  <=>  X(q) < X(p) or (X(q) == X(p) and index(q) < index(p)),
    index = C-order linear index inside one grid, and c(p) is the alternating
    count 1 - #edges + #squares - #cubes of the cells charged to p.

Three independent derivations of the hard curve are given so that each pins
the others: ``ecc_bruteforce`` (Eq. 1-2 literally), ``ecc_cellmax`` (each cell
enters at the maximum of its vertices) and ``coeff`` + ``ecc_from_coeff``
(Eq. 3).  The soft functions evaluate Eq. 6 and Eq. 8-10 in float64.

Pins (tests/test_oracle_*.py): a hand-worked 3x3 example and its curve, a
4x4 frame example, closed forms (ramp, constant, checkerboard, solid shapes
with known Euler characteristic), invariants (ECC = 0 below the minimum, = 1
at the maximum, sum of c = 1), exhaustive agreement of the three derivations
on every three-level 3x3 grid, the expectation formula for i.i.d. grids, and
for the soft part the 1x1 closed form, limits in tau and lambda, finite
differences and the exact identities linking Eq. 8, 9 and 10.
Parity unpinned: none.
"""
from __future__ import annotations

import itertools

import numpy as np
from scipy.special import expit

# ----------------------------------------------------------------------------
# thresholds and binning
# ----------------------------------------------------------------------------


def thresholds_levels(bins: int) -> np.ndarray:
    """One bin per integer level: t_b = b."""
    return np.arange(bins, dtype=np.float64)


def thresholds_equal_width(lo: float, hi: float, bins: int) -> np.ndarray:
    """``bins`` right-closed equal-width bins over [lo, hi].

    t_b = float32( lo + (b+1) * (hi-lo) / bins ) evaluated in float64, and the
    last threshold is ``hi`` itself so the whole grid is inside the last
    sublevel set.  Returned widened to float64.
    """
    lo = np.float64(lo)
    hi = np.float64(hi)
    b1 = np.arange(1, bins + 1, dtype=np.float64)
    t = (lo + (b1 * (hi - lo)) / np.float64(bins)).astype(np.float32)
    t[bins - 1] = np.float32(hi)
    return t.astype(np.float64)


def bin_index(x: np.ndarray, t: np.ndarray) -> np.ndarray:
    """bin(x) = min{ b : x <= t_b };  equals len(t) when x is above every
    threshold (the point is in no sublevel set and is dropped)."""
    return np.searchsorted(t, np.asarray(x, dtype=np.float64), side="left")


# ----------------------------------------------------------------------------
# O1: Eq. 1-2 literally
# ----------------------------------------------------------------------------


def _shifted_and(m: np.ndarray, axes) -> np.ndarray:
    """AND of the mask over the 2^k corners of cells spanning ``axes``."""
    out = m
    for ax in axes:
        n = out.shape[ax]
        a = np.take(out, range(0, n - 1), axis=ax)
        b = np.take(out, range(1, n), axis=ax)
        out = a & b
    return out


def euler_characteristic_mask(m: np.ndarray) -> int:
    """chi of the cubical complex spanned by the True vertices of ``m``."""
    nd = m.ndim
    chi = 0
    for k in range(nd + 1):
        for axes in itertools.combinations(range(nd), k):
            chi += (-1) ** k * int(_shifted_and(m, axes).sum())
    return chi


def ecc_bruteforce(X: np.ndarray, t: np.ndarray) -> np.ndarray:
    Xd = np.asarray(X, dtype=np.float64)
    return np.array([euler_characteristic_mask(Xd <= tb) for tb in t], dtype=np.int64)


# ----------------------------------------------------------------------------
# O2: every cell enters at the maximum of its vertices
# ----------------------------------------------------------------------------


def _shifted_max(v: np.ndarray, axes) -> np.ndarray:
    out = v
    for ax in axes:
        n = out.shape[ax]
        a = np.take(out, range(0, n - 1), axis=ax)
        b = np.take(out, range(1, n), axis=ax)
        out = np.maximum(a, b)
    return out


def ecc_cellmax(X: np.ndarray, t: np.ndarray) -> np.ndarray:
    Xd = np.asarray(X, dtype=np.float64)
    nb = len(t)
    hist = np.zeros(nb + 1, dtype=np.int64)
    for k in range(Xd.ndim + 1):
        for axes in itertools.combinations(range(Xd.ndim), k):
            b = bin_index(_shifted_max(Xd, axes).ravel(), t)
            hist += (-1) ** k * np.bincount(b, minlength=nb + 1).astype(np.int64)
    return np.cumsum(hist[:nb])


# ----------------------------------------------------------------------------
# O3: per-vertex coefficient (Eq. 3)
# ----------------------------------------------------------------------------


def _precedes(X: np.ndarray, descending: bool = False):
    """dict offset -> boolean array: neighbour p+offset exists and precedes p.
    descending: the filtration runs from high values to low ones (superlevel sets),
    so larger values come first; ties still go by the index."""
    nd = X.ndim
    Xd = np.asarray(X, dtype=np.float64)
    if not np.all(np.isfinite(Xd)):
        raise ValueError("grid must be finite")
    if descending:
        Xd = -Xd
    idx = np.arange(Xd.size, dtype=np.int64).reshape(Xd.shape)
    Xp = np.pad(Xd, 1, mode="constant", constant_values=np.inf)
    Ip = np.pad(idx, 1, mode="constant", constant_values=np.iinfo(np.int64).max)
    core = tuple(slice(1, 1 + n) for n in Xd.shape)
    prec = {}
    for s in itertools.product((-1, 0, 1), repeat=nd):
        if not any(s):
            continue
        sl = tuple(slice(1 + d, 1 + d + n) for d, n in zip(s, Xd.shape))
        Xq, Iq = Xp[sl], Ip[sl]
        prec[s] = (Xq < Xp[core]) | ((Xq == Xp[core]) & (Iq < Ip[core]))
    return prec


def coeff(X: np.ndarray, descending: bool = False) -> np.ndarray:
    """c(p) of one 2D or 3D grid, int8, same shape as X."""
    nd = X.ndim
    prec = _precedes(X, descending)
    c = np.ones(X.shape, dtype=np.int64)  # the vertex itself
    for o in itertools.product((-1, 0, 1), repeat=nd):
        dim = sum(1 for a in o if a)
        if dim == 0:
            continue
        owned = np.ones(X.shape, dtype=bool)
        for s in itertools.product(*[(0, a) if a else (0,) for a in o]):
            if any(s):
                owned &= prec[s]
        c += (-1) ** dim * owned
    return c.astype(np.int8)


def ecc_from_coeff(X: np.ndarray, c: np.ndarray, t: np.ndarray) -> np.ndarray:
    nb = len(t)
    b = bin_index(np.asarray(X).ravel(), t)
    hist = np.zeros(nb + 1, dtype=np.int64)
    np.add.at(hist, b, c.ravel().astype(np.int64))
    return np.cumsum(hist[:nb])


def ecc_hard(X: np.ndarray, t: np.ndarray) -> np.ndarray:
    """Hard curve of one grid through Eq. 3."""
    return ecc_from_coeff(X, coeff(X), t)


def ecc_hard_batch(Xb: np.ndarray, t: np.ndarray) -> np.ndarray:
    return np.stack([ecc_hard(x, t) for x in Xb])


# ----------------------------------------------------------------------------
# top-cell construction: grid points are the top-dimensional cells (pixels /
# voxels as squares / cubes); a lower cell is present as soon as one of the top
# cells around it is.  (The Background section leaves the construction open; the
# vertex construction above is the one the rest of this file uses.)
# ----------------------------------------------------------------------------


def _any_shifted(m: np.ndarray, axes) -> np.ndarray:
    """Cells spanned between neighbouring top cells along `axes`: present when ANY
    of the 2^k top cells around them is (m padded with False outside the grid)."""
    out = np.pad(m, [(1, 1) if a in axes else (0, 0) for a in range(m.ndim)], constant_values=False)
    for a in axes:
        lo = [slice(None)] * m.ndim
        hi = [slice(None)] * m.ndim
        lo[a], hi[a] = slice(0, -1), slice(1, None)
        out = out[tuple(lo)] | out[tuple(hi)]
    return out


def euler_characteristic_topcells(m: np.ndarray) -> int:
    """chi of the closed union of the unit squares / cubes marked in m: cells of
    codimension k are indexed by the top cells shifted half a step along k axes."""
    import itertools
    d = m.ndim
    chi = 0
    for k in range(d + 1):
        for axes in itertools.combinations(range(d), k):
            chi += (-1) ** (d - k) * int(_any_shifted(m, axes).sum())
    return chi


def ecc_top_bruteforce(X: np.ndarray, t: np.ndarray) -> np.ndarray:
    return np.array([euler_characteristic_topcells(X <= tb) for tb in t], dtype=np.int64)


def coeff_top(X: np.ndarray, descending: bool = False) -> np.ndarray:
    """Per-top-cell coefficient: every cell is charged to the FIRST top cell around
    it (X, then C-order index).  That is the vertex coefficient of the reversed
    order with everything outside the grid coming before, times (-1)^d.
    descending: superlevel filtration, larger values come first."""
    X = np.asarray(X)
    d = X.ndim
    idx = np.arange(X.size, dtype=np.int64).reshape(X.shape)
    big = -X.astype(np.float64) if descending else X.astype(np.float64)
    c = np.zeros(X.shape, dtype=np.int64)
    import itertools
    pad_v = np.pad(big, 1, constant_values=np.inf)        # outside: never first
    pad_i = np.pad(idx, 1, constant_values=-1)
    centre = tuple(slice(1, -1) for _ in range(d))

    def first_among(offsets):
        """p is the first of the top cells p + s, s over all sub-offsets of `offsets`."""
        ok = np.ones(X.shape, bool)
        for s in itertools.product(*[(0, o) if o else (0,) for o in offsets]):
            if not any(s):
                continue
            sl = tuple(slice(1 + si, 1 + si + n) for si, n in zip(s, X.shape))
            qv, qi = pad_v[sl], pad_i[sl]
            p_first = (big < qv) | ((big == qv) & (idx < qi))
            ok &= p_first
        return ok

    for o in itertools.product((-1, 0, 1), repeat=d):
        k = sum(1 for v in o if v)                      # codimension of the cell between p and p + o
        c += (-1) ** (d - k) * first_among(o)
    return c


def ecc_top(X: np.ndarray, t: np.ndarray) -> np.ndarray:
    return ecc_from_coeff(X, coeff_top(X), t)


def ecc_top_batch(Xb: np.ndarray, t: np.ndarray) -> np.ndarray:
    return np.stack([ecc_top(x, t) for x in Xb])


# ----------------------------------------------------------------------------
# superlevel filtration: Omega^tau = {p : X(p) >= tau} in place of Eq. 1, for
# either construction.  The curve is read at the LOWER edges of the bins,
# t'_0 = lo and t'_b = t_{b-1}, so that its first entry is the whole grid.
# ----------------------------------------------------------------------------


def thresholds_lower(t_upper: np.ndarray, lo: float) -> np.ndarray:
    """Lower bin edges that go with the upper edges t_upper of the same bins:
    float32(lo), then t_upper without its last entry."""
    return np.concatenate([[np.float64(np.float32(lo))], np.asarray(t_upper, dtype=np.float64)[:-1]])


def thresholds_levels_super(bins: int) -> np.ndarray:
    """Integer grids without a range: t'_b = b (X >= b)."""
    return np.arange(bins, dtype=np.float64)


def bin_index_super(x: np.ndarray, t: np.ndarray) -> np.ndarray:
    """max{ b : t_b <= x }; -1 when x is below every threshold (in no superlevel set)."""
    return np.searchsorted(t, np.asarray(x, dtype=np.float64), side="right") - 1


def ecc_super_bruteforce(X: np.ndarray, t: np.ndarray, top: bool = False) -> np.ndarray:
    chi = euler_characteristic_topcells if top else euler_characteristic_mask
    Xd = np.asarray(X, dtype=np.float64)
    return np.array([chi(Xd >= tb) for tb in t], dtype=np.int64)


def ecc_super(X: np.ndarray, t: np.ndarray, top: bool = False) -> np.ndarray:
    """Superlevel curve through the per-point coefficients of the descending order:
    a point with t_b <= X(p) is in the sets of thresholds 0 .. b."""
    c = coeff_top(X, descending=True) if top else coeff(X, descending=True)
    nb = len(t)
    b = bin_index_super(np.asarray(X).ravel(), t)
    hist = np.zeros(nb + 1, dtype=np.int64)          # slot nb collects the dropped points (b = -1)
    np.add.at(hist, b, c.ravel().astype(np.int64))
    return np.cumsum(hist[:nb][::-1])[::-1]


def ecc_super_batch(Xb: np.ndarray, t: np.ndarray, top: bool = False) -> np.ndarray:
    return np.stack([ecc_super(x, t, top) for x in Xb])


# ----------------------------------------------------------------------------
# directional hard ECC: the curve of the tilted field (Background: the Euler
# characteristic transform sweeps a shape along directions; Eq. 6 tilts the
# filtration by alpha <u, p>)
# ----------------------------------------------------------------------------


def tilt_field(X: np.ndarray, u, alpha) -> np.ndarray:
    """Y(p) = X(p) + alpha <u, p> in float32, p = (x, y[, z]) 0-based with x the
    fastest axis.  The float32 operations and their order are part of the
    definition (the order on vertices depends on every rounding):
        a_d = fl(alpha * u_d);  t = fl(fl(a_x x) + fl(a_y y));  [t = fl(t + fl(a_z z));]
        Y = fl(X + t).
    """
    X = np.asarray(X, dtype=np.float32)
    u = np.asarray(u, dtype=np.float32)
    a = (np.float32(alpha) * u).astype(np.float32)
    nd = X.ndim
    shape = X.shape
    xs = np.arange(shape[-1], dtype=np.float32)
    ys = np.arange(shape[-2], dtype=np.float32)
    t = (a[0] * xs)[None, :] + (a[1] * ys)[:, None]          # float32 throughout
    if nd == 3:
        zs = np.arange(shape[0], dtype=np.float32)
        t = t[None, :, :] + (a[2] * zs)[:, None, None]
    assert t.dtype == np.float32
    return (X + t).astype(np.float32)


def ecc_hard_dir(Xb: np.ndarray, U, alpha, t: np.ndarray) -> np.ndarray:
    """Directional curves [ndir, batch, bins]: hard ECC of the tilted fields."""
    U = np.asarray(U, dtype=np.float32).reshape(-1, Xb.ndim - 1)
    return np.stack([np.stack([ecc_hard(tilt_field(x, u, alpha), t) for x in Xb]) for u in U])


# ----------------------------------------------------------------------------
# soft single-direction ECC (Eq. 6) and its derivatives (Eq. 8-10)
# ----------------------------------------------------------------------------


def coordinates(shape):
    """Integer 0-based coordinates p = (x, y[, z]) with x the fastest axis;
    returns an array [N, ndim] in C order of the grid."""
    axes = np.meshgrid(*[np.arange(n, dtype=np.float64) for n in shape], indexing="ij")
    # meshgrid order is slowest-first; p lists the fastest axis first
    return np.stack([a.ravel() for a in axes[::-1]], axis=1)


def _z(X, u, alpha, tau):
    Xd = np.asarray(X, dtype=np.float64)
    P = coordinates(Xd.shape)
    y = Xd.ravel() + np.float64(alpha) * (P @ np.asarray(u, dtype=np.float64))
    return np.asarray(tau, dtype=np.float64)[:, None] - y[None, :], P


def soft_fwd(X, u, alpha, tau, lam, c=None) -> np.ndarray:
    """chi_{lambda,u}(tau_j) for one grid, float64 [T]  (Eq. 6)."""
    if c is None:
        c = coeff(X)
    cd = c.ravel().astype(np.float64)
    out = np.empty(len(tau), dtype=np.float64)
    tau = np.asarray(tau, dtype=np.float64)
    for j0 in range(0, len(tau), 16):  # rows are independent; chunked for memory only
        z, _ = _z(X, u, alpha, tau[j0:j0 + 16])
        out[j0:j0 + 16] = expit(np.float64(lam) * z) @ cd
    return out


def soft_bwd(X, u, alpha, tau, lam, g=None, c=None):
    """Derivatives of Eq. 6 for one grid, float64.

    Returns (grad_X, dchi_dtau, dchi_du):
      grad_X[p]      = sum_j g_j * ( -c(p) sigma'(z_pj) )          (Eq. 8 contracted with g)
      dchi_dtau[j]   = sum_p c(p) sigma'(z_pj)                     (Eq. 9)
      dchi_du[j, :]  = -alpha sum_p c(p) sigma'(z_pj) p            (Eq. 10)
    with sigma'(z) = lambda sigma(z) (1 - sigma(z)).  g defaults to ones.
    """
    if c is None:
        c = coeff(X)
    tau = np.asarray(tau, dtype=np.float64)
    T = len(tau)
    g = np.ones(T, dtype=np.float64) if g is None else np.asarray(g, dtype=np.float64)
    cd = c.ravel().astype(np.float64)
    lam = np.float64(lam)
    grad_X = np.zeros(cd.size, dtype=np.float64)
    dtau = np.empty(T, dtype=np.float64)
    du = np.empty((T, np.asarray(X).ndim), dtype=np.float64)
    for j0 in range(0, T, 16):
        z, P = _z(X, u, alpha, tau[j0:j0 + 16])
        s = expit(lam * z)
        ds = lam * s * (1.0 - s)
        dtau[j0:j0 + 16] = ds @ cd
        du[j0:j0 + 16] = -np.float64(alpha) * ((ds * cd[None, :]) @ P)
        grad_X += -cd * (g[j0:j0 + 16] @ ds)
    return grad_X.reshape(np.asarray(X).shape), dtau, du


def coeff_tilted(X, u, alpha) -> np.ndarray:
    """c(p) of the tilted field (the soft curve then tends to the directional hard curve
    as lambda grows; with the coefficient of X itself it tends to no Euler characteristic)."""
    return coeff(tilt_field(X, u, alpha))


def soft_fwd_batch(Xb, u, alpha, tau, lam):
    return np.stack([soft_fwd(x, u, alpha, tau, lam) for x in Xb])


def soft_bwd_batch(Xb, u, alpha, tau, lam, G=None):
    gx, dt, du = [], [], []
    for i, x in enumerate(Xb):
        a, b, c_ = soft_bwd(x, u, alpha, tau, lam, None if G is None else G[i])
        gx.append(a)
        dt.append(b)
        du.append(c_)
    return np.stack(gx), np.stack(dt), np.stack(du)
