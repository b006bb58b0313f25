"""Seeded synthetic inputs shared by the tests, the benchmark and the CPU oracle.

This module holds data generators only: random draws and a library smoothing
filter.  It contains none of the method's arithmetic (no coefficient, no
binning, no sigmoid), so both the HIP path and the independent CPU oracle may
consume its arrays without sharing any code of the method itself.

The paper benchmarks on unspecified "synthetic grids" (Experiments section,
Tables 1 and 2); these generators are the stand-ins, with the shapes, dtypes
and value distributions of the five workloads this build is measured on:

  C1  one 2D 256x256 uint8 grid, i.i.d. uniform levels 0..255
  C2  16 2D 4096x4096 float32 Gaussian random fields (white noise smoothed
      with a Gaussian of sigma = 4 px, periodic wrap)
  C3  one 3D 256^3 uint16 volume, i.i.d. uniform levels 0..4095
  C4  one 3D 512^3 float32 Gaussian random field (sigma = 3 voxels)
  C5  32 2D 512x512 float32 Gaussian random fields (sigma = 4 px)

Every generator uses numpy's PCG64 through ``default_rng``; item ``i`` of a
batch with base seed ``s`` uses seed ``s * 1000 + i``.
"""
from __future__ import annotations

import numpy as np

SEED_C1 = 1001
SEED_C2 = 1002
SEED_C3 = 1003
SEED_C4 = 1004
SEED_C5 = 1005


def iid_levels(shape, levels: int, dtype, seed: int) -> np.ndarray:
    """i.i.d. uniform integer levels 0..levels-1 (maximal neighbour disorder)."""
    rng = np.random.default_rng(seed)
    return rng.integers(0, levels, size=tuple(shape), dtype=dtype)


def grf(shape, sigma: float, seed: int) -> np.ndarray:
    """float32 N(0,1) white noise smoothed by a Gaussian of width ``sigma``."""
    from scipy.ndimage import gaussian_filter

    rng = np.random.default_rng(seed)
    noise = rng.standard_normal(size=tuple(shape), dtype=np.float32)
    out = gaussian_filter(noise, sigma=sigma, mode="wrap", truncate=4.0)
    return np.ascontiguousarray(out, dtype=np.float32)


def grf_batch(batch: int, shape, sigma: float, seed: int) -> np.ndarray:
    """``batch`` independent smoothed fields stacked on a leading axis."""
    out = np.empty((batch,) + tuple(shape), dtype=np.float32)
    for i in range(batch):
        out[i] = grf(shape, sigma, seed * 1000 + i)
    return out


def config_c1(n: int = 256) -> np.ndarray:
    return iid_levels((n, n), 256, np.uint8, SEED_C1 * 1000)


def config_c2(batch: int = 16, n: int = 4096) -> np.ndarray:
    return grf_batch(batch, (n, n), 4.0, SEED_C2)


def config_c3(n: int = 256) -> np.ndarray:
    return iid_levels((n, n, n), 4096, np.uint16, SEED_C3 * 1000)


def config_c4(n: int = 512) -> np.ndarray:
    return grf((n, n, n), 3.0, SEED_C4 * 1000)


def config_c5(batch: int = 32, n: int = 512) -> np.ndarray:
    return grf_batch(batch, (n, n), 4.0, SEED_C5)


def soft_params_c5(grid: np.ndarray, T: int = 128):
    """Parameters of the soft workload: thresholds evenly spaced over the
    batch-global [min, max] of the grid (float64 linspace rounded to float32),
    sharpness 20, unit direction at angle 0.3 rad given as (u_x, u_y) with x
    the fastest (column) axis, scale 0.01 on 0-based pixel coordinates."""
    lo = float(grid.min())
    hi = float(grid.max())
    tau = np.linspace(lo, hi, T, dtype=np.float64).astype(np.float32)
    u = np.array([np.cos(0.3), np.sin(0.3)], dtype=np.float64).astype(np.float32)
    return dict(tau=tau, u=u, alpha=np.float32(0.01), lam=np.float32(20.0))


def upstream_grad(batch: int, T: int, seed: int = SEED_C5) -> np.ndarray:
    """Seeded N(0,1) upstream gradient g[batch, T] for backward parity."""
    rng = np.random.default_rng(seed * 1000 + 999)
    return rng.standard_normal(size=(batch, T), dtype=np.float32)
