/*
 * CPU oracle for the hard Euler Characteristic Curve, plain C.
 * TEST INFRASTRUCTURE ONLY: never linked or loaded by the product library.
 *
 * Follows the per-vertex form of the curve (Eq. 3 of the paper):
 *     ECC(tau) = sum_p c(p) 1[X(p) <= tau]
 * with grid points as vertices, a cell present once all its vertices are
 * <= tau, and each cell charged to its last vertex under the total order
 *     q before p  <=>  X(q) < X(p), or X(q) == X(p) and index(q) < index(p).
 * c(p) = 1 - #edges + #squares - #cubes charged to p.  Cells must lie inside
 * the grid.  The curve is the inclusive prefix sum of the histogram of c(p)
 * over bin(X(p)) = min{ b : X(p) <= t_b }; points above t_{B-1} are dropped.
 *
 * It is written voxel by voxel with loops over cell offsets and their
 * sub-offsets, exactly as the definition reads.  OpenMP only splits the
 * outermost loop; it is the timed host baseline as it stands.
 *
 * Pinned by tests/test_oracle_hard.py against the numpy brute-force
 * V - E + F - C count, the cell-maximum histogram and the worked examples.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { OR_U8 = 0, OR_U16 = 1, OR_F32 = 2 };

static double load_value(const void* g, int dtype, int64_t i) {
  switch (dtype) {
    case OR_U8: return (double)((const uint8_t*)g)[i];
    case OR_U16: return (double)((const uint16_t*)g)[i];
    default: return (double)((const float*)g)[i];
  }
}

/* does the neighbour at offset (dz,dy,dx) exist and come before p ? */
static int before(const void* g, int dtype, int64_t D, int64_t H, int64_t W,
                  int64_t z, int64_t y, int64_t x, int dz, int dy, int dx) {
  int64_t qz = z + dz, qy = y + dy, qx = x + dx;
  if (qz < 0 || qz >= D || qy < 0 || qy >= H || qx < 0 || qx >= W) return 0;
  int64_t ip = (z * H + y) * W + x;
  int64_t iq = (qz * H + qy) * W + qx;
  double vp = load_value(g, dtype, ip), vq = load_value(g, dtype, iq);
  return vq < vp || (vq == vp && iq < ip);
}

static int coeff_at(const void* g, int dtype, int64_t D, int64_t H, int64_t W,
                    int64_t z, int64_t y, int64_t x) {
  int c = 1; /* the vertex */
  for (int oz = -1; oz <= 1; ++oz)
    for (int oy = -1; oy <= 1; ++oy)
      for (int ox = -1; ox <= 1; ++ox) {
        int dim = (oz != 0) + (oy != 0) + (ox != 0);
        if (dim == 0) continue;
        int owned = 1;
        /* every other vertex of the cell: sub-offsets s with s_a in {0, o_a} */
        for (int sz = 0; sz <= (oz != 0) && owned; ++sz)
          for (int sy = 0; sy <= (oy != 0) && owned; ++sy)
            for (int sx = 0; sx <= (ox != 0) && owned; ++sx) {
              if (!sz && !sy && !sx) continue;
              owned = before(g, dtype, D, H, W, z, y, x, sz * oz, sy * oy, sx * ox);
            }
        if (owned) c += (dim & 1) ? -1 : 1;
      }
  return c;
}

/* c(p) of one grid; 2D grids are passed with D = 1. */
int ecc_oracle_coeff(const void* grid, int dtype, int64_t D, int64_t H, int64_t W,
                     int8_t* c_out) {
#pragma omp parallel for schedule(static)
  for (int64_t zy = 0; zy < D * H; ++zy) {
    int64_t z = zy / H, y = zy % H;
    for (int64_t x = 0; x < W; ++x)
      c_out[(z * H + y) * W + x] = (int8_t)coeff_at(grid, dtype, D, H, W, z, y, x);
  }
  return 0;
}

static int bin_of(double v, const double* t, int bins) {
  /* min{ b : v <= t_b }, bins if none */
  int lo = 0, hi = bins;
  while (lo < hi) {
    int mid = (lo + hi) / 2;
    if (v <= t[mid]) hi = mid; else lo = mid + 1;
  }
  return lo;
}

/* curve[batch][bins] for a batch of grids sharing one threshold table */
int ecc_oracle_hard(const void* grid, int dtype, int64_t D, int64_t H, int64_t W,
                    int64_t batch, int bins, const double* t, int64_t* curve) {
  int64_t N = D * H * W;
  size_t esz = dtype == OR_U8 ? 1 : dtype == OR_U16 ? 2 : 4;
  for (int64_t b = 0; b < batch; ++b) {
    const void* g = (const char*)grid + (size_t)b * N * esz;
    int64_t* hist = curve + b * bins;
    memset(hist, 0, sizeof(int64_t) * bins);
#pragma omp parallel
    {
      int64_t* local = (int64_t*)calloc(bins + 1, sizeof(int64_t));
#pragma omp for schedule(static)
      for (int64_t zy = 0; zy < D * H; ++zy) {
        int64_t z = zy / H, y = zy % H;
        for (int64_t x = 0; x < W; ++x) {
          int c = coeff_at(g, dtype, D, H, W, z, y, x);
          if (c) local[bin_of(load_value(g, dtype, (z * H + y) * W + x), t, bins)] += c;
        }
      }
#pragma omp critical
      for (int i = 0; i < bins; ++i) hist[i] += local[i];
      free(local);
    }
    for (int i = 1; i < bins; ++i) hist[i] += hist[i - 1];
  }
  return 0;
}

int ecc_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
