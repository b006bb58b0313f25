// Soft ECC: reduction of the per-unit partial sums of the fused kernels, shared by the 2D and the
// 3D path.  In float64 and in a fixed order, so results are run-to-run identical.
//
// A wave unit of a sweep leaves, per threshold, up to 2 + NC floats: chi (Eq. 6 of the paper), A0 (the sum
// of c sigma (1 - sigma): Eq. 9 up to the factor lambda) and A_1 .. A_NC (the same sum weighted with
// the vertex coordinates relative to the unit's origin: Eq. 10 up to -alpha lambda and the origin's
// share, which is added here).  A lone large image or volume has thousands of units, so the sum
// is split: block (x = group of 64 thresholds, y = item, z = slice) of 16 waves adds the units of
// its slice -- wave w takes units begin + w, begin + w + 16, ... in order, then wave 0 adds the 16
// sums in order -- and, when there is more than one slice, leaves the slice's sums in `mid`, which
// a second kernel adds in slice order.
#pragma once
#include "ecc_device.h"
#include "ecc_internal.h"

namespace ecc {

constexpr int kRedWaves = 16, kRedSlices = 64;
constexpr int kRedMaxSums = 5;  // chi, A0, three coordinates

// where the results go; a null pointer skips that output.  hdr (may be null): the last kernel
// of the saving forward pass's reduction writes the state's header and raises its generation
struct RedOut {
  float* chi;
  float* dtau;
  float* du;
  SoftStateHeader* hdr;
  unsigned* gen;
  SoftStateHeader stamp;
};

// STRIDE: floats per (unit, threshold) in `partial`; CHI: the first of them is chi; NC: coordinate
// sums behind A0 (-1: no A0 either, the forward pass alone)
template <bool CHI, int NC>
struct RedLayout {
  static constexpr int kA = CHI ? 1 : 0;                            // where A0 sits
  static constexpr int kSums = (CHI ? 1 : 0) + (NC >= 0 ? 1 + NC : 0);
};

template <bool CHI, int NC>
__device__ __forceinline__ void red_finish(const double (&r)[kRedMaxSums], int64_t k, float alpha, float lambda,
                                           const RedOut& o) {
  constexpr int A = RedLayout<CHI, NC>::kA;
  if constexpr (CHI) o.chi[k] = (float)r[0];
  if constexpr (NC >= 0) {
    // dchi_dtau = lambda sum A0;  dchi_du = -alpha lambda sum (origin * A0 + A_coordinates)
    if (o.dtau) o.dtau[k] = (float)((double)lambda * r[A]);
    if (o.du)
      for (int c = 0; c < NC; ++c) o.du[k * NC + c] = (float)(-(double)alpha * (double)lambda * r[A + 1 + c]);
  }
}
__device__ __forceinline__ void red_stamp(const RedOut& o) {
  if (o.hdr && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0) {
    *o.hdr = o.stamp;
    *o.gen = *o.gen + 1u;
  }
}

// Origin: unit -> origin of its coordinates, `void operator()(int unit, int (&o)[3]) const`
template <int STRIDE, bool CHI, int NC, typename Origin>
__global__ __launch_bounds__(kRedWaves * kWave) void soft_reduce_kernel(const float* __restrict__ partial, int units,
                                                                        int per_slice, int T, float alpha, float lambda,
                                                                        Origin origin, double* __restrict__ mid,
                                                                        RedOut out) {
  constexpr int NS = RedLayout<CHI, NC>::kSums, A = RedLayout<CHI, NC>::kA;
  __shared__ double red[NS][kRedWaves][kWave];
  const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
  const int j = blockIdx.x * kWave + lane;
  const int item = blockIdx.y, slice = blockIdx.z;
  const int begin = slice * per_slice, end = min(units, begin + per_slice);
  double s[kRedMaxSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
  if (j < T) {
    for (int q = begin + wv; q < end; q += kRedWaves) {
      float e[STRIDE];
      const float* p = partial + (((int64_t)item * units + q) * T + j) * STRIDE;
      if constexpr (STRIDE == 4) {
        const float4 f = *reinterpret_cast<const float4*>(p);
        e[0] = f.x, e[1] = f.y, e[2] = f.z, e[3] = f.w;
      } else {
#pragma unroll
        for (int c = 0; c < STRIDE; ++c) e[c] = p[c];
      }
      if constexpr (CHI) s[0] += (double)e[0];
      if constexpr (NC >= 0) {
        int o[3];
        origin(q, o);
        const double a0 = (double)e[A];
        s[A] += a0;
#pragma unroll
        for (int c = 0; c < NC; ++c) s[A + 1 + c] += (double)o[c] * a0 + (double)e[A + 1 + c];
      }
    }
  }
  for (int c = 0; c < NS; ++c) red[c][wv][lane] = s[c];
  if (gridDim.z == 1) red_stamp(out);
  __syncthreads();
  if (wv == 0 && j < T) {
    double r[kRedMaxSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
    for (int c = 0; c < NS; ++c) {
      r[c] = red[c][0][lane];
      for (int w = 1; w < kRedWaves; ++w) r[c] += red[c][w][lane];
    }
    if (gridDim.z == 1) {
      red_finish<CHI, NC>(r, (int64_t)item * T + j, alpha, lambda, out);
    } else {
      for (int c = 0; c < NS; ++c) mid[(((int64_t)item * gridDim.z + slice) * T + j) * NS + c] = r[c];
    }
  }
}

// wave w adds slices w, w + 16, ... in order, wave 0 adds the 16 sums in order
template <bool CHI, int NC>
__global__ __launch_bounds__(kRedWaves * kWave) void soft_reduce_final_kernel(const double* __restrict__ mid, int slices,
                                                                              int T, float alpha, float lambda,
                                                                              RedOut out) {
  constexpr int NS = RedLayout<CHI, NC>::kSums;
  __shared__ double red[NS][kRedWaves][kWave];
  const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
  const int j = blockIdx.x * kWave + lane, item = blockIdx.y;
  double s[kRedMaxSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
  if (j < T)
    for (int sl = wv; sl < slices; sl += kRedWaves)
      for (int c = 0; c < NS; ++c) s[c] += mid[(((int64_t)item * slices + sl) * T + j) * NS + c];
  for (int c = 0; c < NS; ++c) red[c][wv][lane] = s[c];
  red_stamp(out);
  __syncthreads();
  if (wv == 0 && j < T) {
    double r[kRedMaxSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
    for (int c = 0; c < NS; ++c) {
      r[c] = red[c][0][lane];
      for (int w = 1; w < kRedWaves; ++w) r[c] += red[c][w][lane];
    }
    red_finish<CHI, NC>(r, (int64_t)item * T + j, alpha, lambda, out);
  }
}

// bytes of `mid` for a batch and T thresholds (the most any of the reductions needs)
static inline size_t soft_reduce_mid_bytes(int64_t batch, int T) {
  return (size_t)batch * kRedSlices * (size_t)T * kRedMaxSums * sizeof(double);
}

template <int STRIDE, bool CHI, int NC, typename Origin>
static void launch_soft_reduce(const float* partial, double* mid, int units, int64_t batch, int T, float alpha,
                               float lambda, const Origin& origin, const RedOut& out, hipStream_t st) {
  // slices the units are split into (about 64 units per slice at least), and units per slice
  int slices = units / (4 * kRedWaves);
  slices = slices < 1 ? 1 : (slices > kRedSlices ? kRedSlices : slices);
  const int per = (units + slices - 1) / slices;
  slices = (units + per - 1) / per;
  const unsigned tg = (unsigned)((T + kWave - 1) / kWave);
  hipLaunchKernelGGL((soft_reduce_kernel<STRIDE, CHI, NC, Origin>), dim3(tg, (unsigned)batch, (unsigned)slices),
                     dim3(kRedWaves * kWave), 0, st, partial, units, per, T, alpha, lambda, origin, mid, out);
  if (slices > 1)
    hipLaunchKernelGGL((soft_reduce_final_kernel<CHI, NC>), dim3(tg, (unsigned)batch), dim3(kRedWaves * kWave), 0, st, mid,
                       slices, T, alpha, lambda, out);
}

}  // namespace ecc
