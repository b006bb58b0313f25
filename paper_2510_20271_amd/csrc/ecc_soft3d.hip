// Soft single-direction ECC for 3D grids, fused into the tube sweep of
// ecc_sweep3d.h: forward (Eq. 6 of the paper) and derivatives (Eq. 8-10).
//
// As in 2D, only the critical vertices (c != 0) carry a term.  The tube sweep
// finds them and queues (position, c); when 64 are drained together each lane
// fetches one value, forms y = X(p) + alpha <u,p> in float64 and parks the entry
// in a small LDS stage, and then every lane runs over the staged entries for the
// thresholds it owns (tau_l, tau_{l+64}, ...; T <= 256): the sums over p of
// Eq. 6 / Eq. 9 / Eq. 10 need no cross-lane reduction, the contraction of Eq. 8
// with the upstream gradient is a fixed-order sum over the lanes.  grad_X is
// cleared by a fill kernel first and written at the critical vertices only.
// Each wave leaves its partial sums in the workspace; a second kernel adds them
// in a fixed order in float64, so results are run-to-run identical.
#include "ecc_sweep3d.h"

#include <cstdlib>

namespace ecc {

constexpr int kSoft3TL = 4;  // thresholds per lane

__device__ __forceinline__ float soft3_exp_neg(float z, float kneg) {
  // exp(-lambda z) = 2^(kneg z); clamped so the result stays finite
  return __builtin_amdgcn_exp2f(fminf(kneg * z, 126.0f));
}

struct Soft3Entry {
  double y;  // X(p) + alpha <u,p>
  float c;
  int x, yy, z;
  unsigned inpl;  // yy * W + x
  int pad;
};

struct Soft3Common {
  static constexpr bool kTrackRange = false;
  double ux, uy, uz, alpha;
  double tj[kSoft3TL];  // this lane's thresholds
  int nt;               // threshold slots in use: ceil(T / 64)
  float kneg;
  int W;
  int oz;             // first plane of the wave's segment
  Soft3Entry* stage;  // wave-private LDS, 64 entries
  __device__ __forceinline__ void init(const float* u, float alpha_, const float* tau, int T, float kneg_, int W_,
                                       Soft3Entry* stage_) {
    ux = (double)u[0];
    uy = (double)u[1];
    uz = (double)u[2];
    alpha = (double)alpha_;
    nt = (T + kWave - 1) / kWave;
    kneg = kneg_;
    W = W_;
    stage = stage_;
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int t = 0; t < kSoft3TL; ++t) {
      const int j = lane + kWave * t;
      tj[t] = j < T ? (double)tau[j] : 0.0;
    }
  }
  // lane i < n parks its entry
  __device__ __forceinline__ void park(int n, float v, int c, unsigned inpl, unsigned zrel) const {
    const int lane = threadIdx.x & (kWave - 1);
    if (lane < n) {
      Soft3Entry e;
      e.yy = (int)(inpl / (unsigned)W);
      e.x = (int)(inpl - (unsigned)e.yy * (unsigned)W);
      e.z = oz + (int)zrel;
      e.y = (double)v + alpha * ((ux * (double)e.x + uy * (double)e.yy) + uz * (double)e.z);
      e.c = (float)c;
      e.inpl = inpl;
      e.pad = 0;
      stage[lane] = e;
    }
  }
};

struct Soft3FwdSink : Soft3Common {
  float acc[kSoft3TL];
  __device__ __forceinline__ void take(int n, float v, int c, unsigned inpl, unsigned zrel) {
    park(n, v, c, inpl, zrel);
    for (int e = 0; e < n; ++e) {
      const double y = stage[e].y;
      const float cf = stage[e].c;
#pragma unroll
      for (int t = 0; t < kSoft3TL; ++t) {
        if (t < nt) {  // wave-uniform
          const float z = (float)(tj[t] - y);
          const float ex = soft3_exp_neg(z, kneg);
          acc[t] += cf * __builtin_amdgcn_rcpf(1.0f + ex);
        }
      }
    }
  }
};

struct Soft3BwdSink : Soft3Common {
  float a0[kSoft3TL], ax[kSoft3TL], ay[kSoft3TL], az[kSoft3TL];
  float gj[kSoft3TL];  // upstream gradient at this lane's thresholds (0 beyond T)
  float* gx;           // grad_X of this item or null
  int64_t plane;       // H * W
  int ox, oy;          // origin of the wave's unit (with oz): coordinates are summed relative to it
  float lambda;
  __device__ __forceinline__ void take(int n, float v, int c, unsigned inpl, unsigned zrel) {
    park(n, v, c, inpl, zrel);
    const int lane = threadIdx.x & (kWave - 1);
    for (int e = 0; e < n; ++e) {
      const Soft3Entry en = stage[e];
      const float rx = (float)(en.x - ox), ry = (float)(en.yy - oy), rz = (float)(en.z - oz);
      float gd = 0.0f;
#pragma unroll
      for (int t = 0; t < kSoft3TL; ++t) {
        if (t < nt) {  // wave-uniform
          const float z = (float)(tj[t] - en.y);
          const float ex = soft3_exp_neg(z, kneg);
          const float s = __builtin_amdgcn_rcpf(1.0f + ex);
          const float d = ex * s * s;  // sigma (1 - sigma)
          const float cd = en.c * d;
          a0[t] += cd;
          ax[t] += cd * rx;
          ay[t] += cd * ry;
          az[t] += cd * rz;
          gd += gj[t] * d;
        }
      }
      if (gx) {  // wave-uniform
        gd = wave_sum_lane63(gd);
        if (lane == kWave - 1) gx[(int64_t)en.z * plane + en.inpl] = -lambda * en.c * gd;
      }
    }
  }
};

// LDS of a block: exchange words, [4 waves] queue entries and tilts, [4 waves] stages
constexpr size_t kSoft3Lds = kFixedLds3d + (size_t)4 * kWave * sizeof(Soft3Entry);

template <typename Sink>
__device__ __forceinline__ void soft3_lds(int* smem, unsigned*& xch, s3::TubeQueue<Sink>& queue, Soft3Entry*& stage) {
  const int wv = threadIdx.x >> 6;
  xch = reinterpret_cast<unsigned*>(smem);
  queue.buf = reinterpret_cast<uint2*>(smem + kXchInts) + wv * kQueueCap;
  queue.tbuf = reinterpret_cast<float*>(smem + kXchInts + 4 * kQueueCap * 2) + wv * kQueueCap;
  queue.count = 0;
  stage = reinterpret_cast<Soft3Entry*>(smem + kXchInts + 4 * kQueueCap * 3) + wv * kWave;
}

// partial[(item * units + unit) * T + j]
// TILTC: the sweep runs on the tilted field, so c(p) is that field's coefficient
template <bool TILTC>
__global__ __launch_bounds__(256) void soft3d_fwd_kernel(const float* __restrict__ grid, int D, int H, int W,
                                                         int64_t N, int nstrip, int ngroup, int nseg,
                                                         int planes_per_seg, const float* __restrict__ u,
                                                         float alpha, const float* __restrict__ tau, int T,
                                                         float kneg, float* __restrict__ partial) {
  extern __shared__ int smem[];
  unsigned* xch;
  Soft3Entry* stage;
  s3::TubeQueue<Soft3FwdSink> queue;
  soft3_lds(smem, xch, queue, stage);
  queue.sink.init(u, alpha, tau, T, kneg, W, stage);
#pragma unroll
  for (int t = 0; t < kSoft3TL; ++t) queue.sink.acc[t] = 0.f;
  const int unit = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int ox, oy;
  unit_origin3(unit, D, H, W, gridDim.y, planes_per_seg, kRows3d, ox, oy, queue.sink.oz);
  WaveRange range;
  const float* g = grid + (int64_t)blockIdx.y * N;
  if constexpr (TILTC) {
    const DirArgs da = {u, alpha, 1, 3};
    const Tilt t = load_tilt(da, 0);
    TiltRaw tr;
    tr.ax = t.ax, tr.ay = t.ay, tr.az = t.az;
    sweep3d_wave<float, kRows3d>(g, D, H, W, N, nstrip, ngroup, nseg, planes_per_seg, queue, xch, range, tr);
  } else {
    sweep3d_wave<float, kRows3d>(g, D, H, W, N, nstrip, ngroup, nseg, planes_per_seg, queue, xch, range, NoTilt());
  }
  const int units = gridDim.x * 4;
  float* out = partial + ((int64_t)blockIdx.y * units + unit) * T;
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
  for (int t = 0; t < kSoft3TL; ++t) {
    const int j = lane + kWave * t;
    if (j < T) out[j] = queue.sink.acc[t];
  }
}

// partial[((item * units + unit) * T + j) * 4 + {0: A0, 1: Ax, 2: Ay, 3: Az}]
template <bool TILTC>
__global__ __launch_bounds__(256) void soft3d_bwd_kernel(const float* __restrict__ grid, int D, int H, int W,
                                                         int64_t N, int nstrip, int ngroup, int nseg,
                                                         int planes_per_seg, const float* __restrict__ u,
                                                         float alpha, const float* __restrict__ tau, int T,
                                                         float kneg, float lambda, const float* __restrict__ gup,
                                                         float* __restrict__ grad_X, float* __restrict__ partial) {
  extern __shared__ int smem[];
  unsigned* xch;
  Soft3Entry* stage;
  s3::TubeQueue<Soft3BwdSink> queue;
  soft3_lds(smem, xch, queue, stage);
  Soft3BwdSink& s = queue.sink;
  s.init(u, alpha, tau, T, kneg, W, stage);
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
  for (int t = 0; t < kSoft3TL; ++t) {
    s.a0[t] = s.ax[t] = s.ay[t] = s.az[t] = 0.f;
    const int j = lane + kWave * t;
    s.gj[t] = j < T ? (gup ? gup[(int64_t)blockIdx.y * T + j] : 1.0f) : 0.0f;
  }
  s.gx = grad_X ? grad_X + (int64_t)blockIdx.y * N : nullptr;
  s.plane = (int64_t)H * W;
  s.lambda = lambda;
  const int unit = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  unit_origin3(unit, D, H, W, gridDim.y, planes_per_seg, kRows3d, s.ox, s.oy, s.oz);
  WaveRange range;
  const float* g = grid + (int64_t)blockIdx.y * N;
  if constexpr (TILTC) {
    const DirArgs da = {u, alpha, 1, 3};
    const Tilt t = load_tilt(da, 0);
    TiltRaw tr;
    tr.ax = t.ax, tr.ay = t.ay, tr.az = t.az;
    sweep3d_wave<float, kRows3d>(g, D, H, W, N, nstrip, ngroup, nseg, planes_per_seg, queue, xch, range, tr);
  } else {
    sweep3d_wave<float, kRows3d>(g, D, H, W, N, nstrip, ngroup, nseg, planes_per_seg, queue, xch, range, NoTilt());
  }
  if (partial) {
    const int units = gridDim.x * 4;
    float4* out = reinterpret_cast<float4*>(partial) + ((int64_t)blockIdx.y * units + unit) * (int64_t)T;
#pragma unroll
    for (int t = 0; t < kSoft3TL; ++t) {
      const int j = lane + kWave * t;
      if (j < T) out[j] = make_float4(s.a0[t], s.ax[t], s.ay[t], s.az[t]);
    }
  }
}

// Reduction over units: block (x = group of 64 thresholds, y = item) of 16 waves; wave w
// adds units w, w+16, ... in order (eight loads in flight at a time: a lone volume has
// thousands of units and one block per 64 thresholds), then wave 0 adds the 16 sums in order.
constexpr int kRedWaves = 16, kRedUnroll = 8;

__global__ __launch_bounds__(kRedWaves * kWave) void soft3d_fwd_reduce_kernel(const float* __restrict__ partial,
                                                                              int units, int T,
                                                                              float* __restrict__ chi) {
  __shared__ double red[kRedWaves][kWave];
  const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
  const int j = blockIdx.x * kWave + lane;
  const float* p = partial + (int64_t)blockIdx.y * units * T + j;
  double s = 0.0;
  if (j < T) {
    int q = wv;
    for (; q + (kRedUnroll - 1) * kRedWaves < units; q += kRedUnroll * kRedWaves) {
      float v[kRedUnroll];
#pragma unroll
      for (int k = 0; k < kRedUnroll; ++k) v[k] = p[(int64_t)(q + k * kRedWaves) * T];
#pragma unroll
      for (int k = 0; k < kRedUnroll; ++k) s += (double)v[k];
    }
    for (; q < units; q += kRedWaves) s += (double)p[(int64_t)q * T];
  }
  red[wv][lane] = s;
  __syncthreads();
  if (wv == 0 && j < T) {
    double r = red[0][lane];
    for (int w = 1; w < kRedWaves; ++w) r += red[w][lane];
    chi[(int64_t)blockIdx.y * T + j] = (float)r;
  }
}

// dchi_dtau = lambda sum A0;  dchi_du = -alpha lambda sum (origin * A0 + A_xyz)
__global__ __launch_bounds__(kRedWaves * kWave) void soft3d_bwd_reduce_kernel(
    const float* __restrict__ partial, int units, int D, int H, int W, int planes_per_seg, int T, float alpha,
    float lambda, float* __restrict__ dtau, float* __restrict__ du) {
  __shared__ double red[4][kRedWaves][kWave];
  const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
  const int j = blockIdx.x * kWave + lane;
  const float4* p = reinterpret_cast<const float4*>(partial) + (int64_t)blockIdx.y * units * T + j;
  double s0 = 0.0, sx = 0.0, sy = 0.0, sz = 0.0;
  auto add = [&](int q, const float4& e) {
    int ox, oy, oz;
    unit_origin3(q, D, H, W, gridDim.y, planes_per_seg, kRows3d, ox, oy, oz);
    const double a0 = (double)e.x;
    s0 += a0;
    sx += (double)ox * a0 + (double)e.y;
    sy += (double)oy * a0 + (double)e.z;
    sz += (double)oz * a0 + (double)e.w;
  };
  if (j < T) {
    int q = wv;
    for (; q + (kRedUnroll - 1) * kRedWaves < units; q += kRedUnroll * kRedWaves) {
      float4 v[kRedUnroll];
#pragma unroll
      for (int k = 0; k < kRedUnroll; ++k) v[k] = p[(int64_t)(q + k * kRedWaves) * T];
#pragma unroll
      for (int k = 0; k < kRedUnroll; ++k) add(q + k * kRedWaves, v[k]);
    }
    for (; q < units; q += kRedWaves) add(q, p[(int64_t)q * T]);
  }
  red[0][wv][lane] = s0;
  red[1][wv][lane] = sx;
  red[2][wv][lane] = sy;
  red[3][wv][lane] = sz;
  __syncthreads();
  if (wv == 0 && j < T) {
    const int64_t k = (int64_t)blockIdx.y * T + j;
    double r[4];
    for (int c = 0; c < 4; ++c) {
      r[c] = red[c][0][lane];
      for (int w = 1; w < kRedWaves; ++w) r[c] += red[c][w][lane];
    }
    if (dtau) dtau[k] = (float)((double)lambda * r[0]);
    if (du)
      for (int c = 0; c < 3; ++c) du[k * 3 + c] = (float)(-(double)alpha * (double)lambda * r[1 + c]);
  }
}

static float kneg3d(float lambda) { return (float)(-(double)lambda * 1.4426950408889634); }

bool soft3d_supported(const Shape& s, int T) {
  return s.ndim == 3 && T <= kSoft3TL * kWave && sweep3d_supported(s, 1);
}

size_t soft3d_workspace_bytes(const Shape& s, int T) {
  if (!soft3d_supported(s, T)) return 0;
  const Plan3d pl = plan3d<float>(s);
  return (size_t)256 + (size_t)s.batch * pl.grid.x * 4 * (size_t)T * 4 * sizeof(float);
}

void launch_soft3d_fwd(const float* grid, const Shape& s, const float* u, float alpha, const float* tau, int T,
                       float lambda, float* chi, void* ws, hipStream_t st, bool tiltc) {
  const Plan3d pl = plan3d<float>(s);
  float* partial = static_cast<float*>(ws);
#define ECC_GO(TC)                                                                                          \
  hipLaunchKernelGGL(soft3d_fwd_kernel<TC>, pl.grid, dim3(256), kSoft3Lds, st, grid, (int)s.D, (int)s.H,      \
                     (int)s.W, s.N, pl.nstrip, pl.ngroup, pl.nseg, pl.planes_per_seg, u, alpha, tau, T,       \
                     kneg3d(lambda), partial)
  if (tiltc) ECC_GO(true);
  else ECC_GO(false);
#undef ECC_GO
  hipLaunchKernelGGL(soft3d_fwd_reduce_kernel, dim3((unsigned)((T + kWave - 1) / kWave), (unsigned)s.batch),
                     dim3(kRedWaves * kWave), 0, st, partial, (int)pl.grid.x * 4, T, chi);
}

void launch_soft3d_bwd(const float* grid, const Shape& s, const float* u, float alpha, const float* tau, int T,
                       float lambda, const float* gup, float* grad_X, float* dtau, float* du, void* ws,
                       hipStream_t st, bool tiltc) {
  const Plan3d pl = plan3d<float>(s);
  float* partial = (dtau || du) ? static_cast<float*>(ws) : nullptr;
  if (grad_X) launch_clear_f32(grad_X, s.N * s.batch, st);  // zero away from the critical vertices
#define ECC_GO(TC)                                                                                          \
  hipLaunchKernelGGL(soft3d_bwd_kernel<TC>, pl.grid, dim3(256), kSoft3Lds, st, grid, (int)s.D, (int)s.H,      \
                     (int)s.W, s.N, pl.nstrip, pl.ngroup, pl.nseg, pl.planes_per_seg, u, alpha, tau, T,       \
                     kneg3d(lambda), lambda, gup, grad_X, partial)
  if (tiltc) ECC_GO(true);
  else ECC_GO(false);
#undef ECC_GO
  if (partial) {
    hipLaunchKernelGGL(soft3d_bwd_reduce_kernel, dim3((unsigned)((T + kWave - 1) / kWave), (unsigned)s.batch),
                       dim3(kRedWaves * kWave), 0, st, partial, (int)pl.grid.x * 4, (int)s.D, (int)s.H, (int)s.W, pl.planes_per_seg, T,
                       alpha, lambda, dtau, du);
  }
}

}  // namespace ecc
