// Soft single-direction ECC for 2D grids, fused into the strip sweep of
// ecc_sweep2d.h: forward (Eq. 6 of the paper) and derivatives (Eq. 8-10).
//
// Every term of Eq. 6 / Eq. 8-10 carries the integer factor c(p), so only the
// critical vertices (c != 0) contribute.  The sweep finds them with the
// bit-sliced stencil and hands them to this file's sinks 64 at a time, straight
// from the wave's LDS queue.  A sink evaluates the sigmoid on entries x
// thresholds pairs only:
//   - threshold-major: lane l owns thresholds tau_l, tau_{l+64}, ... (up to 4,
//     so T <= 256) and runs over the queue entries (LDS broadcast reads): the
//     sums over p of Eq. 6 / Eq. 9 / Eq. 10 need no cross-lane reduction;
//   - backward: the same pass also forms, per entry, the contraction of Eq. 8 with
//     the upstream gradient as a fixed-order sum over the lanes (grad_X).
// grad_X is zero away from critical vertices; the sweep writes those zeros row
// by row for the vertices it owns, before any entry of those rows is drained
// (measured a little quicker than a fill kernel in front of the sweep).
// Each wave writes its partial sums to the workspace; a second kernel adds them
// in a fixed order in float64, so results are run-to-run identical.
//
// z = tau_j - X(p) - alpha <u,p> is formed in float64 and rounded once; exp2 and
// the reciprocal run on the float32 transcendental unit.
#include "ecc_sweep2d.h"

namespace ecc {

constexpr int kSoftTL = 4;  // thresholds per lane

__device__ __forceinline__ float soft_exp_neg(float z, float kneg) {
  // exp(-lambda z) = 2^(kneg z); clamped so the result stays finite
  return __builtin_amdgcn_exp2f(fminf(kneg * z, 126.0f));
}

struct SoftEntry {
  double y;  // X(p) + alpha <u,p>
  float c;
  int col, row;
  int pad;
};

struct SoftCommon {
  typedef SoftEntry Entry;
  static constexpr bool kTrackRange = false;
  double ux, uy, alpha;
  double tj[kSoftTL];  // this lane's thresholds
  int T;
  int nt;  // threshold slots in use: ceil(T / 64)
  float kneg;
  // The sweep ran on the tilted field (c of the tilted field): the value it hands over
  // is the tilted one in float32; X is read again so that y is formed as always.
  const float* xsrc;  // this item's grid, or null when the sweep ran on X itself
  int xW;
  __device__ __forceinline__ Entry make(float v, int c, int col, int row) const {
    Entry e;
    if (xsrc) v = xsrc[(int64_t)row * xW + col];  // wave-uniform condition
    e.y = (double)v + alpha * (ux * (double)col + uy * (double)row);
    e.c = (float)c;
    e.col = col;
    e.row = row;
    e.pad = 0;
    return e;
  }
  __device__ __forceinline__ void init(const float* u, float alpha_, const float* tau, int T_, float kneg_) {
    ux = (double)u[0];
    uy = (double)u[1];
    alpha = (double)alpha_;
    T = T_;
    nt = (T_ + kWave - 1) / kWave;
    kneg = kneg_;
    xsrc = nullptr;
    xW = 0;
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int t = 0; t < kSoftTL; ++t) {
      const int j = lane + kWave * t;
      tj[t] = j < T ? (double)tau[j] : 0.0;
    }
  }
};

struct SoftFwdSink : SoftCommon {
  static constexpr bool kZeroFill = false;
  float acc[kSoftTL];
  __device__ __forceinline__ void consume(const Entry* buf, int n) {
    for (int e = 0; e < n; ++e) {
      const double y = buf[e].y;
      const float c = buf[e].c;
#pragma unroll
      for (int t = 0; t < kSoftTL; ++t) {
        if (t < nt) {  // wave-uniform
          const float z = (float)(tj[t] - y);
          const float ex = soft_exp_neg(z, kneg);
          acc[t] += c * __builtin_amdgcn_rcpf(1.0f + ex);
        }
      }
    }
  }
};

struct SoftBwdSink : SoftCommon {
  static constexpr bool kZeroFill = true;
  float a0[kSoftTL], ax[kSoftTL], ay[kSoftTL];
  float gj[kSoftTL];  // upstream gradient at this lane's thresholds (0 beyond T)
  float* gx;          // grad_X of this item or null
  int W;
  int col0, row0;    // origin of the wave's unit: coordinates are summed relative to it
  float lambda;

  template <bool EDGE>
  __device__ __forceinline__ void zero_row(int row, int col, const bool (&ok)[kNC], bool out_lane) const {
    if (!gx || !out_lane) return;
    float* p = gx + (int64_t)row * W + col;
    if (!EDGE && (reinterpret_cast<uintptr_t>(p) & 15) == 0) {
      *reinterpret_cast<float4*>(p) = make_float4(0.f, 0.f, 0.f, 0.f);
    } else {
#pragma unroll
      for (int e = 0; e < kNC; ++e)
        if (ok[e]) p[e] = 0.f;
    }
  }

  // One pass over entries x thresholds serves all three derivatives: lane l holds
  // sigma'(z) / lambda for its thresholds; the sums over p stay in the lane, the
  // contraction with the upstream gradient (Eq. 8) is a fixed-order sum over the lanes.
  __device__ __forceinline__ void consume(const Entry* buf, int n) {
    const int lane = threadIdx.x & (kWave - 1);
    for (int e = 0; e < n; ++e) {
      const double y = buf[e].y;
      const float c = buf[e].c;
      const float rx = (float)(buf[e].col - col0), ry = (float)(buf[e].row - row0);
      float gd = 0.0f;
#pragma unroll
      for (int t = 0; t < kSoftTL; ++t) {
        if (t < nt) {  // wave-uniform
          const float z = (float)(tj[t] - y);
          const float ex = soft_exp_neg(z, kneg);
          const float s = __builtin_amdgcn_rcpf(1.0f + ex);
          const float d = ex * s * s;  // sigma (1 - sigma)
          const float cd = c * d;
          a0[t] += cd;
          ax[t] += cd * rx;
          ay[t] += cd * ry;
          gd += gj[t] * d;
        }
      }
      if (gx) {  // wave-uniform
        gd = wave_sum_lane63(gd);
        if (lane == kWave - 1) gx[(int64_t)buf[e].row * W + buf[e].col] = -lambda * c * gd;
      }
    }
  }
};

// LDS: [4 waves] value rings, then [4 waves] queues of SoftEntry
__device__ __forceinline__ void soft_lds(int* smem, float*& ring, SoftEntry*& qbuf) {
  const int wv = threadIdx.x >> 6;
  ring = reinterpret_cast<float*>(smem) + wv * (kChunkRows * kWave * kNC);
  qbuf = reinterpret_cast<SoftEntry*>(smem + 4 * kChunkRows * kWave * kNC) + wv * kQueueCap;
}

// partial[(item * units + unit) * T + j]
// TILTC: the sweep runs on the tilted field, so c(p) is that field's coefficient
template <bool TILTC>
__global__ __launch_bounds__(256) void soft2d_fwd_kernel(const float* __restrict__ grid, int H, int W,
                                                         int64_t N, int nstrip, int nseg, int rows_per_seg,
                                                         const float* __restrict__ u, float alpha,
                                                         const float* __restrict__ tau, int T, float kneg,
                                                         float* __restrict__ partial) {
  extern __shared__ int smem[];
  float* ring;
  SoftEntry* qbuf;
  soft_lds(smem, ring, qbuf);
  WaveQueue<SoftFwdSink> queue;
  queue.buf = qbuf;
  queue.count = 0;
  queue.sink.init(u, alpha, tau, T, kneg);
#pragma unroll
  for (int t = 0; t < kSoftTL; ++t) queue.sink.acc[t] = 0.f;
  WaveRange range;
  if constexpr (TILTC) {
    queue.sink.xsrc = grid + (int64_t)blockIdx.y * N;
    queue.sink.xW = W;
    const DirArgs da = {u, alpha, 1, 2};
    sweep2d_wave<float>(grid + (int64_t)blockIdx.y * N, H, W, N, nstrip, nseg, rows_per_seg, queue, ring, range,
                        load_tilt(da, 0));
  } else {
    sweep2d_wave<float>(grid + (int64_t)blockIdx.y * N, H, W, N, nstrip, nseg, rows_per_seg, queue, ring, range,
                        NoTilt());
  }
  const int unit = blockIdx.x * 4 + (threadIdx.x >> 6), units = nstrip * nseg;
  if (unit < units) {
    float* out = partial + ((int64_t)blockIdx.y * units + unit) * T;
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int t = 0; t < kSoftTL; ++t) {
      const int j = lane + kWave * t;
      if (j < T) out[j] = queue.sink.acc[t];
    }
  }
}

// partial[((item * units + unit) * T + j) * 4 + {0: A0, 1: Ax, 2: Ay}]
template <bool TILTC>
__global__ __launch_bounds__(256) void soft2d_bwd_kernel(const float* __restrict__ grid, int H, int W,
                                                         int64_t N, int nstrip, int nseg, int rows_per_seg,
                                                         const float* __restrict__ u, float alpha,
                                                         const float* __restrict__ tau, int T, float kneg,
                                                         float lambda, const float* __restrict__ gup,
                                                         float* __restrict__ grad_X,
                                                         float* __restrict__ partial) {
  extern __shared__ int smem[];
  float* ring;
  SoftEntry* qbuf;
  soft_lds(smem, ring, qbuf);
  WaveQueue<SoftBwdSink> queue;
  queue.buf = qbuf;
  queue.count = 0;
  SoftBwdSink& s = queue.sink;
  s.init(u, alpha, tau, T, kneg);
#pragma unroll
  for (int t = 0; t < kSoftTL; ++t) s.a0[t] = s.ax[t] = s.ay[t] = 0.f;
  {
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int t = 0; t < kSoftTL; ++t) {
      const int j = lane + kWave * t;
      s.gj[t] = j < T ? (gup ? gup[(int64_t)blockIdx.y * T + j] : 1.0f) : 0.0f;
    }
  }
  s.gx = grad_X ? grad_X + (int64_t)blockIdx.y * N : nullptr;
  s.W = W;
  s.lambda = lambda;
  const int unit = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), units = nstrip * nseg;
  s.col0 = (unit % nstrip) * kStripOut - kNC;
  s.row0 = (unit / nstrip) * rows_per_seg;
  WaveRange range;
  if constexpr (TILTC) {
    queue.sink.xsrc = grid + (int64_t)blockIdx.y * N;
    queue.sink.xW = W;
    const DirArgs da = {u, alpha, 1, 2};
    sweep2d_wave<float>(grid + (int64_t)blockIdx.y * N, H, W, N, nstrip, nseg, rows_per_seg, queue, ring, range,
                        load_tilt(da, 0));
  } else {
    sweep2d_wave<float>(grid + (int64_t)blockIdx.y * N, H, W, N, nstrip, nseg, rows_per_seg, queue, ring, range,
                        NoTilt());
  }
  if (partial && unit < units) {
    float* out = partial + ((int64_t)blockIdx.y * units + unit) * (int64_t)T * 4;
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int t = 0; t < kSoftTL; ++t) {
      const int j = lane + kWave * t;
      if (j < T) {
        out[j * 4 + 0] = s.a0[t];
        out[j * 4 + 1] = s.ax[t];
        out[j * 4 + 2] = s.ay[t];
      }
    }
  }
}

// Reduction over units: block (x = group of 64 thresholds, y = item) of 16 waves; wave w
// adds units w, w+16, ... in order (eight loads in flight at a time: a lone large image
// has thousands of units and one block per 64 thresholds), then wave 0 adds the 16 sums
// in order.
constexpr int kRedWaves = 16, kRedUnroll = 8;

__global__ __launch_bounds__(kRedWaves * kWave) void soft2d_fwd_reduce_kernel(const float* __restrict__ partial,
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

// dchi_dtau = lambda sum A0;  dchi_du = -alpha lambda sum (origin * A0 + A_xy)
__global__ __launch_bounds__(kRedWaves * kWave) void soft2d_bwd_reduce_kernel(
    const float* __restrict__ partial, int units, int nstrip, int rows_per_seg, int T, float alpha, float lambda,
    float* __restrict__ dtau, float* __restrict__ du) {
  __shared__ double red[3][kRedWaves][kWave];
  const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
  const int j = blockIdx.x * kWave + lane;
  const float4* p = reinterpret_cast<const float4*>(partial) + (int64_t)blockIdx.y * units * T + j;
  double s0 = 0.0, sx = 0.0, sy = 0.0;
  auto add = [&](int q, const float4& e) {
    const double ox = (double)((q % nstrip) * kStripOut - kNC), oy = (double)((q / nstrip) * rows_per_seg);
    const double a0 = (double)e.x;
    s0 += a0;
    sx += ox * a0 + (double)e.y;
    sy += oy * a0 + (double)e.z;
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
  __syncthreads();
  if (wv == 0 && j < T) {
    const int64_t k = (int64_t)blockIdx.y * T + j;
    double r[3];
    for (int c = 0; c < 3; ++c) {
      r[c] = red[c][0][lane];
      for (int w = 1; w < kRedWaves; ++w) r[c] += red[c][w][lane];
    }
    if (dtau) dtau[k] = (float)((double)lambda * r[0]);
    if (du) {
      du[k * 2 + 0] = (float)(-(double)alpha * (double)lambda * r[1]);
      du[k * 2 + 1] = (float)(-(double)alpha * (double)lambda * r[2]);
    }
  }
}

static float kneg2d(float lambda) { return (float)(-(double)lambda * 1.4426950408889634); }
constexpr size_t kSoftLds = ring_bytes2d<SoftEntry>();

bool soft2d_supported(const Shape& s, int T) {
  return s.D == 1 && s.ndim == 2 && T <= kSoftTL * kWave && s.W >= 8 && s.W <= (1 << 22) &&
         s.H <= (1 << 30) && s.N < ((int64_t)1 << 31);
}

size_t soft2d_workspace_bytes(const Shape& s, int T) {
  if (!soft2d_supported(s, T)) return 0;
  const Plan2d pl = plan2d<float>(s, true);
  return (size_t)256 + (size_t)s.batch * pl.nstrip * pl.nseg * (size_t)T * 4 * sizeof(float);
}

void launch_soft2d_fwd(const float* grid, const Shape& s, const float* u, float alpha, const float* tau,
                       int T, float lambda, float* chi, void* ws, hipStream_t st, bool tiltc) {
  const Plan2d pl = plan2d<float>(s, true);
  float* partial = static_cast<float*>(ws);
  if (tiltc)
    hipLaunchKernelGGL(soft2d_fwd_kernel<true>, pl.grid, dim3(256), kSoftLds, st, grid, (int)s.H, (int)s.W, s.N,
                       pl.nstrip, pl.nseg, pl.rows_per_seg, u, alpha, tau, T, kneg2d(lambda), partial);
  else
    hipLaunchKernelGGL(soft2d_fwd_kernel<false>, pl.grid, dim3(256), kSoftLds, st, grid, (int)s.H, (int)s.W, s.N,
                       pl.nstrip, pl.nseg, pl.rows_per_seg, u, alpha, tau, T, kneg2d(lambda), partial);
  hipLaunchKernelGGL(soft2d_fwd_reduce_kernel, dim3((unsigned)((T + kWave - 1) / kWave), (unsigned)s.batch),
                     dim3(kRedWaves * kWave), 0, st, partial, pl.nstrip * pl.nseg, T, chi);
}

void launch_soft2d_bwd(const float* grid, const Shape& s, const float* u, float alpha, const float* tau,
                       int T, float lambda, const float* gup, float* grad_X, float* dtau, float* du,
                       void* ws, hipStream_t st, bool tiltc) {
  const Plan2d pl = plan2d<float>(s, true);
  float* partial = (dtau || du) ? static_cast<float*>(ws) : nullptr;
  if (tiltc)
    hipLaunchKernelGGL(soft2d_bwd_kernel<true>, pl.grid, dim3(256), kSoftLds, st, grid, (int)s.H, (int)s.W, s.N,
                       pl.nstrip, pl.nseg, pl.rows_per_seg, u, alpha, tau, T, kneg2d(lambda), lambda, gup,
                       grad_X, partial);
  else
    hipLaunchKernelGGL(soft2d_bwd_kernel<false>, pl.grid, dim3(256), kSoftLds, st, grid, (int)s.H, (int)s.W, s.N,
                       pl.nstrip, pl.nseg, pl.rows_per_seg, u, alpha, tau, T, kneg2d(lambda), lambda, gup,
                       grad_X, partial);
  if (partial) {
    hipLaunchKernelGGL(soft2d_bwd_reduce_kernel, dim3((unsigned)((T + kWave - 1) / kWave), (unsigned)s.batch),
                       dim3(kRedWaves * kWave), 0, st, partial, pl.nstrip * pl.nseg, pl.nstrip, pl.rows_per_seg, T, alpha,
                       lambda, dtau, du);
  }
}

}  // namespace ecc
