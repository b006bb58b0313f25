// Soft single-direction ECC for 3D grids, fused into the tube sweep of
// ecc_sweep3d.h: forward (Eq. 6 of the paper) and derivatives (Eq. 8-10).
//
// As in 2D, only the critical vertices (c != 0) carry a term.  The tube sweep
// finds them and queues (position, c); when 64 are drained together each lane
// fetches one value, forms y = X(p) + alpha <u,p> in float64, carries it on as two
// floats (yh + yl, so that (tau_j - yh) - yl is the float64 difference to an ulp) and
// parks the entry in a small LDS stage -- unless y lies so far outside [min tau, max tau]
// that every sigmoid is 0 or 1 to 2^-64: such an entry adds c or nothing to every
// threshold and is not evaluated.  Then every lane runs over the staged entries for the
// thresholds it owns (tau_l, tau_{l+64}, ...; T <= 256): the sums over p of
// Eq. 6 / Eq. 9 / Eq. 10 need no cross-lane reduction, the contraction of Eq. 8
// with the upstream gradient is a fixed-order sum over the lanes.  grad_X is
// cleared by a fill kernel first and written at the critical vertices only.
// Each wave leaves its partial sums in the workspace; a second kernel adds them
// in a fixed order in float64, so results are run-to-run identical.
#include "ecc_sweep3d.h"
#include "ecc_soft_saved.h"
#include "ecc_soft_reduce.h"

#include <cstdlib>

namespace ecc {

constexpr int kSoft3TL = 4;  // thresholds per lane

struct Soft3Entry {
  float yh, yl;  // X(p) + alpha <u,p> = yh + yl
  float c;
  int x, yy, z;
  unsigned inpl;  // yy * W + x
  int pad;
};

struct Soft3Common {
  static constexpr bool kTrackRange = false;
  double ux, uy, uz, alpha;
  float tj[kSoft3TL];  // this lane's thresholds
  int nt;              // threshold slots in use: ceil(T / 64)
  float kneg;
  float sat_lo, sat_hi;  // y <= sat_lo: every sigma is 1;  y >= sat_hi: every sigma is 0 (to 2^-64)
  int W;
  int64_t plane;      // H * W
  int oz;             // first plane of the wave's segment
  Soft3Entry* stage;  // wave-private LDS, 64 entries
  __device__ __forceinline__ void init(const float* u, float alpha_, const float* tau, int T, float kneg_, int H_, int W_,
                                       Soft3Entry* stage_) {
    ux = (double)u[0];
    uy = (double)u[1];
    uz = (double)u[2];
    alpha = (double)alpha_;
    nt = (T + kWave - 1) / kWave;
    kneg = kneg_;
    W = W_;
    plane = (int64_t)H_ * W_;
    stage = stage_;
    const int lane = threadIdx.x & (kWave - 1);
    float lo = INFINITY, hi = -INFINITY;
#pragma unroll
    for (int t = 0; t < kSoft3TL; ++t) {
      const int j = lane + kWave * t;
      tj[t] = j < T ? tau[j] : 0.0f;
      if (j < T) {
        lo = fminf(lo, tj[t]);
        hi = fmaxf(hi, tj[t]);
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      lo = fminf(lo, __shfl_xor(lo, o));
      hi = fmaxf(hi, __shfl_xor(hi, o));
    }
    soft_sat_bounds(lo, hi, kneg_, sat_lo, sat_hi);
  }
  // Lane i < n forms its entry; the entries that have to be evaluated are packed into the stage
  // and counted (the return value).  A dropped entry whose sigmoids are all 1 adds its c to
  // *csat, one whose sigmoids are all 0 adds nothing; neither has a derivative above 2^-64 lambda.
  // save_to (may be null): room for the n entries, every one of them, as the backward pass wants them.
  __device__ __forceinline__ int park(int n, float v, int c, unsigned inpl, unsigned zrel, float* csat,
                                      SavedEntry* save_to = nullptr) const {
    const int lane = threadIdx.x & (kWave - 1);
    const bool in = lane < n;
    Soft3Entry e;
    e.yy = (int)(inpl / (unsigned)W);
    e.x = (int)(inpl - (unsigned)e.yy * (unsigned)W);
    e.z = oz + (int)zrel;
    const double y = (double)v + alpha * ((ux * (double)e.x + uy * (double)e.yy) + uz * (double)e.z);
    e.yh = (float)y;
    e.yl = (float)(y - (double)e.yh);
    e.c = (float)c;
    e.inpl = inpl;
    e.pad = 0;
    if (save_to && in) {
      SavedEntry o;
      o.y = y;
      o.idx = (int)((int64_t)e.z * plane + inpl);
      o.c = c;
      save_to[lane] = o;
    }
    const bool keep = in && e.yh > sat_lo && e.yh < sat_hi;
    const unsigned long long m = __builtin_amdgcn_ballot_w64(keep);
    const int kept = __builtin_popcountll(m);
    if (kept != n && csat) {  // wave-uniform
      const float ones = wave_sum_lane63((in && e.yh <= sat_lo) ? e.c : 0.0f);
      *csat += __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, ones), kWave - 1));
    }
    const int pos = (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
    if (keep) stage[pos] = e;
    return kept;
  }
  __device__ __forceinline__ float zarg(int t, float yh, float yl) const { return (tj[t] - yh) - yl; }
};

struct Soft3FwdSink : Soft3Common {
  float acc[kSoft3TL];
  float csat;  // sum of c over the entries whose sigmoids are all 1 (wave-uniform)
  __device__ __forceinline__ void take(int n, float v, int c, unsigned inpl, unsigned zrel) {
    n = park(n, v, c, inpl, zrel, &csat);
    for (int e = 0; e < n; ++e) {
      const float yh = stage[e].yh, yl = stage[e].yl;
      const float cf = stage[e].c;
#pragma unroll
      for (int t = 0; t < kSoft3TL; ++t) {
        if (t < nt) {  // wave-uniform
          const float ex = soft_exp_neg(zarg(t, yh, yl), kneg);
          acc[t] += cf * __builtin_amdgcn_rcpf(1.0f + ex);
        }
      }
    }
  }
  __device__ __forceinline__ float total(int t) const { return acc[t] + csat; }
};

struct Soft3BwdSink : Soft3Common {
  float a0[kSoft3TL], ax[kSoft3TL], ay[kSoft3TL], az[kSoft3TL];
  float gj[kSoft3TL];  // upstream gradient at this lane's thresholds (0 beyond T)
  float* gx;           // grad_X of this item or null
  int ox, oy;          // origin of the wave's unit (with oz): coordinates are summed relative to it
  float lambda;
  __device__ __forceinline__ void take(int n, float v, int c, unsigned inpl, unsigned zrel) {
    n = park(n, v, c, inpl, zrel, nullptr);  // grad_X stays 0 at a saturated vertex
    const int lane = threadIdx.x & (kWave - 1);
    for (int e = 0; e < n; ++e) {
      const Soft3Entry en = stage[e];
      const float rx = (float)(en.x - ox), ry = (float)(en.yy - oy), rz = (float)(en.z - oz);
      float gd = 0.0f;
#pragma unroll
      for (int t = 0; t < kSoft3TL; ++t) {
        if (t < nt) {  // wave-uniform
          const float ex = soft_exp_neg(zarg(t, en.yh, en.yl), kneg);
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
  queue.sink.init(u, alpha, tau, T, kneg, H, W, stage);
#pragma unroll
  for (int t = 0; t < kSoft3TL; ++t) queue.sink.acc[t] = 0.f;
  queue.sink.csat = 0.f;
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
    if (j < T) out[j] = queue.sink.total(t);
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
  s.init(u, alpha, tau, T, kneg, H, W, stage);
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
  for (int t = 0; t < kSoft3TL; ++t) {
    s.a0[t] = s.ax[t] = s.ay[t] = s.az[t] = 0.f;
    const int j = lane + kWave * t;
    s.gj[t] = j < T ? (gup ? gup[(int64_t)blockIdx.y * T + j] : 1.0f) : 0.0f;
  }
  s.gx = grad_X ? grad_X + (int64_t)blockIdx.y * N : nullptr;
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

// Forward pass that saves its critical vertices: chi as Soft3FwdSink, optionally the sums of
// Eq. 9 / Eq. 10 in the same pass (they share the sigmoid), and every entry appended to the
// unit's own list in the state buffer (sweep order, no atomics: the same on every run).
template <bool DERIV>
struct Soft3SaveSink : Soft3Common {
  float acc[kSoft3TL], a0[kSoft3TL], ax[kSoft3TL], ay[kSoft3TL], az[kSoft3TL];
  float csat;
  int ox, oy;
  SavedEntry* list;     // this unit's list
  unsigned cap, saved;  // saved: entries seen so far (wave-uniform; may pass cap)
  __device__ __forceinline__ void take(int n, float v, int c, unsigned inpl, unsigned zrel) {
    const bool room = saved + (unsigned)n <= cap;  // (a batch that does not fit is left out whole)
    const unsigned at = saved;
    saved += (unsigned)n;
    n = park(n, v, c, inpl, zrel, &csat, room ? list + at : nullptr);
    for (int e = 0; e < n; ++e) {
      const Soft3Entry en = stage[e];
      const float rx = (float)(en.x - ox), ry = (float)(en.yy - oy), rz = (float)(en.z - oz);
#pragma unroll
      for (int t = 0; t < kSoft3TL; ++t) {
        if (t < nt) {  // wave-uniform
          const float ex = soft_exp_neg(zarg(t, en.yh, en.yl), kneg);
          const float sg = __builtin_amdgcn_rcpf(1.0f + ex);
          acc[t] += en.c * sg;
          if (DERIV) {
            const float cd = en.c * (ex * sg * sg);  // c sigma (1 - sigma)
            a0[t] += cd;
            ax[t] += cd * rx;
            ay[t] += cd * ry;
            az[t] += cd * rz;
          }
        }
      }
    }
  }
};

// partial[((item * units + unit) * T + j) * 5 + {0: chi, 1: A0, 2: Ax, 3: Ay, 4: Az}]
template <bool TILTC, bool DERIV>
__global__ __launch_bounds__(256) void soft3d_fwd_save_kernel(const float* __restrict__ grid, int D, int H, int W,
                                                              int64_t N, int nstrip, int ngroup, int nseg,
                                                              int planes_per_seg, const float* __restrict__ u,
                                                              float alpha, const float* __restrict__ tau, int T,
                                                              float kneg, float* __restrict__ partial, StateView sv,
                                                              unsigned cap) {
  extern __shared__ int smem[];
  unsigned* xch;
  Soft3Entry* stage;
  s3::TubeQueue<Soft3SaveSink<DERIV>> queue;
  soft3_lds(smem, xch, queue, stage);
  Soft3SaveSink<DERIV>& s = queue.sink;
  s.init(u, alpha, tau, T, kneg, H, W, stage);
#pragma unroll
  for (int t = 0; t < kSoft3TL; ++t) s.acc[t] = s.a0[t] = s.ax[t] = s.ay[t] = s.az[t] = 0.f;
  s.csat = 0.f;
  const int unit = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), units = gridDim.x * 4;
  unit_origin3(unit, D, H, W, gridDim.y, planes_per_seg, kRows3d, s.ox, s.oy, s.oz);
  s.cap = cap;
  s.saved = 0u;
  s.list = sv.lists + ((size_t)blockIdx.y * units + unit) * cap;
  const unsigned next_gen = *sv.gen + 1u;  // (the reduction kernel that follows stores it)
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
  const int lane = threadIdx.x & (kWave - 1);
  if (lane == 0) {
    sv.counts[(size_t)blockIdx.y * units + unit] = s.saved;
    if (s.saved > cap) sv.overflow[blockIdx.y] = next_gen;
  }
  float* out = partial + ((int64_t)blockIdx.y * units + unit) * (int64_t)T * 5;
#pragma unroll
  for (int t = 0; t < kSoft3TL; ++t) {
    const int j = lane + kWave * t;
    if (j < T) {
      out[j * 5 + 0] = s.acc[t] + s.csat;
      out[j * 5 + 1] = s.a0[t];
      out[j * 5 + 2] = s.ax[t];
      out[j * 5 + 3] = s.ay[t];
      out[j * 5 + 4] = s.az[t];
    }
  }
}

// grad_X from the saved lists (Eq. 8 contracted with the upstream gradient): a block per unit of
// the forward sweep walks that unit's list; grad_X has been cleared by a fill kernel.  An item
// whose lists cannot be used (header of another shape, a unit ran out of room) is computed from
// the grid instead, vertex by vertex with the plain stencil: slow, but rare.
template <bool TILTC>
__global__ __launch_bounds__(256) void soft3d_bwd_saved_kernel(const float* __restrict__ grid, int D, int H, int W,
                                                               int64_t N, const float* __restrict__ u, float alpha,
                                                               const float* __restrict__ tau, int T, float kneg,
                                                               float lambda, const float* __restrict__ gup,
                                                               float* __restrict__ grad_X, StateView sv,
                                                               SoftStateHeader expect) {
  const int item = blockIdx.y, unit = blockIdx.x, units = gridDim.x;
  const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
  __shared__ float stau[kSoft3TL * kWave];
  __shared__ float sg[kSoft3TL * kWave];
  __shared__ StagedEntry stage[256];
  __shared__ float sred[2][4];
  __shared__ int skept[4];
  // requested up front, in one round trip to memory: the state's header words, the unit's count
  // and the first 256 slots of its list (whatever the count says)
  const bool usable = state_usable(sv, expect, item);
  const unsigned cnt_raw = sv.counts[(size_t)item * units + unit];
  const SavedEntry* list = sv.lists + ((size_t)item * units + unit) * expect.cap;
  const SavedEntry first = list[min((unsigned)threadIdx.x, expect.cap - 1u)];
  float lo = INFINITY, hi = -INFINITY;
  for (int j = threadIdx.x; j < T; j += 256) {
    const float t = tau[j];
    stau[j] = t;
    sg[j] = gup ? gup[(int64_t)item * T + j] : 1.0f;
    lo = fminf(lo, t);
    hi = fmaxf(hi, t);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    lo = fminf(lo, __shfl_xor(lo, o));
    hi = fmaxf(hi, __shfl_xor(hi, o));
  }
  if (lane == 0) {
    sred[0][wv] = lo;
    sred[1][wv] = hi;
  }
  __syncthreads();
  lo = fminf(fminf(sred[0][0], sred[0][1]), fminf(sred[0][2], sred[0][3]));
  hi = fmaxf(fmaxf(sred[1][0], sred[1][1]), fmaxf(sred[1][2], sred[1][3]));
  float sat_lo, sat_hi;
  soft_sat_bounds(lo, hi, kneg, sat_lo, sat_hi);
  float* gx = grad_X + (int64_t)item * N;
  if (!usable) {
    const float* g = grid + (int64_t)item * N;
    Tilt tilt;
    if (TILTC) {
      const DirArgs da = {u, alpha, 1, 3};
      tilt = load_tilt(da, 0);
    }
    const double ux = (double)u[0], uy = (double)u[1], uz = (double)u[2];
    for (int64_t i = (int64_t)unit * 256 + threadIdx.x; i < N; i += (int64_t)units * 256) {
      const int64_t x = i % W, r = i / W, y = r % H, z = r / H;
      int c;
      if (TILTC) c = coeff_tilted_at<3>(g, tilt, D, H, W, z, y, x);
      else c = coeff_at<float, 3>(g, D, H, W, z, y, x);
      if (c != 0) {
        const double yv = (double)g[i] + (double)alpha * ((ux * (double)x + uy * (double)y) + uz * (double)z);
        const float yh = (float)yv, yl = (float)(yv - (double)yh);
        if (yh > sat_lo && yh < sat_hi) {
          float gd = 0.0f;
          for (int j = 0; j < T; ++j) gd += sg[j] * soft_dsig(stau[j], yh, yl, kneg);
          gx[i] = -lambda * (float)c * gd;
        }
      }
    }
    return;
  }
  saved_lists_to_grad(list, cnt_raw, expect.cap, first, stau, sg, T, kneg, lambda, sat_lo, sat_hi, gx, N, stage, skept);
}

// origin of a unit's coordinates, for the reduction of ecc_soft_reduce.h
struct Origin3 {
  int D, H, W, nitems, planes_per_seg;
  __device__ __forceinline__ void operator()(int unit, int (&o)[3]) const {
    unit_origin3(unit, D, H, W, nitems, planes_per_seg, kRows3d, o[0], o[1], o[2]);
  }
};
static Origin3 origin3(const Shape& s, const Plan3d& pl) {
  return Origin3{(int)s.D, (int)s.H, (int)s.W, (int)s.batch, pl.planes_per_seg};
}

static float kneg3d(float lambda) { return (float)(-(double)lambda * 1.4426950408889634); }

bool soft3d_supported(const Shape& s, int T) {
  return s.ndim == 3 && T <= kSoft3TL * kWave && sweep3d_supported(s, 1);
}

// per-unit partial sums (up to five floats per unit and threshold), a multiple of 256 bytes
static size_t soft3d_partial_bytes(const Shape& s, const Plan3d& pl, int T) {
  const size_t n = (size_t)s.batch * pl.grid.x * 4 * (size_t)T * 5 * sizeof(float);
  return (n + 255) / 256 * 256;
}

size_t soft3d_workspace_bytes(const Shape& s, int T) {
  if (!soft3d_supported(s, T)) return 0;
  const Plan3d pl = plan3d<float>(s);
  return (size_t)256 + soft3d_partial_bytes(s, pl, T) + soft_reduce_mid_bytes(s.batch, T);
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
  double* mid = reinterpret_cast<double*>(static_cast<char*>(ws) + soft3d_partial_bytes(s, pl, T));
  const RedOut out = {chi, nullptr, nullptr, nullptr, nullptr, {}};
  launch_soft_reduce<1, true, -1>(partial, mid, (int)pl.grid.x * 4, s.batch, T, alpha, lambda, origin3(s, pl), out, st);
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
    double* mid = reinterpret_cast<double*>(static_cast<char*>(ws) + soft3d_partial_bytes(s, pl, T));
    const RedOut out = {nullptr, dtau, du, nullptr, nullptr, {}};
    launch_soft_reduce<4, false, 3>(partial, mid, (int)pl.grid.x * 4, s.batch, T, alpha, lambda, origin3(s, pl), out, st);
  }
}

// ---- forward that saves its critical vertices, backward from the saved lists ----------------
static unsigned state_cap3(const Plan3d& pl) {
  // room for one vertex in eight of a unit's planes x 4 rows x 62 columns (64 entries at least)
  const unsigned v = ((unsigned)pl.planes_per_seg * (unsigned)kRows3d * (unsigned)s3::kOut / 8u + 63u) / 64u * 64u;
  return v < 64u ? 64u : v;
}
static bool soft3d_saves(const Shape& s) { return soft3d_supported(s, 1) && s.N < ((int64_t)1 << 31); }
size_t soft3d_state_bytes(const Shape& s) {
  if (!soft3d_saves(s)) return 256;
  const Plan3d pl = plan3d<float>(s);
  return state_bytes(s.batch, (size_t)pl.grid.x * 4, state_cap3(pl));
}
bool soft3d_state_supported(const Shape& s, int T) { return soft3d_supported(s, T) && soft3d_saves(s); }

static SoftStateHeader state_header3(const Shape& s, const Plan3d& pl, bool tiltc) {
  SoftStateHeader h;
  h.magic = kSoftStateMagic;
  h.D = (int)s.D;
  h.H = (int)s.H;
  h.W = (int)s.W;
  h.batch = (int)s.batch;
  h.nstrip = pl.nstrip;
  h.nseg = pl.nseg;
  h.rows_per_seg = pl.planes_per_seg;
  h.units = (int)pl.grid.x * 4;
  h.tiltc = tiltc ? 1 : 0;
  h.cap = state_cap3(pl);
  return h;
}

void launch_soft3d_fwd_save(const float* grid, const Shape& s, const float* u, float alpha, const float* tau, int T,
                            float lambda, float* chi, float* dtau, float* du, void* state, void* ws, hipStream_t st,
                            bool tiltc) {
  const Plan3d pl = plan3d<float>(s);
  const SoftStateHeader hdr = state_header3(s, pl, tiltc);
  const StateView sv = state_view(state, s.batch, (size_t)hdr.units);
  float* partial = static_cast<float*>(ws);
  double* mid = reinterpret_cast<double*>(static_cast<char*>(ws) + soft3d_partial_bytes(s, pl, T));
  const bool deriv = dtau || du;
#define ECC_GO(TC, DV)                                                                                        \
  hipLaunchKernelGGL((soft3d_fwd_save_kernel<TC, DV>), pl.grid, dim3(256), kSoft3Lds, st, grid, (int)s.D, (int)s.H, \
                     (int)s.W, s.N, pl.nstrip, pl.ngroup, pl.nseg, pl.planes_per_seg, u, alpha, tau, T,         \
                     kneg3d(lambda), partial, sv, hdr.cap)
  if (tiltc) { if (deriv) ECC_GO(true, true); else ECC_GO(true, false); }
  else       { if (deriv) ECC_GO(false, true); else ECC_GO(false, false); }
#undef ECC_GO
  const RedOut out = {chi, dtau, du, sv.hdr, sv.gen, hdr};
  launch_soft_reduce<5, true, 3>(partial, mid, (int)pl.grid.x * 4, s.batch, T, alpha, lambda, origin3(s, pl), out, st);
}

void launch_soft3d_bwd_saved(const float* grid, const Shape& s, const float* u, float alpha, const float* tau, int T,
                             float lambda, const float* gup, float* grad_X, const void* state, hipStream_t st,
                             bool tiltc) {
  const Plan3d pl = plan3d<float>(s);
  const SoftStateHeader expect = state_header3(s, pl, tiltc);
  const StateView sv = state_view(const_cast<void*>(state), s.batch, (size_t)expect.units);
  launch_clear_f32(grad_X, s.N * s.batch, st);  // zero away from the critical vertices
  const dim3 g((unsigned)expect.units, (unsigned)s.batch);
  if (tiltc)
    hipLaunchKernelGGL(soft3d_bwd_saved_kernel<true>, g, dim3(256), 0, st, grid, (int)s.D, (int)s.H, (int)s.W, s.N, u,
                       alpha, tau, T, kneg3d(lambda), lambda, gup, grad_X, sv, expect);
  else
    hipLaunchKernelGGL(soft3d_bwd_saved_kernel<false>, g, dim3(256), 0, st, grid, (int)s.D, (int)s.H, (int)s.W, s.N, u,
                       alpha, tau, T, kneg3d(lambda), lambda, gup, grad_X, sv, expect);
}

}  // namespace ecc
