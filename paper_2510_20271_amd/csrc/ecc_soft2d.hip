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
// y = X(p) + alpha <u,p> is formed in float64 and carried as two floats (yh + yl), so that
// z = (tau_j - yh) - yl is the float64 difference to within an ulp of z; exp2 and the
// reciprocal run on the float32 transcendental unit.  An entry whose y lies so far outside
// [min tau, max tau] that every sigmoid is 0 or 1 to 2^-64 is not evaluated at all: it adds
// c to every threshold (sigma = 1) or nothing, and nothing to the derivatives.
#include "ecc_sweep2d.h"
#include "ecc_soft_saved.h"
#include "ecc_soft_reduce.h"

namespace ecc {

constexpr int kSoftTL = 4;  // thresholds per lane

struct SoftEntry {
  float yh, yl;  // X(p) + alpha <u,p> = yh + yl
  float c;
  int col, row;
  int pad;
};

struct SoftCommon {
  typedef SoftEntry Entry;
  static constexpr bool kTrackRange = false;
  double ux, uy, alpha;
  float tj[kSoftTL];  // this lane's thresholds
  int T;
  int nt;  // threshold slots in use: ceil(T / 64)
  float kneg;
  float sat_lo, sat_hi;  // y <= sat_lo: every sigma is 1;  y >= sat_hi: every sigma is 0 (to 2^-64)
  // The sweep ran on the tilted field (c of the tilted field): the value it hands over
  // is the tilted one in float32; X is read again so that y is formed as always.
  const float* xsrc;  // this item's grid, or null when the sweep ran on X itself
  int xW;
  __device__ __forceinline__ Entry make(float v, int c, int col, int row) const {
    Entry e;
    if (xsrc) v = xsrc[(int64_t)row * xW + col];  // wave-uniform condition
    const double y = (double)v + alpha * (ux * (double)col + uy * (double)row);
    e.yh = (float)y;
    e.yl = (float)(y - (double)e.yh);
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
    float lo = INFINITY, hi = -INFINITY;
#pragma unroll
    for (int t = 0; t < kSoftTL; ++t) {
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
  // Packs the entries of buf[0..n) that have to be evaluated to the front of buf (a wave's LDS
  // reads and writes execute in order: every lane has read its entry before any lane overwrites
  // one) and returns how many there are; *csat receives the sum of c over the dropped entries whose
  // sigmoids are all 1 (dropped entries whose sigmoids are all 0 add nothing).
  __device__ __forceinline__ int drop_saturated(Entry* buf, int n, float* csat) const {
    const int lane = threadIdx.x & (kWave - 1);
    Entry e = buf[lane < n ? lane : 0];
    const bool in = lane < n;
    const bool keep = in && e.yh > sat_lo && e.yh < sat_hi;
    const unsigned long long m = __builtin_amdgcn_ballot_w64(keep);
    const int kept = __builtin_popcountll(m);
    if (kept == n) return n;  // wave-uniform: nothing to drop
    if (csat) {
      const float ones = wave_sum_lane63((in && e.yh <= sat_lo) ? e.c : 0.0f);
      *csat += __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, ones), kWave - 1));
    }
    const int pos = (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
    if (keep) buf[pos] = e;
    return kept;
  }
  __device__ __forceinline__ float zarg(int t, float yh, float yl) const { return (tj[t] - yh) - yl; }
};

struct SoftFwdSink : SoftCommon {
  static constexpr bool kZeroFill = false;
  float acc[kSoftTL];
  float csat;  // sum of c over the entries whose sigmoids are all 1 (wave-uniform)
  __device__ __forceinline__ void consume(Entry* buf, int n) {
    n = drop_saturated(buf, n, &csat);
    for (int e = 0; e < n; ++e) {
      const float yh = buf[e].yh, yl = buf[e].yl;
      const float c = buf[e].c;
#pragma unroll
      for (int t = 0; t < kSoftTL; ++t) {
        if (t < nt) {  // wave-uniform
          const float ex = soft_exp_neg(zarg(t, yh, yl), kneg);
          acc[t] += c * __builtin_amdgcn_rcpf(1.0f + ex);
        }
      }
    }
  }
  __device__ __forceinline__ float total(int t) const { return acc[t] + csat; }
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
  __device__ __forceinline__ void consume(Entry* buf, int n) {
    const int lane = threadIdx.x & (kWave - 1);
    n = drop_saturated(buf, n, nullptr);  // sigma' < 2^-64 lambda at every threshold; grad_X stays 0 there
    for (int e = 0; e < n; ++e) {
      const float yh = buf[e].yh, yl = buf[e].yl;
      const float c = buf[e].c;
      const float rx = (float)(buf[e].col - col0), ry = (float)(buf[e].row - row0);
      float gd = 0.0f;
#pragma unroll
      for (int t = 0; t < kSoftTL; ++t) {
        if (t < nt) {  // wave-uniform
          const float ex = soft_exp_neg(zarg(t, yh, yl), kneg);
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

static unsigned state_cap(const Plan2d& pl) {
  // room for one vertex in eight of a unit's rows x 248 columns (64 entries at least)
  const unsigned v = (unsigned)pl.rows_per_seg * (unsigned)kStripOut / 8u;
  return (v < 64u ? 64u : v);
}
size_t soft2d_state_bytes(const Shape& s) {
  if (!soft2d_supported(s, 1)) return 256;
  const Plan2d pl = plan2d<float>(s, true);
  return state_bytes(s.batch, (size_t)pl.nstrip * pl.nseg, state_cap(pl));
}

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
  queue.sink.csat = 0.f;
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
      if (j < T) out[j] = queue.sink.total(t);
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


// Forward pass that saves its critical vertices: chi as SoftFwdSink, optionally the sums of
// Eq. 9 / Eq. 10 in the same pass (they share the sigmoid), and every entry appended to the
// unit's own list in the state buffer.
template <bool DERIV>
struct SoftSaveSink : SoftCommon {
  static constexpr bool kZeroFill = false;
  float acc[kSoftTL], a0[kSoftTL], ax[kSoftTL], ay[kSoftTL];
  float csat;
  int W, col0, row0;
  SavedEntry* list;     // this unit's list
  unsigned cap, saved;  // saved: entries seen so far (wave-uniform; may pass cap)
  __device__ __forceinline__ void consume(Entry* buf, int n) {
    const int lane = threadIdx.x & (kWave - 1);
    if (lane < n && saved + (unsigned)lane < cap) {
      const Entry e = buf[lane];
      SavedEntry o;
      o.y = (double)e.yh + (double)e.yl;
      o.idx = e.row * W + e.col;
      o.c = (int)e.c;
      list[saved + lane] = o;
    }
    saved += (unsigned)n;
    n = drop_saturated(buf, n, &csat);
    for (int e = 0; e < n; ++e) {
      const float yh = buf[e].yh, yl = buf[e].yl;
      const float c = buf[e].c;
      const float rx = (float)(buf[e].col - col0), ry = (float)(buf[e].row - row0);
#pragma unroll
      for (int t = 0; t < kSoftTL; ++t) {
        if (t < nt) {  // wave-uniform
          const float ex = soft_exp_neg(zarg(t, yh, yl), kneg);
          const float sg = __builtin_amdgcn_rcpf(1.0f + ex);
          acc[t] += c * sg;
          if (DERIV) {
            const float cd = c * (ex * sg * sg);  // c sigma (1 - sigma)
            a0[t] += cd;
            ax[t] += cd * rx;
            ay[t] += cd * ry;
          }
        }
      }
    }
  }
};

// partial[((item * units + unit) * T + j) * 4 + {0: chi, 1: A0, 2: Ax, 3: Ay}]
template <bool TILTC, bool DERIV>
__global__ __launch_bounds__(256) void soft2d_fwd_save_kernel(const float* __restrict__ grid, int H, int W, int64_t N,
                                                              int nstrip, int nseg, int rows_per_seg,
                                                              const float* __restrict__ u, float alpha,
                                                              const float* __restrict__ tau, int T, float kneg,
                                                              float* __restrict__ partial, StateView sv, unsigned cap) {
  extern __shared__ int smem[];
  float* ring;
  SoftEntry* qbuf;
  soft_lds(smem, ring, qbuf);
  WaveQueue<SoftSaveSink<DERIV>> queue;
  queue.buf = qbuf;
  queue.count = 0;
  SoftSaveSink<DERIV>& s = queue.sink;
  s.init(u, alpha, tau, T, kneg);
#pragma unroll
  for (int t = 0; t < kSoftTL; ++t) s.acc[t] = s.a0[t] = s.ax[t] = s.ay[t] = 0.f;
  s.csat = 0.f;
  const int unit = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), units = nstrip * nseg;
  s.W = W;
  s.col0 = (unit % nstrip) * kStripOut - kNC;
  s.row0 = (unit / nstrip) * rows_per_seg;
  s.cap = cap;
  s.saved = 0u;
  s.list = sv.lists + ((size_t)blockIdx.y * units + (unit < units ? unit : 0)) * cap;
  const unsigned next_gen = *sv.gen + 1u;  // (the reduction kernel that follows stores it)
  WaveRange range;
  if constexpr (TILTC) {
    s.xsrc = grid + (int64_t)blockIdx.y * N;
    s.xW = W;
    const DirArgs da = {u, alpha, 1, 2};
    sweep2d_wave<float>(grid + (int64_t)blockIdx.y * N, H, W, N, nstrip, nseg, rows_per_seg, queue, ring, range,
                        load_tilt(da, 0));
  } else {
    sweep2d_wave<float>(grid + (int64_t)blockIdx.y * N, H, W, N, nstrip, nseg, rows_per_seg, queue, ring, range,
                        NoTilt());
  }
  if (unit < units) {
    const int lane = threadIdx.x & (kWave - 1);
    if (lane == 0) {
      sv.counts[(size_t)blockIdx.y * units + unit] = s.saved;
      if (s.saved > cap) sv.overflow[blockIdx.y] = next_gen;
    }
    float4* out = reinterpret_cast<float4*>(partial) + ((int64_t)blockIdx.y * units + unit) * (int64_t)T;
#pragma unroll
    for (int t = 0; t < kSoftTL; ++t) {
      const int j = lane + kWave * t;
      if (j < T) out[j] = make_float4(s.acc[t] + s.csat, s.a0[t], s.ax[t], s.ay[t]);
    }
  }
}

// origin of a unit's coordinates, for the reduction of ecc_soft_reduce.h
struct Origin2 {
  int nstrip, rows_per_seg;
  __device__ __forceinline__ void operator()(int unit, int (&o)[3]) const {
    o[0] = (unit % nstrip) * kStripOut - kNC;
    o[1] = (unit / nstrip) * rows_per_seg;
    o[2] = 0;
  }
};

// grad_X from the saved lists (Eq. 8 contracted with the upstream gradient).  A block takes one
// unit of the forward sweep.  It clears the part of grad_X the unit owns (its rows x its 248
// output columns), then goes through the unit's list 256 entries at a time: entries whose
// sigmoids are all saturated are dropped (grad_X stays 0 there, see soft_sat_bounds), the others
// are packed into an LDS stage and get eight lanes each -- every lane sums an eighth of the
// thresholds, three lane swaps add the eight partial sums.  A unit's work is spread over four
// waves because the lists are uneven: with a tilt, whole regions of the image are saturated and
// the call lasts as long as its busiest unit.
// An item whose lists cannot be used (header of another shape, a unit ran out of room) is
// computed from the grid instead, vertex by vertex with the plain stencil: slow, but rare.
template <bool TILTC>
__global__ __launch_bounds__(256) void soft2d_bwd_saved_kernel(const float* __restrict__ grid, int H, int W, int64_t N,
                                                               int nstrip, int nseg, int rows_per_seg,
                                                               const float* __restrict__ u, float alpha,
                                                               const float* __restrict__ tau, int T, float kneg,
                                                               float lambda, const float* __restrict__ gup,
                                                               float* __restrict__ grad_X, StateView sv,
                                                               SoftStateHeader expect) {
  const int item = blockIdx.y, unit = blockIdx.x, units = nstrip * nseg;
  const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
  __shared__ float stau[kSoftTL * kWave];
  __shared__ float sg[kSoftTL * kWave];
  __shared__ StagedEntry stage[256];
  __shared__ float sred[2][4];
  __shared__ int skept[4];
  // Everything the block needs from memory is requested up front, so that the call costs one
  // round trip to memory and not four in a row: the state's header words, the unit's count and
  // the first 256 entries of its list (or as many as the unit has room for, whatever the count says).
  const bool usable = state_usable(sv, expect, item);
  const unsigned cnt_raw = sv.counts[(size_t)item * units + unit];
  const SavedEntry* list = sv.lists + ((size_t)item * units + unit) * expect.cap;
  SavedEntry first = list[min((unsigned)threadIdx.x, expect.cap - 1u)];
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
  float* gx = grad_X + (int64_t)item * N;
  const int seg = unit / nstrip, strip = unit - seg * nstrip;
  const int x0 = strip * kStripOut, x1 = min(x0 + kStripOut, W);
  const int y0 = seg * rows_per_seg, y1 = min(y0 + rows_per_seg, H);
  if (usable) {  // block-uniform
    if (((reinterpret_cast<uintptr_t>(gx) | (uintptr_t)(W * 4) | (uintptr_t)(x0 * 4) | (uintptr_t)((x1 - x0) * 4)) & 15) == 0) {
      const int w4 = (x1 - x0) / 4;  // 16-byte stores: rows, first column and width all fit
      for (int y = y0 + wv; y < y1; y += 4)
        if (lane < w4) reinterpret_cast<float4*>(gx + (int64_t)y * W + x0)[lane] = make_float4(0.f, 0.f, 0.f, 0.f);
    } else {
      for (int y = y0 + wv; y < y1; y += 4)
        for (int x = x0 + lane; x < x1; x += kWave) gx[(int64_t)y * W + x] = 0.0f;
    }
  }
  __syncthreads();  // thresholds in LDS; the fill has reached memory before any entry is written
  lo = fminf(fminf(sred[0][0], sred[0][1]), fminf(sred[0][2], sred[0][3]));
  hi = fmaxf(fmaxf(sred[1][0], sred[1][1]), fmaxf(sred[1][2], sred[1][3]));
  float sat_lo, sat_hi;
  soft_sat_bounds(lo, hi, kneg, sat_lo, sat_hi);

  if (!usable) {
    const float* g = grid + (int64_t)item * N;
    Tilt tilt;
    if (TILTC) {
      const DirArgs da = {u, alpha, 1, 2};
      tilt = load_tilt(da, 0);
    }
    const double ux = (double)u[0], uy = (double)u[1];
    for (int y = y0 + wv; y < y1; y += 4) {
      for (int x = x0 + lane; x < x1; x += kWave) {
        int c;
        if (TILTC) c = coeff_tilted_at<2>(g, tilt, 1, H, W, 0, y, x);
        else c = coeff_at<float, 2>(g, 1, H, W, 0, y, x);
        float out = 0.0f;
        if (c != 0) {
          const double yv = (double)g[(int64_t)y * W + x] + (double)alpha * (ux * (double)x + uy * (double)y);
          const float yh = (float)yv, yl = (float)(yv - (double)yh);
          if (yh > sat_lo && yh < sat_hi) {
            float gd = 0.0f;
            for (int j = 0; j < T; ++j) gd += sg[j] * soft_dsig(stau[j], yh, yl, kneg);
            out = -lambda * (float)c * gd;
          }
        }
        gx[(int64_t)y * W + x] = out;
      }
    }
    return;
  }

  saved_lists_to_grad(list, cnt_raw, expect.cap, first, stau, sg, T, kneg, lambda, sat_lo, sat_hi, gx, N, stage, skept);
}

static float kneg2d(float lambda) { return (float)(-(double)lambda * 1.4426950408889634); }
constexpr size_t kSoftLds = ring_bytes2d<SoftEntry>();

bool soft2d_supported(const Shape& s, int T) {
  return s.D == 1 && s.ndim == 2 && T <= kSoftTL * kWave && s.W >= 8 && s.W <= (1 << 22) &&
         s.H <= (1 << 30) && s.N < ((int64_t)1 << 31);
}

// per-unit partial sums (up to four floats per unit and threshold), a multiple of 256 bytes
static size_t soft2d_partial_bytes(const Shape& s, const Plan2d& pl, int T) {
  const size_t n = (size_t)s.batch * pl.nstrip * pl.nseg * (size_t)T * 4 * sizeof(float);
  return (n + 255) / 256 * 256;
}
static double* soft2d_mid(void* ws, const Shape& s, const Plan2d& pl, int T) {
  return reinterpret_cast<double*>(static_cast<char*>(ws) + soft2d_partial_bytes(s, pl, T));
}

size_t soft2d_workspace_bytes(const Shape& s, int T) {
  if (!soft2d_supported(s, T)) return 0;
  const Plan2d pl = plan2d<float>(s, true);
  return (size_t)256 + soft2d_partial_bytes(s, pl, T) + soft_reduce_mid_bytes(s.batch, T);
}

void launch_soft2d_fwd(const float* grid, const Shape& s, const float* u, float alpha, const float* tau,
                       int T, float lambda, float* chi, void* ws, hipStream_t st, bool tiltc) {
  const Plan2d pl = plan2d<float>(s, true);
  float* partial = static_cast<float*>(ws);
  profile_mark(st, false);
  if (tiltc)
    hipLaunchKernelGGL(soft2d_fwd_kernel<true>, pl.grid, dim3(256), kSoftLds, st, grid, (int)s.H, (int)s.W, s.N,
                       pl.nstrip, pl.nseg, pl.rows_per_seg, u, alpha, tau, T, kneg2d(lambda), partial);
  else
    hipLaunchKernelGGL(soft2d_fwd_kernel<false>, pl.grid, dim3(256), kSoftLds, st, grid, (int)s.H, (int)s.W, s.N,
                       pl.nstrip, pl.nseg, pl.rows_per_seg, u, alpha, tau, T, kneg2d(lambda), partial);
  profile_mark(st, true);
  const RedOut out = {chi, nullptr, nullptr, nullptr, nullptr, {}};
  launch_soft_reduce<1, true, -1>(partial, soft2d_mid(ws, s, pl, T), pl.nstrip * pl.nseg, s.batch, T, alpha, lambda,
                                  Origin2{pl.nstrip, pl.rows_per_seg}, out, st);
}

void launch_soft2d_bwd(const float* grid, const Shape& s, const float* u, float alpha, const float* tau,
                       int T, float lambda, const float* gup, float* grad_X, float* dtau, float* du,
                       void* ws, hipStream_t st, bool tiltc) {
  const Plan2d pl = plan2d<float>(s, true);
  float* partial = (dtau || du) ? static_cast<float*>(ws) : nullptr;
  profile_mark(st, false);
  if (tiltc)
    hipLaunchKernelGGL(soft2d_bwd_kernel<true>, pl.grid, dim3(256), kSoftLds, st, grid, (int)s.H, (int)s.W, s.N,
                       pl.nstrip, pl.nseg, pl.rows_per_seg, u, alpha, tau, T, kneg2d(lambda), lambda, gup,
                       grad_X, partial);
  else
    hipLaunchKernelGGL(soft2d_bwd_kernel<false>, pl.grid, dim3(256), kSoftLds, st, grid, (int)s.H, (int)s.W, s.N,
                       pl.nstrip, pl.nseg, pl.rows_per_seg, u, alpha, tau, T, kneg2d(lambda), lambda, gup,
                       grad_X, partial);
  profile_mark(st, true);
  if (partial) {
    const RedOut out = {nullptr, dtau, du, nullptr, nullptr, {}};
    launch_soft_reduce<4, false, 2>(partial, soft2d_mid(ws, s, pl, T), pl.nstrip * pl.nseg, s.batch, T, alpha, lambda,
                                    Origin2{pl.nstrip, pl.rows_per_seg}, out, st);
  }
}

static SoftStateHeader state_header(const Shape& s, const Plan2d& pl, bool tiltc) {
  SoftStateHeader h;
  h.magic = kSoftStateMagic;
  h.D = 1;
  h.units = pl.nstrip * pl.nseg;
  h.H = (int)s.H;
  h.W = (int)s.W;
  h.batch = (int)s.batch;
  h.nstrip = pl.nstrip;
  h.nseg = pl.nseg;
  h.rows_per_seg = pl.rows_per_seg;
  h.tiltc = tiltc ? 1 : 0;
  h.cap = state_cap(pl);
  return h;
}

void launch_soft2d_fwd_save(const float* grid, const Shape& s, const float* u, float alpha, const float* tau, int T,
                            float lambda, float* chi, float* dtau, float* du, void* state, void* ws, hipStream_t st,
                            bool tiltc) {
  const Plan2d pl = plan2d<float>(s, true);
  const StateView sv = state_view(state, s.batch, (size_t)pl.nstrip * pl.nseg);
  const SoftStateHeader hdr = state_header(s, pl, tiltc);
  float* partial = static_cast<float*>(ws);
  const bool deriv = dtau || du;
  profile_mark(st, false);
#define ECC_GO(TC, DV)                                                                                        \
  hipLaunchKernelGGL((soft2d_fwd_save_kernel<TC, DV>), pl.grid, dim3(256), kSoftLds, st, grid, (int)s.H, (int)s.W, \
                     s.N, pl.nstrip, pl.nseg, pl.rows_per_seg, u, alpha, tau, T, kneg2d(lambda), partial, sv, hdr.cap)
  if (tiltc) { if (deriv) ECC_GO(true, true); else ECC_GO(true, false); }
  else       { if (deriv) ECC_GO(false, true); else ECC_GO(false, false); }
#undef ECC_GO
  profile_mark(st, true);
  const RedOut out = {chi, dtau, du, sv.hdr, sv.gen, hdr};
  launch_soft_reduce<4, true, 2>(partial, soft2d_mid(ws, s, pl, T), pl.nstrip * pl.nseg, s.batch, T, alpha, lambda,
                                 Origin2{pl.nstrip, pl.rows_per_seg}, out, st);
}

void launch_soft2d_bwd_saved(const float* grid, const Shape& s, const float* u, float alpha, const float* tau, int T,
                             float lambda, const float* gup, float* grad_X, const void* state, hipStream_t st,
                             bool tiltc) {
  const Plan2d pl = plan2d<float>(s, true);
  const StateView sv = state_view(const_cast<void*>(state), s.batch, (size_t)pl.nstrip * pl.nseg);
  const SoftStateHeader expect = state_header(s, pl, tiltc);
  const dim3 g((unsigned)(pl.nstrip * pl.nseg), (unsigned)s.batch);
  profile_mark(st, false);
  if (tiltc)
    hipLaunchKernelGGL(soft2d_bwd_saved_kernel<true>, g, dim3(256), 0, st, grid, (int)s.H, (int)s.W, s.N, pl.nstrip,
                       pl.nseg, pl.rows_per_seg, u, alpha, tau, T, kneg2d(lambda), lambda, gup, grad_X, sv, expect);
  else
    hipLaunchKernelGGL(soft2d_bwd_saved_kernel<false>, g, dim3(256), 0, st, grid, (int)s.H, (int)s.W, s.N, pl.nstrip,
                       pl.nseg, pl.rows_per_seg, u, alpha, tau, T, kneg2d(lambda), lambda, gup, grad_X, sv, expect);
  profile_mark(st, true);
}

}  // namespace ecc
