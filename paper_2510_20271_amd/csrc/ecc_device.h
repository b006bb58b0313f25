// Device-side helpers shared by the HIP kernels of libecc_hip (gfx950 only).
//
// Order on vertices (per-vertex form of the curve, Eq. 3 of the paper): q comes
// before p when X(q) < X(p), or X(q) == X(p) and q has the smaller C-order
// linear index.  For a neighbour with a larger index that is a strict "<", for
// a neighbour with a smaller index it is "<=".
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ecc_internal.h"

namespace ecc {

constexpr int kWave = 64;

// ---- neighbourhood ring of the 3x3 stencil --------------------------------
// bit k of an 8-bit ring mask: 0:(+x) 1:(+x,+y) 2:(+y) 3:(-x,+y) 4:(-x)
// 5:(-x,-y) 6:(-y) 7:(+x,-y).  Even bits are edge neighbours, odd bits the
// diagonal vertex of the square between its two ring neighbours.
__device__ __forceinline__ int ring_bit(int dy, int dx) {
  // dy,dx in {-1,0,1}, not both 0
  constexpr int tab[3][3] = {{5, 6, 7}, {4, -1, 0}, {3, 2, 1}};
  return tab[dy + 1][dx + 1];
}

// 2D coefficient from the ring of "neighbour comes before p" bits:
// 1 - #edges + #squares, a square being charged to p when its three other
// vertices all come before p.
__device__ __forceinline__ int coeff_ring(unsigned m) {
  unsigned w = m | (m << 8);
  unsigned sq = m & (w >> 1) & (w >> 7) & 0xAAu;
  return 1 - __popc(m & 0x55u) + __popc(sq);
}

// 3D coefficient.  a: ring of the in-plane neighbours; up/dn: rings of the 8
// outer vertices of the plane above (+z) / below (-z); up0/dn0: the vertex
// straight above / below.  A cell reaching into the upper plane is charged to
// p iff the vertical edge is, and the cell's in-plane footprint is charged
// with every footprint vertex ALSO preceding in the upper plane; its sign is
// minus the sign of the footprint.  Hence
//   c = ring(a) - up0 * ring(a & up) - dn0 * ring(a & dn).
__device__ __forceinline__ int coeff_3d(unsigned a, unsigned up, bool up0, unsigned dn, bool dn0) {
  int c = coeff_ring(a);
  if (up0) c -= coeff_ring(a & up);
  if (dn0) c -= coeff_ring(a & dn);
  return c;
}

// Coefficient of the vertex (z,y,x) read straight from global memory, with
// bounds checks; the reference path for every dtype and shape.
// REV: larger values come first (ties still by index).  OUTFIRST: vertices outside
// the grid come before every vertex instead of after.  Both together give, up to the
// sign (-1)^d the caller applies, the top-cell construction (see TopCells below);
// REV alone the vertex construction of superlevel sets; OUTFIRST alone the top-cell
// construction of superlevel sets.
// The field is given by value(index, z, y, x), called for in-grid vertices only.
template <int ND, bool OUTFIRST, bool REV, typename F>
__device__ __forceinline__ int coeff_of(const F& value, int64_t D, int64_t H, int64_t W, int64_t z, int64_t y,
                                        int64_t x) {
  const auto vp = value((z * H + y) * W + x, z, y, x);
  unsigned ring[3] = {0u, 0u, 0u};
  bool centre[3] = {false, false, false};
  constexpr int z0 = (ND == 3) ? -1 : 0, z1 = (ND == 3) ? 1 : 0;
#pragma unroll
  for (int dz = z0; dz <= z1; ++dz) {
#pragma unroll
    for (int dy = -1; dy <= 1; ++dy) {
#pragma unroll
      for (int dx = -1; dx <= 1; ++dx) {
        if (dz == 0 && dy == 0 && dx == 0) continue;
        const int64_t qz = z + dz, qy = y + dy, qx = x + dx;
        bool b = OUTFIRST;
        if (qz >= 0 && qz < D && qy >= 0 && qy < H && qx >= 0 && qx < W) {
          const auto vq = value((qz * H + qy) * W + qx, qz, qy, qx);
          const bool later = (dz > 0) || (dz == 0 && (dy > 0 || (dy == 0 && dx > 0)));
          if (REV) b = later ? (vq > vp) : (vq >= vp);
          else b = later ? (vq < vp) : (vq <= vp);
        }
        if (dy == 0 && dx == 0) centre[dz + 1] = b;
        else ring[dz + 1] |= (b ? 1u : 0u) << ring_bit(dy, dx);
      }
    }
  }
  if (ND == 2) return coeff_ring(ring[1]);
  return coeff_3d(ring[1], ring[2], centre[2], ring[0], centre[0]);
}
template <typename T, int ND, bool OUTFIRST = false, bool REV = false>
__device__ __forceinline__ int coeff_at(const T* __restrict__ g, int64_t D, int64_t H, int64_t W,
                                        int64_t z, int64_t y, int64_t x) {
  return coeff_of<ND, OUTFIRST, REV>([g](int64_t i, int64_t, int64_t, int64_t) { return g[i]; }, D, H, W, z, y, x);
}

// ---- bins -----------------------------------------------------------------
// Header at the start of the workspace of ecc_hard, followed by the threshold
// table (float[bins]) at byte offset kTableOffset, the per-item list counters and
// the per-item lists of critical vertices (single-pass mode).
struct HardHeader {
  unsigned min_key;  // order-preserving uint encodings of the batch min / max
  unsigned max_key;
  float lo;          // float(lo) used for the bin guess
  float scale;       // bins / (hi - lo), 0 when hi <= lo
  unsigned overflow; // single-pass mode: a critical-vertex list ran out of room
};
constexpr size_t kTableOffset = 256;

__device__ __forceinline__ unsigned float_key(float f) {
  unsigned b = __float_as_uint(f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_float(unsigned k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// Threshold b of B equal-width bins over [lo, hi]: t_b = float32(lo + (b+1)(hi-lo)/B)
// in float64 with every operation rounded on its own (no contraction), the last
// one float32(hi); and the factor of the bin guess, B / (hi - lo) (0 when hi <= lo).
__device__ __forceinline__ float threshold_at(int b, int bins, double lo, double hi) {
  const double w = __dsub_rn(hi, lo);
  const double t = __dadd_rn(lo, __ddiv_rn(__dmul_rn((double)(b + 1), w), (double)bins));
  return (b == bins - 1) ? __double2float_rn(hi) : __double2float_rn(t);
}
__device__ __forceinline__ float bin_scale(int bins, double lo, double hi) {
  const double w = __dsub_rn(hi, lo);
  return (w > 0.0) ? __double2float_rn(__ddiv_rn((double)bins, w)) : 0.0f;
}

// bin(x) = min{ b : x <= t_b } on the float32 table; `bins` when x is above
// every threshold.  The guess comes from float arithmetic, the answer from
// comparisons with the table only, so it is the same on every machine.
__device__ __forceinline__ int bin_from_table(float x, const float* __restrict__ t, int bins,
                                              float lo, float scale) {
  float f = (x - lo) * scale;
  int b = (f > 0.0f) ? (int)fminf(f, (float)(bins - 1)) : 0;
  while (b > 0 && x <= t[b - 1]) --b;
  while (b < bins && x > t[b]) ++b;
  return b;
}

// Superlevel curves (X >= tau) are read at the LOWER edges of the same bins:
// t'_0 = float32(lo), t'_b = t_{b-1}.  bin(x) = max{ b : t'_b <= x }; `bins` when
// x is below every threshold (in no superlevel set).
__device__ __forceinline__ float threshold_lower_at(int b, int bins, double lo, double hi) {
  return (b == 0) ? __double2float_rn(lo) : threshold_at(b - 1, bins, lo, hi);
}
__device__ __forceinline__ int bin_super_from_table(float x, const float* __restrict__ t, int bins,
                                                    float lo, float scale) {
  float f = (x - lo) * scale;
  int b = (f > 0.0f) ? (int)fminf(f, (float)(bins - 1)) : 0;
  while (b < bins - 1 && x >= t[b + 1]) ++b;
  while (b >= 0 && x < t[b]) --b;
  return b < 0 ? bins : b;
}
// integer grids without a range: thresholds t_b = b; X <= b (sublevel) or X >= b (superlevel)
template <bool SUPER>
__device__ __forceinline__ int bin_levels(float v, int bins) {
  if (SUPER) return (v < (float)bins) ? (int)v : bins - 1;
  return (v < (float)bins) ? (int)v : bins;
}
template <bool SUPER>
__device__ __forceinline__ int bin_table(float x, const float* __restrict__ t, int bins, float lo, float scale) {
  return SUPER ? bin_super_from_table(x, t, bins, lo, scale) : bin_from_table(x, t, bins, lo, scale);
}

template <typename T> __device__ __forceinline__ float as_float(T v) { return (float)v; }

// Two-byte element types the strip / tube sweeps also load directly (all three widen to float32
// without rounding, so the sweep runs on exactly the grid's values).
struct Bf16 {
  uint16_t bits;
  __device__ __forceinline__ operator float() const { return __uint_as_float((unsigned)bits << 16); }
};
typedef _Float16 F16;
// float32 view of a two-byte element given as the low 16 bits of `b`
template <typename T> __device__ __forceinline__ float widen16(unsigned b);
template <> __device__ __forceinline__ float widen16<uint16_t>(unsigned b) { return (float)(b & 0xffffu); }
template <> __device__ __forceinline__ float widen16<int16_t>(unsigned b) { return (float)(int16_t)(uint16_t)b; }
template <> __device__ __forceinline__ float widen16<F16>(unsigned b) {
  return (float)__builtin_bit_cast(F16, (uint16_t)b);
}
template <> __device__ __forceinline__ float widen16<Bf16>(unsigned b) { return __uint_as_float(b << 16); }
// element types that have a -0 (made +0 as the value is loaded, so that equal values differ by +0)
template <typename T> struct HasNegZero { static constexpr bool value = false; };
template <> struct HasNegZero<float> { static constexpr bool value = true; };
template <> struct HasNegZero<F16> { static constexpr bool value = true; };
template <> struct HasNegZero<Bf16> { static constexpr bool value = true; };

// ---- tilted filtration (directional curves) ------------------------------------
// The sweeps can add a linear function of the vertex's coordinates to the field as
// they load it: Y(p) = X(p) + t(p), t = fl(fl(fl(a_x x) + fl(a_y y)) + fl(a_z z))
// (the last term in 3D only), a_d = fl(alpha u_d), every operation a float32 one
// in this order.  A launch then runs over directions x batch items: blockIdx.y =
// direction * batch + item.
// float32 product / sum rounded on their own: never contracted into an fma with a
// neighbouring operation (the tilt's rounding sequence is part of its definition)
__device__ __forceinline__ float mul_rn(float a, float b) {
#pragma clang fp contract(off)
  return a * b;
}
__device__ __forceinline__ float add_rn(float a, float b) {
#pragma clang fp contract(off)
  return a + b;
}

//
// TopCells is the third way a sweep can take the field: negated, with everything
// outside the grid coming first (-inf).  The vertex coefficient of that order is,
// up to the sign (-1)^d, the coefficient of the top-cell construction (grid
// points are squares / cubes; a lower cell belongs to the FIRST top cell around
// it), so the same stencil serves both constructions; the value that is binned is
// the original one.
struct NoTilt {
  static constexpr bool kOn = false, kNeg = false, kTop = false, kRaw = false;
  float ax, ay, az;
};
struct Tilt {
  static constexpr bool kOn = true, kNeg = false, kTop = false, kRaw = false;
  float ax, ay, az;
};
struct TopCells {
  static constexpr bool kOn = false, kNeg = true, kTop = true, kRaw = false;
  float ax, ay, az;
};
// Superlevel sets (X >= tau): the same two constructions on the descending order.
// Vertex construction: the negated field, outside last (kNeg only).  Top-cell
// construction: the descending order reversed is the field's own order, so the
// field is swept as it is with the top-cell conventions (kTop only).
struct Super {
  static constexpr bool kOn = false, kNeg = true, kTop = false, kRaw = false;
  float ax, ay, az;
};
struct TopSuper {
  static constexpr bool kOn = false, kNeg = false, kTop = true, kRaw = false;
  float ax, ay, az;
};
// Tilted sweep whose consumer wants the untilted value of a critical vertex (the soft
// path with the tilted field's coefficient): kRaw.
struct TiltRaw : Tilt {
  static constexpr bool kRaw = true;
};
// kNeg: the field is negated as it is loaded (zeros stay +0).  kTop: what lies
// outside the grid comes before every vertex, and the coefficient is (-1)^d times
// the stencil's.  The value that is binned is always the original one.
enum SweepMode { kPlain = 0, kTilted = 1, kTopCells = 2, kSuper = 3, kTopSuper = 4 };
__host__ __device__ constexpr bool mode_is_super(int mode) { return mode == kSuper || mode == kTopSuper; }
template <int MODE> struct ModeTransform { typedef NoTilt type; };
template <> struct ModeTransform<kTopCells> { typedef TopCells type; };
template <> struct ModeTransform<kSuper> { typedef Super type; };
template <> struct ModeTransform<kTopSuper> { typedef TopSuper type; };
constexpr int mode_of_conv(int conv) {
  return conv == 0 ? kPlain : conv == kConvTop ? kTopCells : conv == kConvSuper ? kSuper : kTopSuper;
}
struct DirArgs {
  const float* u;  // device [ndir][ndim]
  float alpha;
  int batch;       // items per direction
  int ndim;
};
__device__ __forceinline__ Tilt load_tilt(const DirArgs& d, int dir) {
  Tilt t;
  t.ax = mul_rn(d.alpha, d.u[dir * d.ndim]);
  t.ay = mul_rn(d.alpha, d.u[dir * d.ndim + 1]);
  t.az = d.ndim == 3 ? mul_rn(d.alpha, d.u[dir * d.ndim + 2]) : 0.0f;
  return t;
}

// The tilted field at one vertex, as every sweep forms it.
template <int ND>
__device__ __forceinline__ float tilted_value(float v, const Tilt& t, int64_t z, int64_t y, int64_t x) {
  float tt = add_rn(mul_rn(t.ax, (float)x), mul_rn(t.ay, (float)y));
  if (ND == 3) tt = add_rn(tt, mul_rn(t.az, (float)z));
  return add_rn(v, tt);
}
// Coefficient of the tilted field at one vertex (read straight from global memory).
template <int ND>
__device__ __forceinline__ int coeff_tilted_at(const float* __restrict__ g, const Tilt& t, int64_t D, int64_t H,
                                               int64_t W, int64_t z, int64_t y, int64_t x) {
  return coeff_of<ND, false, false>(
      [g, &t](int64_t i, int64_t qz, int64_t qy, int64_t qx) { return tilted_value<ND>(g[i], t, qz, qy, qx); }, D, H,
      W, z, y, x);
}

// Sum of v over the 64 lanes, delivered in lane 63: four steps inside each row of 16
// lanes (quad swaps, half-row and row mirrors), then the rows' totals handed on by
// row_bcast.  Data-parallel-primitive moves only: nothing goes through LDS, unlike a
// shuffle butterfly.  Fixed order, so the result is the same on every run.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move(float x) {  // 0 where the move has no source or the row is masked
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_sum_lane63(float v) {
  v += dpp_move<0xB1, 0xf>(v);   // quad_perm [1,0,3,2]
  v += dpp_move<0x4E, 0xf>(v);   // quad_perm [2,3,0,1]
  v += dpp_move<0x141, 0xf>(v);  // row_half_mirror
  v += dpp_move<0x140, 0xf>(v);  // row_mirror: every lane holds its row's sum
  v += dpp_move<0x142, 0xa>(v);  // row_bcast:15 into rows 1 and 3
  v += dpp_move<0x143, 0xc>(v);  // row_bcast:31 into rows 2 and 3: lane 63 holds the total
  return v;
}

// ---- sigmoid pieces shared by the fused soft kernels (Eq. 6, Eq. 8-10) ------
__device__ __forceinline__ float soft_exp_neg(float z, float kneg) {
  // exp(-lambda z) = 2^(kneg z); clamped so the result stays finite
  return __builtin_amdgcn_exp2f(fminf(kneg * z, 126.0f));
}

constexpr float kSatLog2 = 64.0f;  // |lambda z| log2(e) beyond which sigma is 0 or 1 and sigma' is 0

// Saturation bounds for thresholds in [lo, hi]: with k = lambda log2(e) = -kneg, sigma(tau - y) differs from
// 1 by less than 2^-64 for y <= lo - 64/k and from 0 for y >= hi + 64/k (a little margin covers
// the rounding of yh); sigma' is below 2^-64 lambda in both cases.
__device__ __forceinline__ void soft_sat_bounds(float lo, float hi, float kneg, float& sat_lo, float& sat_hi) {
  const float w = (kSatLog2 + 2.0f) / -kneg;
  sat_lo = lo - w - 1e-6f * fabsf(lo);
  sat_hi = hi + w + 1e-6f * fabsf(hi);
}

// ---- critical-vertex queue of a wave ----------------------------------------
// Critical vertices (c != 0) turn up a few lanes at a time.  Instead of running
// the binning code with most lanes idle, a wave appends (value, c) to a small
// LDS queue (lane-compacted with a ballot) and drains it 64 entries at a time
// with every lane busy.
// A sink names its entry type (what the queue stores per critical vertex), makes
// an entry from (value, c, column, row) and consumes the first n entries of the
// queue buffer with the whole wave (n is wave-uniform, n <= 64).
template <bool LEVELS, bool SUPER = false>
struct HistSink {  // drain target: the block's LDS histogram
  typedef float2 Entry;
  static constexpr bool kTrackRange = false;
  static constexpr bool kZeroFill = false;
  int* lhist;
  const float* table;  // float[bins] thresholds (LDS or global), unused for LEVELS
  int bins;
  float lo, scale;
  static __device__ __forceinline__ Entry make(float v, int c, int, int) {
    return make_float2(v, __int_as_float(c));
  }
  __device__ __forceinline__ void consume(const Entry* buf, int n) {
    const int lane = threadIdx.x & (kWave - 1);
    if (lane >= n) return;
    const Entry e = buf[lane];
    const float v = e.x;
    int b;
    if (LEVELS) b = bin_levels<SUPER>(v, bins);
    else b = bin_table<SUPER>(v, table, bins, lo, scale);
    if (b < bins) atomicAdd(&lhist[b], __float_as_int(e.y));
  }
  // the same with the entries already in registers: lane i < n holds (v, c)
  __device__ __forceinline__ void take(int n, float v, int c, unsigned = 0, unsigned = 0) {
    const int lane = threadIdx.x & (kWave - 1);
    if (lane >= n) return;
    int b;
    if (LEVELS) b = bin_levels<SUPER>(v, bins);
    else b = bin_table<SUPER>(v, table, bins, lo, scale);
    if (b < bins) atomicAdd(&lhist[b], c);
  }
};

// Drain target of the single-pass mode: a list of critical vertices (value, c)
// in the workspace.  A wave reserves n slots with one atomic; when the list is
// full the overflow flag is raised and the entries are dropped (the caller then
// runs the two-pass path instead).
// An item's list is split into sub-lists (up to 1024 of them, a block appends to
// sub-list blockIdx.x mod that number): atomics on one address serialise in the
// L2, and there is one per 64 critical vertices plus one per wave.
constexpr unsigned kMaxSubLists = 1024;
constexpr unsigned kMinSubListCap = 256;  // entries (unless the whole item has fewer)

struct ListSink {
  typedef float2 Entry;
  static constexpr bool kTrackRange = true;
  static constexpr bool kZeroFill = false;
  float2* list;       // this block's sub-list
  unsigned* counter;  // its fill count
  unsigned cap;       // entries per sub-list
  unsigned* overflow;
  static __device__ __forceinline__ Entry make(float v, int c, int, int) {
    return make_float2(v, __int_as_float(c));
  }
  __device__ __forceinline__ void consume(const Entry* buf, int n) {
    const int lane = threadIdx.x & (kWave - 1);
    unsigned base = 0;
    if (lane == 0) base = atomicAdd(counter, (unsigned)n);
    base = __builtin_amdgcn_readfirstlane(base);
    if (base + (unsigned)n <= cap) {
      if (lane < n) list[base + lane] = buf[lane];
    } else if (lane == 0) {
      atomicOr(overflow, 1u);
    }
  }
  __device__ __forceinline__ void take(int n, float v, int c, unsigned = 0, unsigned = 0) {
    const int lane = threadIdx.x & (kWave - 1);
    unsigned base = 0;
    if (lane == 0) base = atomicAdd(counter, (unsigned)n);
    base = __builtin_amdgcn_readfirstlane(base);
    if (base + (unsigned)n <= cap) {
      if (lane < n) list[base + lane] = make_float2(v, __int_as_float(c));
    } else if (lane == 0) {
      atomicOr(overflow, 1u);
    }
  }
};

constexpr int kQueueCap = 128;  // entries per wave

template <typename Sink>
struct WaveQueue {
  typedef typename Sink::Entry Entry;
  Entry* buf;  // wave-private LDS, kQueueCap entries
  int count;   // wave-uniform
  Sink sink;

  __device__ __forceinline__ void drain64() {
    const int lane = threadIdx.x & (kWave - 1);
    sink.consume(buf, kWave);
    const int rest = count - kWave;  // < 64
    Entry m = buf[lane < rest ? lane + kWave : lane];
    if (lane < rest) buf[lane] = m;
    count = rest;
  }
  // every lane calls; `active` lanes append the critical vertex (v, c) at (col, row)
  __device__ __forceinline__ void push(bool active, float v, int c, int col, int row) {
    const unsigned long long m = __builtin_amdgcn_ballot_w64(active);
    const int idx = count + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32),
                                                           __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
    if (active) buf[idx] = sink.make(v, c, col, row);
    count += __builtin_popcountll(m);
    if (count >= kWave) drain64();
  }
  __device__ __forceinline__ void flush() {
    if (count > 0) sink.consume(buf, count);  // wave-uniform
    count = 0;
  }
};

// Running min / max of the values a wave has seen (single-pass mode); merged
// into the header with ordered-uint atomics when the wave is done.
struct WaveRange {
  float lo = INFINITY, hi = -INFINITY;
  __device__ __forceinline__ void add(float v) {
    lo = fminf(lo, v);
    hi = fmaxf(hi, v);
  }
  __device__ __forceinline__ void add_if(float v, bool ok) {
    lo = fminf(lo, ok ? v : INFINITY);
    hi = fmaxf(hi, ok ? v : -INFINITY);
  }
  __device__ __forceinline__ void commit(HardHeader* h) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      lo = fminf(lo, __shfl_xor(lo, o));
      hi = fmaxf(hi, __shfl_xor(hi, o));
    }
    // Thousands of waves meet here; atomics on one address serialise in the L2, so
    // only a wave that would improve the value it reads issues one (a stale read can
    // only cause a needless atomic, never a missed one).
    if ((threadIdx.x & (kWave - 1)) == 0 && lo <= hi) {
      const unsigned klo = float_key(lo), khi = float_key(hi);
      if (klo < __hip_atomic_load(&h->min_key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
        atomicMin(&h->min_key, klo);
      if (khi > __hip_atomic_load(&h->max_key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
        atomicMax(&h->max_key, khi);
    }
  }
};

// ---- a list per block (ListArgs::heads) -------------------------------------------------------
// The four waves of a block append to one list through a fill count in LDS; when the sweep is done
// the block leaves the count and the range of the values it saw in its head.  own: 4 words of LDS.
__device__ __forceinline__ void block_list_begin(const ListArgs& la, ListSink& sink, unsigned* own) {
  const unsigned blk = blockIdx.y * gridDim.x + blockIdx.x;
  if (threadIdx.x == 0) {
    own[0] = 0u;
    own[1] = 0xffffffffu;
    own[2] = 0u;
    own[3] = 0u;
  }
  // the item's histogram, cleared by the item's blocks together
  for (int b = blockIdx.x * blockDim.x + threadIdx.x; b < la.bins; b += gridDim.x * blockDim.x)
    la.zero_hist[(int64_t)blockIdx.y * la.bins + b] = 0ull;
  __syncthreads();
  sink.list = la.lists + (size_t)blk * la.cap;
  sink.counter = &own[0];
  sink.overflow = &own[3];
}
__device__ __forceinline__ void block_list_end(const ListArgs& la, WaveRange& range, unsigned* own) {
  float lo = range.lo, hi = range.hi;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    lo = fminf(lo, __shfl_xor(lo, o));
    hi = fmaxf(hi, __shfl_xor(hi, o));
  }
  if ((threadIdx.x & (kWave - 1)) == 0 && lo <= hi) {
    atomicMin(&own[1], float_key(lo));
    atomicMax(&own[2], float_key(hi));
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    ListHead h;
    h.count = own[0];
    h.min_key = own[1];
    h.max_key = own[2];
    h.pad = own[3];
    la.heads[blockIdx.y * gridDim.x + blockIdx.x] = h;
  }
}

}  // namespace ecc
