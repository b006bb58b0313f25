// 2D sweep for gfx950: coefficient c(p) (Eq. 3 of the paper) + LDS histogram,
// one wavefront per column strip, marching down the rows.
//
// Layout.  A wave owns a strip of 62 output columns; its 64 lanes hold columns
// xs-1 .. xs+62 (one halo column each side), one float per lane per row, so a
// row is a single coalesced 256-byte load and the rows of the strip stream
// through registers (current row, next row, kPF rows in flight).  Nothing is
// staged in LDS: a vertex is loaded from HBM once per strip plus the 2/62 halo.
//
// Stencil on lane masks.  "q comes before p" is a strict "<" towards the four
// later neighbours (+x, and the three in the next row).  Those four compares
// give four 64-bit lane masks per row (one bit per column).  The four earlier
// neighbours need no compare: [q before p] = not [p before q], and
// [p before q] is the mask the row above / the lane to the left produced for
// its later neighbour, so they are complements of shifted masks.  Vertices
// outside the grid read as +inf, which makes every bit that involves them
// come out right ("never before p") with no boundary masks.
//
// Coefficient from run starts.  The vertices before p cut the 8-ring around p
// into arcs; a diagonal joins its two edge neighbours only if all three come
// before p.  c(p) = 1 - (#arcs), and an arc starts at edge neighbour k when k
// comes before p but not both its clockwise predecessors:
//     start_k = r_k & ~(r_{k-1} & r_{k-2}),   c = 1 - sum_k start_k.
// Four start masks, a handful of scalar ops on 64 columns at a time.  Lanes
// with exactly one start have c = 0 (regular vertices: almost all of a smooth
// field) and never reach the histogram code.
#include "ecc_device.h"
#include "ecc_internal.h"

namespace ecc {

constexpr int kStripOut = 62;
constexpr int kPF = 4;  // rows prefetched ahead of the row being compared

__device__ __forceinline__ float lane_from_right(float v) {  // lane i <- lane i+1 (lane 63 <- 0)
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x130,
                                                               0xf, 0xf, true));
}
__device__ __forceinline__ float lane_from_left(float v) {  // lane i <- lane i-1 (lane 0 <- 0)
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x138,
                                                               0xf, 0xf, true));
}
__device__ __forceinline__ unsigned long long ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }
__device__ __forceinline__ bool lane_bit(unsigned long long m) {
  return __builtin_amdgcn_inverse_ballot_w64(m);
}

template <bool LEVELS, bool TLDS>
__device__ __forceinline__ void add_to_hist(float v, int c, int bins, float lo, float scale,
                                            const float* __restrict__ gtable, const float* ltable,
                                            int* lhist) {
  int b;
  if (LEVELS) {
    b = (v < (float)bins) ? (int)v : bins;
  } else if (TLDS) {
    b = bin_from_table(v, ltable, bins, lo, scale);
  } else {
    b = bin_from_table(v, gtable, bins, lo, scale);
  }
  if (b < bins) atomicAdd(&lhist[b], c);
}

// Rows ya..yb (all inside the grid) are streamed; row r is "current" for
// r = ya..y1-1 and produces output when r >= y0.  The masks of the row above
// the first current row start as all ones, which is exact for the grid's first
// row (no vertex above comes before p) and is overwritten by the warm-up row
// otherwise.
template <typename T, bool LEVELS, bool TLDS, bool EDGE>
__device__ __forceinline__ void sweep_strip(const T* __restrict__ g, int H, int W, int xs, int y0,
                                            int y1, int bins, float lo, float scale,
                                            const float* __restrict__ gtable, const float* ltable,
                                            int* lhist) {
  const int lane = threadIdx.x & (kWave - 1);
  const int x = xs + lane;
  const bool inb = !EDGE || (x >= 0 && x < W);
  const unsigned long long out_mask = ballot(lane >= 1 && lane <= kStripOut && x >= 0 && x < W);
  const int ya = max(y0 - 1, 0), yb = min(y1, H - 1);
  const unsigned xoff = EDGE ? (inb ? (unsigned)x : 0u) : (unsigned)lane;
  const T* base = EDGE ? g : g + xs;   // wave-uniform
  const T* rowp = base + (int64_t)ya * W;
  int r = ya;  // row rowp points at

  auto fetch = [&]() -> float {  // value of row r for this lane, then advance (clamped at yb)
    float v = (float)rowp[xoff];
    if (EDGE) v = inb ? v : INFINITY;
    const bool more = r < yb;  // wave-uniform
    rowp += more ? W : 0;
    r += more ? 1 : 0;
    return v;
  };

  float cur = fetch();
  float nxt = fetch();
  float pf[kPF];
#pragma unroll
  for (int k = 0; k < kPF; ++k) pf[k] = fetch();
  float curR = lane_from_right(cur);
  unsigned long long pN = ~0ull, pNE = ~0ull, pNW = ~0ull;

  auto step = [&](bool output, bool refill) {
    const float nxtL = lane_from_left(nxt);
    const float nxtR = lane_from_right(nxt);
    const unsigned long long PE = ballot(curR < cur);
    const unsigned long long PN = ballot(nxt < cur);
    const unsigned long long PNE = ballot(nxtR < cur);
    const unsigned long long PNW = ballot(nxtL < cur);
    if (output) {
      const unsigned long long sE = PE & ((pNW >> 1) | pN);
      const unsigned long long sN = PN & ~(PNE & PE);
      const unsigned long long sW = ~((PE << 1) | (PNW & PN));
      const unsigned long long sS = ((pNE | PE) << 1) & ~pN;
      const unsigned long long x1 = sE ^ sN, c1 = sE & sN, x2 = sW ^ sS, c2 = sW & sS;
      const unsigned long long one = (x1 ^ x2) & ~(c1 | c2);
      const unsigned long long nz = out_mask & ~one;
      if (lane_bit(nz)) {
        const int c = 1 - (int)lane_bit(sE) - (int)lane_bit(sN) - (int)lane_bit(sW) - (int)lane_bit(sS);
        add_to_hist<LEVELS, TLDS>(cur, c, bins, lo, scale, gtable, ltable, lhist);
      }
    }
    pN = PN;
    pNE = PNE;
    pNW = PNW;
    cur = nxt;
    curR = nxtR;
    nxt = pf[0];
#pragma unroll
    for (int k = 0; k + 1 < kPF; ++k) pf[k] = pf[k + 1];
    if (refill) pf[kPF - 1] = fetch();
  };

  int y = ya;
  if (ya < y0) {  // warm-up row: masks only
    step(false, true);
    ++y;
  }
  // steady state: current rows y .. y1-2 have a real next row
  for (; y + kPF <= y1 - 1; y += kPF) {
#pragma unroll
    for (int k = 0; k < kPF; ++k) step(true, true);
  }
  for (; y < y1 - 1; ++y) step(true, true);
  // last row of the segment: below it is either a real row or the outside
  if (y1 >= H) nxt = INFINITY;
  step(true, false);
}

// Work unit of a wave: (segment of rows) x (strip of columns) of one item;
// blockIdx.y is the item, the four waves of a block take adjacent strips.
template <typename T, bool LEVELS, bool TLDS>
__global__ __launch_bounds__(256) void sweep2d_kernel(
    const T* __restrict__ grid, int H, int W, int64_t N, int bins, int nstrip, int nseg, int rows_per_seg,
    const HardHeader* __restrict__ hdr, const float* __restrict__ table,
    unsigned long long* __restrict__ hist) {
  extern __shared__ int smem[];
  int* lhist = smem;
  float* ltable = reinterpret_cast<float*>(smem + bins);
  for (int b = threadIdx.x; b < bins; b += 256) {
    lhist[b] = 0;
    if (TLDS) ltable[b] = table[b];
  }
  __syncthreads();
  float lo = 0.f, scale = 0.f;
  if (!LEVELS) { lo = hdr->lo; scale = hdr->scale; }
  const T* g = grid + (int64_t)blockIdx.y * N;
  const int unit = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform
  if (unit < nstrip * nseg) {
    const int seg = unit / nstrip, strip = unit - seg * nstrip;
    const int xs = strip * kStripOut - 1;
    const int y0 = seg * rows_per_seg;
    const int y1 = min(y0 + rows_per_seg, H);
    const bool edge = (xs < 0) || (xs + kWave > W);
    if (edge)
      sweep_strip<T, LEVELS, TLDS, true>(g, H, W, xs, y0, y1, bins, lo, scale, table, ltable, lhist);
    else
      sweep_strip<T, LEVELS, TLDS, false>(g, H, W, xs, y0, y1, bins, lo, scale, table, ltable, lhist);
  }
  __syncthreads();
  unsigned long long* out = hist + (int64_t)blockIdx.y * bins;
  for (int b = threadIdx.x; b < bins; b += 256) {
    const int v = lhist[b];
    if (v != 0) atomicAdd(&out[b], (unsigned long long)(long long)v);
  }
}

template <typename T>
static void launch2d_t(const void* grid, const Shape& s, bool levels, int bins, const HardHeader* hdr,
                       const float* table, unsigned long long* hist, hipStream_t st) {
  const int H = (int)s.H, W = (int)s.W;
  const int nstrip = (W + kStripOut - 1) / kStripOut;
  // enough wave units to fill 256 CUs several times over, segments of >= 32 rows
  const int64_t target = 16384;
  int64_t nseg = (target + (int64_t)nstrip * s.batch - 1) / ((int64_t)nstrip * s.batch);
  const int64_t max_seg = (H + 31) / 32;
  if (nseg > max_seg) nseg = max_seg;
  if (nseg < 1) nseg = 1;
  const int rows_per_seg = (int)((H + nseg - 1) / nseg);
  nseg = (H + rows_per_seg - 1) / rows_per_seg;
  const int units = nstrip * (int)nseg;
  dim3 g((unsigned)((units + 3) / 4), (unsigned)s.batch);
  const bool tlds = !levels && (size_t)bins * 8 <= 48 * 1024;
  const size_t lds = (size_t)bins * (tlds ? 8 : 4);
  const T* p = static_cast<const T*>(grid);
#define ECC_GO(LV, TL)                                                                          \
  hipLaunchKernelGGL((sweep2d_kernel<T, LV, TL>), g, dim3(256), lds, st, p, H, W, s.N, bins, nstrip, \
                     (int)nseg, rows_per_seg, hdr, table, hist)
  if (levels) ECC_GO(true, false);
  else if (tlds) ECC_GO(false, true);
  else ECC_GO(false, false);
#undef ECC_GO
}

bool sweep2d_supported(const Shape& s) {
  return s.D == 1 && s.W >= 8 && s.W <= (1 << 30) && s.H <= (1 << 30);
}

void launch_sweep2d(const void* grid, const Shape& s, int dtype, bool levels, int bins,
                    const HardHeader* hdr, const float* table, unsigned long long* hist,
                    hipStream_t st) {
  switch (dtype) {
    case 0: launch2d_t<uint8_t>(grid, s, levels, bins, hdr, table, hist, st); break;
    case 1: launch2d_t<uint16_t>(grid, s, levels, bins, hdr, table, hist, st); break;
    default: launch2d_t<float>(grid, s, levels, bins, hdr, table, hist, st); break;
  }
}

}  // namespace ecc
