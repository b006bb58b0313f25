// 2D sweep for gfx950: coefficient c(p) (Eq. 3 of the paper) + LDS histogram,
// one wavefront per column strip, marching down the rows.
//
// Layout.  A wave owns a strip of 62 output columns; its 64 lanes hold columns
// xs-1 .. xs+62 (one halo column each side), one value per lane per row, so a
// row is a single coalesced 256-byte load and the rows of the strip stream
// through registers.  Nothing is staged in LDS: a vertex is read from HBM once
// per strip plus the 2/62 halo.
//
// Stencil, bit-sliced down the rows.  "q comes before p" is a strict "<"
// towards the four later neighbours (+x and the three in the next row): the
// sign bit of the float difference q - p (zeros are made +0 on load so that
// equal values give +0).  Each lane shifts those sign bits into four 32-bit
// words, one bit per row, so after 32 rows a lane holds the four later-
// neighbour relations of 32 vertices of its column.  The four earlier
// neighbours need no compare: [q before p] = not [p before q], which is the
// bit the row above (word shifted by one bit) or the lane to the left / right
// (word moved by one lane) produced for ITS later neighbour.  Vertices outside
// the grid read as +inf, which makes every bit that involves them come out
// right ("never before p") with no boundary cases.  All the Boolean work of
// the coefficient then runs on whole words: 32 vertices per lane per
// instruction.
//
// Coefficient from arc starts.  The vertices before p cut the 8-ring around p
// into arcs; a diagonal joins its two edge neighbours only if all three come
// before p.  c(p) = 1 - (#arcs), and an arc starts at edge neighbour k when k
// comes before p but not both its clockwise predecessors:
//     start_k = r_k & ~(r_{k-1} & r_{k-2}),   c = 1 - sum_k start_k.
// Vertices with exactly one start have c = 0 (regular vertices: almost all of
// a smooth field).  Only the others are walked bit by bit; their value is
// re-read (an L2 hit) and binned into the block's LDS histogram.
//
// A chunk is 32 consecutive rows r0 .. r0+31; the first row only supplies the
// "row above" bits, rows r0+1 .. r0+31 produce output, and the next chunk
// starts at r0+31.
#include "ecc_device.h"
#include "ecc_internal.h"

namespace ecc {

constexpr int kStripOut = 62;
constexpr int kPF = 8;  // rows in flight ahead of the row being compared

__device__ __forceinline__ float lane_from_right(float v) {  // lane i <- lane i+1 (lane 63 <- 0)
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x130,
                                                               0xf, 0xf, true));
}
__device__ __forceinline__ float lane_from_left(float v) {  // lane i <- lane i-1 (lane 0 <- 0)
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x138,
                                                               0xf, 0xf, true));
}
__device__ __forceinline__ unsigned word_from_right(unsigned v) {
  return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x130, 0xf, 0xf, true);
}
__device__ __forceinline__ unsigned word_from_left(unsigned v) {
  return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x138, 0xf, 0xf, true);
}
__device__ __forceinline__ unsigned long long ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }

// w <- (w << 1) | [q < p]
__device__ __forceinline__ unsigned push_lt(unsigned w, float q, float p) {
  return __builtin_amdgcn_alignbit(w, __float_as_uint(q - p), 31);
}
__device__ __forceinline__ unsigned push_sign(unsigned w, float d) {
  return __builtin_amdgcn_alignbit(w, __float_as_uint(d), 31);
}

// The three differences whose left operand comes from a neighbouring lane, as
// DPP-modified subtractions (no separate lane move):
//   dE[i] = cur[i+1] - cur[i], dNE[i] = nxt[i+1] - cur[i], dNW[i] = nxt[i-1] - cur[i].
// Lanes without a source lane read 0; their bits are never used (halo lanes).
// The leading s_nop covers the two wait states a DPP read needs after a VALU
// write of its source register.
__device__ __forceinline__ void side_differences(float cur, float nxt, float& dE, float& dNE,
                                                 float& dNW) {
  asm("s_nop 1\n\t"
      "v_sub_f32_dpp %0, %3, %3 wave_shl:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_sub_f32_dpp %1, %4, %3 wave_shl:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_sub_f32_dpp %2, %4, %3 wave_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:1"
      : "=&v"(dE), "=&v"(dNE), "=&v"(dNW)
      : "v"(cur), "v"(nxt));
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

// Raw buffer loads: wave-uniform resource + scalar row offset + constant lane
// offset, so addressing costs no vector instruction, and reads past the end of
// the item return 0 instead of faulting.
template <typename T> struct RowLoad;
template <> struct RowLoad<float> {
  static __device__ __forceinline__ float get(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
  }
};
template <> struct RowLoad<uint16_t> {
  static __device__ __forceinline__ uint16_t get(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
    return (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0);
  }
};
template <> struct RowLoad<uint8_t> {
  static __device__ __forceinline__ uint8_t get(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
    return (uint8_t)__builtin_amdgcn_raw_buffer_load_b8(r, voff, soff, 0);
  }
};

// One strip, output rows y0 .. y1-1 (y0 < y1 <= H).
//
// Rows are "current" one after the other; a step pushes the four later-
// neighbour bits of the current row into the words.  A chunk is up to 32
// steps; the bits of the row above a chunk's first row are bit 0 of the
// previous chunk's words (one warm-up step on row y0-1 provides them for the
// first chunk; above the grid they are all ones, i.e. "never before p").
template <typename T, bool LEVELS, bool TLDS, bool EDGE>
__device__ __forceinline__ void sweep_strip(const T* __restrict__ g, int64_t item_elems, int H, int W,
                                            int xs, int y0, int y1, int bins, float lo, float scale,
                                            const float* __restrict__ gtable, const float* ltable,
                                            int* lhist) {
  const int lane = threadIdx.x & (kWave - 1);
  const int x = xs + lane;
  const bool inb = !EDGE || (x >= 0 && x < W);
  const bool out_lane = lane >= 1 && lane <= kStripOut && x >= 0 && x < W;
  const unsigned voff = (EDGE ? (inb ? (unsigned)x : 0u) : (unsigned)lane) * (unsigned)sizeof(T);

  // resource starts at the first streamed row (and at column xs for interior strips)
  const int ya = max(y0 - 1, 0);
  const int64_t first = (int64_t)ya * W + (EDGE ? 0 : xs);
  const int64_t left = (item_elems - first) * (int64_t)sizeof(T);
  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<T*>(g + first), 0, (int)(left > 0x7fffffff ? 0x7fffffff : left), 0x00020000);
  const unsigned row_bytes = (unsigned)W * (unsigned)sizeof(T);
  unsigned soff = 0;  // byte offset of the next row to load
  auto load_raw = [&]() -> T {
    const T v = RowLoad<T>::get(rsrc, voff, soff);
    soff += row_bytes;
    return v;
  };
  auto fix = [&](T raw) -> float {
    float v = (float)raw;
    if (sizeof(T) == 4) v += 0.0f;  // -0 -> +0 so that equal values differ by +0
    if (EDGE) v = inb ? v : INFINITY;
    return v;
  };

  float cur = fix(load_raw());
  float nxt = fix(load_raw());
  T pf[kPF];
#pragma unroll
  for (int k = 0; k < kPF; ++k) pf[k] = load_raw();

  unsigned wE = 0, wN = 0, wNE = 0, wNW = 0;
  auto step = [&]() {
    float dE, dNE, dNW;
    side_differences(cur, nxt, dE, dNE, dNW);
    wE = push_sign(wE, dE);
    wN = push_lt(wN, nxt, cur);
    wNE = push_sign(wNE, dNE);
    wNW = push_sign(wNW, dNW);
    cur = nxt;
    nxt = fix(pf[0]);
#pragma unroll
    for (int q = 0; q + 1 < kPF; ++q) pf[q] = pf[q + 1];
    pf[kPF - 1] = load_raw();
  };

  unsigned oN = 1, oNE = 1, oNW = 1;  // bit 0: the row above the first output row
  if (y0 > 0) {
    step();  // warm-up on row y0-1
    oN = wN;
    oNE = wNE;
    oNW = wNW;
  }

  for (int r = y0; r < y1; r += 32) {
    const int n = min(32, y1 - r);
    wE = wN = wNE = wNW = 0;
    int k = 0;
    for (; k + kPF <= n; k += kPF) {
#pragma unroll
      for (int q = 0; q < kPF; ++q) step();
    }
    for (; k < n; ++k) step();
    if (r + n >= H) {  // the grid's last row has nothing below it
      wN &= ~1u;
      wNE &= ~1u;
      wNW &= ~1u;
    }
    const int pad = 32 - n;  // row r+j sits at bit 31-j
    const unsigned E = wE << pad, N = wN << pad, NE = wNE << pad, NW = wNW << pad;

    // earlier neighbours: the row above is one bit up (bit 31 from the previous
    // chunk), the side columns are the neighbouring lanes
    const unsigned pN = __builtin_amdgcn_alignbit(oN, N, 1);
    const unsigned pNE = __builtin_amdgcn_alignbit(oNE, NE, 1);
    const unsigned pNW = __builtin_amdgcn_alignbit(oNW, NW, 1);
    oN = wN;
    oNE = wNE;
    oNW = wNW;
    const unsigned sE = E & (word_from_right(pNW) | pN);
    const unsigned sN = N & ~(NE & E);
    const unsigned sW = ~(word_from_left(E) | (NW & N));
    const unsigned sS = word_from_left(pNE | E) & ~pN;
    const unsigned x1 = sE ^ sN, c1 = sE & sN, x2 = sW ^ sS, c2 = sW & sS;
    const unsigned one = (x1 ^ x2) & ~(c1 | c2);
    const unsigned rows = 0xffffffffu << pad;
    unsigned nz = out_lane ? (~one & rows) : 0u;
    while (ballot(nz != 0)) {
      if (nz != 0) {
        const int b = 31 - __clz(nz);
        nz &= ~(1u << b);
        const int c = 1 - (int)((sE >> b) & 1u) - (int)((sN >> b) & 1u) - (int)((sW >> b) & 1u) -
                      (int)((sS >> b) & 1u);
        const int rr = r + 31 - b - ya;  // row relative to the resource
        const float v = (float)RowLoad<T>::get(rsrc, voff + (unsigned)rr * row_bytes, 0);  // L2 hit
        add_to_hist<LEVELS, TLDS>(v, c, bins, lo, scale, gtable, ltable, lhist);
      }
    }
  }
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
      sweep_strip<T, LEVELS, TLDS, true>(g, N, H, W, xs, y0, y1, bins, lo, scale, table, ltable, lhist);
    else
      sweep_strip<T, LEVELS, TLDS, false>(g, N, H, W, xs, y0, y1, bins, lo, scale, table, ltable, lhist);
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
  // whole chunks of 32 rows per segment; segment + prefetch must stay below 2^31 bytes
  int64_t rows = ((H + nseg - 1) / nseg + 31) / 32 * 32;
  const int64_t row_bytes = (int64_t)W * (int64_t)sizeof(T);
  const int64_t cap = ((((int64_t)1 << 31) / row_bytes - 16) / 32) * 32;
  if (rows > cap) rows = cap;
  const int rows_per_seg = (int)rows;
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
  return s.D == 1 && s.W >= 8 && s.W <= (1 << 22) && s.H <= (1 << 30);
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
