// 2D sweep for gfx950 (device templates shared by the hard and the soft kernels): coefficient c(p) (Eq. 3 of the paper) + LDS histogram,
// one wavefront per column strip, marching down the rows.
//
// Layout.  A wave owns a strip of 248 output columns; its 64 lanes hold four
// consecutive columns each, 256 columns starting four before the first output
// column, so lanes 0 and 63 are halo lanes and a row of the strip is a single
// 16-byte-aligned 1 KiB load (buffer_load_dwordx4).  The rows of the strip
// stream through registers; nothing is staged in LDS, and a vertex is read
// from HBM once per strip plus the 8/248 halo.
//
// Stencil, bit-sliced down the rows.  "q comes before p" is a strict "<"
// towards the four later neighbours (+x and the three in the next row): the
// sign bit of the float difference q - p (zeros are made +0 on load so that
// equal values give +0).  Each lane shifts those sign bits into four 32-bit
// words per column, one bit per row, so after 32 rows a word holds one
// later-neighbour relation of 32 vertices of a column.  The four earlier
// neighbours need no compare: [q before p] = not [p before q], which is the
// bit the row above (word shifted by one bit) or the column to the left /
// right (the neighbouring word, one lane over at a lane boundary) produced for
// ITS later neighbour.  Vertices outside the grid read as +inf, which makes
// every bit that involves them come out right ("never before p") with no
// boundary cases.  All Boolean work then runs on whole words: 32 vertices per
// lane per instruction.
//
// Coefficient from arc starts.  The vertices before p cut the 8-ring around p
// into arcs; a diagonal joins its two edge neighbours only if all three come
// before p.  c(p) = 1 - (#arcs), and an arc starts at edge neighbour k when k
// comes before p but not both its clockwise predecessors:
//     start_k = r_k & ~(r_{k-1} & r_{k-2}),   c = 1 - sum_k start_k.
// Vertices with exactly one start have c = 0 (regular vertices: almost all of
// a smooth field).  Only the others are walked bit by bit and binned into the
// block's LDS histogram; their values come from a small LDS ring into which the
// wave copies each row as it becomes current (re-reading them from memory
// would miss the L2 once per critical vertex, a 128-byte line for 4 bytes).
#pragma once
#include <algorithm>

#include "ecc_device.h"
#include "ecc_internal.h"

namespace ecc {

constexpr int kNC = 4;                       // columns per lane
constexpr int kStripOut = (kWave - 2) * kNC;  // 248 output columns per wave
constexpr int kPF = 4;                        // rows in flight ahead of the row being compared
constexpr int kChunkRows = 8;                 // rows per chunk = rows of the LDS value ring

__device__ __forceinline__ unsigned word_from_right(unsigned v) {  // lane i <- lane i+1
  return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x130, 0xf, 0xf, true);
}
__device__ __forceinline__ unsigned word_from_left(unsigned v) {  // lane i <- lane i-1
  return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x138, 0xf, 0xf, true);
}
__device__ __forceinline__ unsigned long long ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }

// w <- (w << 1) | signbit(d)
__device__ __forceinline__ unsigned push_sign(unsigned w, float d) {
  return __builtin_amdgcn_alignbit(w, __float_as_uint(d), 31);
}

// The three differences of a row step whose left operand lives in a
// neighbouring lane, as DPP-modified subtractions (no separate lane move):
//   dE  = cur_first[i+1] - cur_last[i]     (+x neighbour of a lane's last column)
//   dNE = nxt_first[i+1] - cur_last[i]
//   dNW = nxt_last[i-1]  - cur_first[i]
// Lanes without a source lane read 0; their bits belong to halo lanes and are
// never used.  The s_nop covers the two wait states a DPP read needs after a
// VALU write of its source register.
__device__ __forceinline__ void lane_edge_differences(float cur_first, float cur_last, float nxt_first,
                                                      float nxt_last, float& dE, float& dNE, float& dNW) {
  asm("s_nop 1\n\t"
      "v_sub_f32_dpp %0, %3, %4 wave_shl:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_sub_f32_dpp %1, %5, %4 wave_shl:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_sub_f32_dpp %2, %6, %3 wave_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:1"
      : "=&v"(dE), "=&v"(dNE), "=&v"(dNW)
      : "v"(cur_first), "v"(cur_last), "v"(nxt_first), "v"(nxt_last));
}

// Raw buffer loads: wave-uniform resource + scalar row offset + constant lane
// offset, so addressing costs no vector instruction, and reads past the end of
// the item return 0 instead of faulting.
template <typename T> struct Raw4;  // four consecutive elements of a row
template <> struct Raw4<float> {
  typedef __attribute__((ext_vector_type(4))) unsigned vec;
  vec v;
  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
    v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
  }
  __device__ __forceinline__ float get(int e) const { return __uint_as_float(v[e]); }
};
// two-byte elements: one 8-byte load, widened to float32 element by element
template <typename T> struct Raw4x16 {
  typedef __attribute__((ext_vector_type(2))) unsigned vec;
  vec v;
  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
    v = __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
  }
  __device__ __forceinline__ float get(int e) const { return widen16<T>(v[e >> 1] >> (16 * (e & 1))); }
};
template <> struct Raw4<uint16_t> : Raw4x16<uint16_t> {};
template <> struct Raw4<int16_t> : Raw4x16<int16_t> {};
template <> struct Raw4<F16> : Raw4x16<F16> {};
template <> struct Raw4<Bf16> : Raw4x16<Bf16> {};
template <> struct Raw4<uint8_t> {
  unsigned v;
  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
    v = __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0);
  }
  __device__ __forceinline__ float get(int e) const { return (float)((v >> (8 * e)) & 0xffu); }
};
template <typename T> struct Raw1;  // one element
template <> struct Raw1<float> {
  static __device__ __forceinline__ float get(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
  }
};
template <typename T> struct Raw1x16 {
  static __device__ __forceinline__ float get(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
    return widen16<T>((unsigned)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0));
  }
};
template <> struct Raw1<uint16_t> : Raw1x16<uint16_t> {};
template <> struct Raw1<int16_t> : Raw1x16<int16_t> {};
template <> struct Raw1<F16> : Raw1x16<F16> {};
template <> struct Raw1<Bf16> : Raw1x16<Bf16> {};
template <> struct Raw1<uint8_t> {
  static __device__ __forceinline__ float get(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
    return (float)(uint8_t)__builtin_amdgcn_raw_buffer_load_b8(r, voff, soff, 0);
  }
};

// A row of the strip for one lane: four values.  Interior strips load them
// with one aligned 4-element load; edge strips (some column outside the grid)
// load element by element with the column clamped, and patch +inf in.
template <typename T, bool EDGE> struct RowRegs;
template <typename T> struct RowRegs<T, false> {
  Raw4<T> raw;
  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, const unsigned (&)[kNC], unsigned voff4,
                                       unsigned soff) {
    raw.load(r, voff4, soff);
  }
  __device__ __forceinline__ float raw_value(int e) const { return raw.get(e); }
};
template <typename T> struct RowRegs<T, true> {
  float f[kNC];
  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, const unsigned (&voff)[kNC], unsigned,
                                       unsigned soff) {
#pragma unroll
    for (int e = 0; e < kNC; ++e) f[e] = Raw1<T>::get(r, voff[e], soff);
  }
  __device__ __forceinline__ float raw_value(int e) const { return f[e]; }
};

// One strip: lanes hold columns c0 + 4*lane + e; output rows y0 .. y1-1
// (y0 < y1 <= H).
//
// Rows are "current" one after the other; a step pushes the four later-
// neighbour bits of every column of the current row into the words and copies
// the row into the wave's LDS ring.  A chunk is up to kChunkRows steps; the bits of the row above a chunk's first row are bit 0
// of the previous chunk's words (one warm-up step on row y0-1 provides them
// for the first chunk; above the grid they are all ones, i.e. "never before
// p" once complemented).
//
// Tilt: the field swept is Y(p) = X(p) + t(p) with t = fl(fl(a_x x) + fl(a_y y)),
// every operation a float32 one in this order (directional curves; NoTilt: Y = X).
//
// Lanes lane_lo .. lane_hi put out their vertices; the others are halo lanes.  A strip inside the
// grid has one halo lane on each side (1 .. 62).  A strip that starts at the grid's first column
// (open_left) or ends at its last one (open_right) has no neighbour lane there: the vertices beyond
// the grid are "never before p" (always, for the top-cell order), and the words that would come
// from the missing lane are set to say so once per chunk.
// OPEN: the strip may be such a first / last strip (compiled apart, so that the strips inside the
// grid carry none of this).
template <typename T, typename Sink, bool EDGE, typename Tilt, bool OPEN = false>
__device__ __forceinline__ void sweep_strip(const T* __restrict__ g, int64_t item_elems, int H, int W,
                                            int c0, int y0, int y1, WaveQueue<Sink>& queue,
                                            float* ring /* [kChunkRows][64][kNC] */, WaveRange& range,
                                            const Tilt& tilt, int lane_lo_ = 1, int lane_hi_ = kWave - 2,
                                            bool open_left_ = false, bool open_right_ = false) {
  const int lane_lo = OPEN ? lane_lo_ : 1, lane_hi = OPEN ? lane_hi_ : kWave - 2;
  const bool open_left = OPEN && open_left_, open_right = OPEN && open_right_;
  const int lane = threadIdx.x & (kWave - 1);
  bool ok[kNC];         // column inside the grid
  unsigned voff[kNC];   // byte offset of the column inside a row (clamped into the row)
#pragma unroll
  for (int e = 0; e < kNC; ++e) {
    const int x = c0 + kNC * lane + e;
    ok[e] = x >= 0 && x < W;
    voff[e] = (unsigned)min(max(x, 0), W - 1) * (unsigned)sizeof(T);
  }
  const bool out_lane = lane >= lane_lo && lane <= lane_hi;
  // what a relation towards a vertex beyond the grid reads: never before p, or always (top-cell order)
  constexpr unsigned kBeyond = Tilt::kTop ? 0xffffffffu : 0u;
  const bool first_lane = open_left && lane == 0, last_lane = open_right && lane == kWave - 1;
  const unsigned voff4 = (unsigned)(kNC * lane) * (unsigned)sizeof(T);  // interior strips: from column c0

  // the resource starts at the first streamed row (and at column c0 for interior strips)
  const int ya = max(y0 - 1, 0);
  const int64_t first = (int64_t)ya * W + (EDGE ? 0 : c0);
  const int64_t left = (item_elems - first) * (int64_t)sizeof(T);
  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<T*>(g + first), 0, (int)(left > 0x7fffffff ? 0x7fffffff : left), 0x00020000);
  const unsigned row_bytes = (unsigned)W * (unsigned)sizeof(T);
  unsigned soff = 0;  // byte offset of the next row to load
  // The last row this segment needs is y1 (the row below its last output row), or
  // the grid's last row; the rows the pipeline would fetch beyond it are not read
  // from memory again: the offset stays on that row (a cache hit).
  const unsigned soff_last = (unsigned)(min(y1, H - 1) - ya) * row_bytes;
  auto next_row = [&]() { soff = min(soff + row_bytes, soff_last); };

  typedef RowRegs<T, EDGE> Row;
  // value of column e of a loaded row, which is row y of the grid
  float lx[kNC];  // the column's share of the tilt (zero made +0: equal values must differ by +0)
#pragma unroll
  for (int e = 0; e < kNC; ++e)
    lx[e] = Tilt::kOn ? add_rn(mul_rn(tilt.ax, (float)(c0 + kNC * lane + e)), 0.0f) : 0.0f;
  // (zeros come out as +0 in every mode, so that equal values differ by +0; a column
  // outside the grid reads as "never before p": +inf, or -inf where the order is reversed)
  auto value_at = [&](const Row& r, int e, int y) -> float {
    float f = r.raw_value(e);
    if (Tilt::kNeg) {
      // 0 - f, zeros coming out as +0.  Kept opaque: left to itself the compiler replaces later
      // uses of it by a negated source operand, which turns +0 into -0 in a difference.
      f = 0.0f - f;
      asm volatile("" : "+v"(f));
    }
    else if (Tilt::kOn) f = add_rn(f, add_rn(lx[e], mul_rn(tilt.ay, (float)y)));
    else if (HasNegZero<T>::value) f += 0.0f;
    if (EDGE) f = ok[e] ? f : (Tilt::kTop ? -INFINITY : INFINITY);
    return f;
  };
  auto original = [](float f) -> float { return Tilt::kNeg ? -f : f; };  // the value that is binned
  Row pf[kPF];
  float cur[kNC], nxt[kNC];
  int yn = ya + 2;  // row of the grid that becomes nxt at the next step
  {
    Row a, b;
    a.load(rsrc, voff, voff4, soff);
    next_row();
    b.load(rsrc, voff, voff4, soff);
    next_row();
#pragma unroll
    for (int k = 0; k < kPF; ++k) {
      pf[k].load(rsrc, voff, voff4, soff);
      next_row();
    }
#pragma unroll
    for (int e = 0; e < kNC; ++e) {
      cur[e] = value_at(a, e, ya);
      nxt[e] = value_at(b, e, ya + 1);
    }
  }

  // Range (single-pass mode).  The smallest vertex of the grid is critical
  // (c = 1) and so is the largest one unless it lies on the grid's boundary (an
  // interior vertex with all eight neighbours before it has c = 1 as well), so
  // the range is taken over the critical vertices and the boundary vertices:
  // EDGE strips look at all their values, interior strips at the grid's first
  // and last row here and at the critical vertices where they are pushed.
  if (Sink::kTrackRange && !EDGE) {
    if (y0 == 0) {
      Row t;
      t.load(rsrc, voff, voff4, 0);
#pragma unroll
      for (int e = 0; e < kNC; ++e) range.add(original(value_at(t, e, 0)));
    }
    if (y1 >= H) {
      Row t;
      t.load(rsrc, voff, voff4, (unsigned)(H - 1 - ya) * row_bytes);
#pragma unroll
      for (int e = 0; e < kNC; ++e) range.add(original(value_at(t, e, H - 1)));
    }
  }

  unsigned wE[kNC], wN[kNC], wNE[kNC], wNW[kNC];
#pragma unroll
  for (int e = 0; e < kNC; ++e) wE[e] = wN[e] = wNE[e] = wNW[e] = 0;

  int slot = 0;  // ring row of the current row
  auto step = [&]() {
    *reinterpret_cast<float4*>(ring + (slot * kWave + lane) * kNC) =
        make_float4(cur[0], cur[1], cur[2], cur[3]);
    ++slot;
    if (Sink::kTrackRange && EDGE) {
#pragma unroll
      for (int e = 0; e < kNC; ++e) range.add_if(original(cur[e]), ok[e]);
    }
    if (Sink::kTrackRange && !EDGE) {  // the grid's first / last column (wave-uniform conditions)
      if (open_left) range.add_if(original(cur[0]), first_lane);
      if (open_right) range.add_if(original(cur[kNC - 1]), last_lane);
    }
    float dE, dNE, dNW;
    lane_edge_differences(cur[0], cur[kNC - 1], nxt[0], nxt[kNC - 1], dE, dNE, dNW);
#pragma unroll
    for (int e = 0; e < kNC; ++e) {
      wE[e] = push_sign(wE[e], e + 1 < kNC ? cur[e + 1] - cur[e] : dE);
      wN[e] = push_sign(wN[e], nxt[e] - cur[e]);
      wNE[e] = push_sign(wNE[e], e + 1 < kNC ? nxt[e + 1] - cur[e] : dNE);
      wNW[e] = push_sign(wNW[e], e > 0 ? nxt[e - 1] - cur[e] : dNW);
    }
#pragma unroll
    for (int e = 0; e < kNC; ++e) {
      cur[e] = nxt[e];
      nxt[e] = value_at(pf[0], e, yn);
    }
    ++yn;
#pragma unroll
    for (int q = 0; q + 1 < kPF; ++q) pf[q] = pf[q + 1];
    pf[kPF - 1].load(rsrc, voff, voff4, soff);
    next_row();
  };

  // relations of the strip's outermost columns towards vertices beyond the grid (the lane that would
  // supply the other operand does not exist: the differences pushed there mean nothing)
  auto beyond_the_grid = [&]() {
    if (open_left) wNW[0] = first_lane ? kBeyond : wNW[0];
    if (open_right) {
      wE[kNC - 1] = last_lane ? kBeyond : wE[kNC - 1];
      wNE[kNC - 1] = last_lane ? kBeyond : wNE[kNC - 1];
    }
  };
  unsigned oN[kNC], oNE[kNC], oNW[kNC];  // bit 0: the row above the first output row
#pragma unroll
  for (int e = 0; e < kNC; ++e) oN[e] = oNE[e] = oNW[e] = Tilt::kTop ? 0 : 1;  // (reversed order: always before p)
  if (y0 > 0) {
    step();  // warm-up on row y0-1
    beyond_the_grid();
#pragma unroll
    for (int e = 0; e < kNC; ++e) {
      oN[e] = wN[e];
      oNE[e] = wNE[e];
      oNW[e] = wNW[e];
    }
  }

  for (int r = y0; r < y1; r += kChunkRows) {
    const int n = min(kChunkRows, y1 - r);
#pragma unroll
    for (int e = 0; e < kNC; ++e) wE[e] = wN[e] = wNE[e] = wNW[e] = 0;
    slot = 0;
    int k = 0;
    for (; k + kPF <= n; k += kPF) {
#pragma unroll
      for (int q = 0; q < kPF; ++q) step();
    }
    for (; k < n; ++k) step();
    beyond_the_grid();
    if constexpr (Sink::kZeroFill) {  // the sink's per-vertex output is 0 except at critical vertices
      for (int j = 0; j < n; ++j) queue.sink.template zero_row<EDGE>(r + j, c0 + kNC * lane, ok, out_lane);
    }
    const bool bottom = r + n >= H;  // the grid's last row has nothing below it
    const int pad = 32 - n;          // row r+j sits at bit 31-j
    const unsigned rows = 0xffffffffu << pad;

    unsigned E[kNC], N[kNC], NE[kNC], NW[kNC], pN[kNC], pNE[kNC], pNW[kNC];
#pragma unroll
    for (int e = 0; e < kNC; ++e) {
      if (bottom) {
        if (Tilt::kTop) {  // reversed order: what lies outside the grid comes before p
          wN[e] |= 1u;
          wNE[e] |= 1u;
          wNW[e] |= 1u;
        } else {
          wN[e] &= ~1u;
          wNE[e] &= ~1u;
          wNW[e] &= ~1u;
        }
      }
      E[e] = wE[e] << pad;
      N[e] = wN[e] << pad;
      NE[e] = wNE[e] << pad;
      NW[e] = wNW[e] << pad;
      // the row above is one bit up (bit 31 from the previous chunk)
      pN[e] = __builtin_amdgcn_alignbit(oN[e], N[e], 1);
      pNE[e] = __builtin_amdgcn_alignbit(oNE[e], NE[e], 1);
      pNW[e] = __builtin_amdgcn_alignbit(oNW[e], NW[e], 1);
      oN[e] = wN[e];
      oNE[e] = wNE[e];
      oNW[e] = wNW[e];
    }
    // words of the columns just left / right of this lane's four
    const unsigned E_left = word_from_left(E[kNC - 1]);
    const unsigned pNEE_left = word_from_left(pNE[kNC - 1] | E[kNC - 1]);
    unsigned pNW_right = word_from_right(pNW[0]);
    // [p before its neighbour] towards a neighbour beyond the grid, where no lane supplies the word
    unsigned E_left_ = E_left, pNEE_left_ = pNEE_left;
    if (open_left) {
      E_left_ = first_lane ? ~kBeyond : E_left;
      pNEE_left_ = first_lane ? ~kBeyond : pNEE_left;
    }
    if (open_right) pNW_right = last_lane ? ~kBeyond : pNW_right;
    // A chunk uses the top kChunkRows (8) bits of a word, so the four columns of a
    // lane are packed into one word (column e in byte 3-e) and walked in one loop.
    static_assert(kChunkRows * kNC <= 32, "four columns of a chunk must fit one word");
    unsigned pE = 0, pNn = 0, pW = 0, pS = 0, nz = 0;
#pragma unroll
    for (int e = 0; e < kNC; ++e) {
      const unsigned El = e > 0 ? E[e - 1] : E_left_;                             // [p before its -x neighbour]
      const unsigned pNEEl = e > 0 ? (pNE[e - 1] | E[e - 1]) : pNEE_left_;        // SW or W relation, complemented
      const unsigned pNWr = e + 1 < kNC ? pNW[e + 1] : pNW_right;                 // SE relation, complemented
      const unsigned sE = E[e] & (pNWr | pN[e]);
      const unsigned sN = N[e] & ~(NE[e] & E[e]);
      const unsigned sW = ~(El | (NW[e] & N[e]));
      const unsigned sS = pNEEl & ~pN[e];
      const unsigned x1 = sE ^ sN, c1 = sE & sN, x2 = sW ^ sS, c2 = sW & sS;
      const unsigned one = (x1 ^ x2) & ~(c1 | c2);
      const unsigned crit = ok[e] ? (~one & rows) : 0u;
      const unsigned top = 0xff000000u;
      pE |= (sE & top) >> (8 * e);
      pNn |= (sN & top) >> (8 * e);
      pW |= (sW & top) >> (8 * e);
      pS |= (sS & top) >> (8 * e);
      nz |= (crit & top) >> (8 * e);
    }
    if (!out_lane) nz = 0u;
    while (ballot(nz != 0)) {
      const bool active = nz != 0;
      const int b = active ? 31 - __clz(nz) : 0;
      nz &= ~(1u << b);
      const int c = 1 - (int)((pE >> b) & 1u) - (int)((pNn >> b) & 1u) - (int)((pW >> b) & 1u) -
                    (int)((pS >> b) & 1u);
      const int pos = 31 - b;  // column pos / 8, row pos % 8 of the chunk
      const float v = original(ring[((pos & 7) * kWave + lane) * kNC + (pos >> 3)]);
      if (Sink::kTrackRange && !EDGE) range.add_if(v, active);
      queue.push(active, v, c, c0 + kNC * lane + (pos >> 3), r + (pos & 7));
    }
  }
  queue.flush();
}

// Work unit of a wave: (segment of rows) x (strip of columns) of one item;
// blockIdx.y is the item, the four waves of a block take adjacent strips.
template <typename T, typename Sink, typename Tilt>
__device__ __forceinline__ void sweep2d_wave(const T* __restrict__ g, int H, int W, int64_t N, int nstrip,
                                             int nseg, int rows_per_seg, WaveQueue<Sink>& queue, float* ring,
                                             WaveRange& range, const Tilt& tilt) {
  const int unit = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform
  if (unit < nstrip * nseg) {
    const int seg = unit / nstrip, strip = unit - seg * nstrip;
    const int y0 = seg * rows_per_seg;
    const int y1 = min(y0 + rows_per_seg, H);
    // Strip s puts out the columns [248 s, 248 s + 248).  One aligned 4-element load per lane and row
    // needs all 256 columns of the wave inside the grid and 4-element alignment of the rows; then
    // the strip inside the grid starts four columns early (a halo lane on each side), the first
    // strip starts at column 0 (its first lane puts out, two halo lanes at the end) and the last
    // strip ends at column W - 1 (its last lane puts out, the lanes before its first column are halo).
    const bool wide = (W % kNC == 0) && W >= kNC * kWave &&
                      ((reinterpret_cast<uintptr_t>(g) & (kNC * sizeof(T) - 1)) == 0);
    if (wide) {
      int c0 = strip * kStripOut - kNC, lo = 1, hi = kWave - 2;
      const bool left = strip == 0, right = strip == nstrip - 1;  // (W >= 256: at least two strips)
      if (left) {
        c0 = 0;
        lo = 0;
        hi = kWave - 3;
      }
      if (right) {
        c0 = W - kNC * kWave;
        lo = (strip * kStripOut - c0) / kNC;
        hi = kWave - 1;
      }
      if (left || right)
        sweep_strip<T, Sink, false, Tilt, true>(g, N, H, W, c0, y0, y1, queue, ring, range, tilt, lo, hi, left, right);
      else
        sweep_strip<T, Sink, false>(g, N, H, W, c0, y0, y1, queue, ring, range, tilt);
    } else {
      sweep_strip<T, Sink, true>(g, N, H, W, strip * kStripOut - kNC, y0, y1, queue, ring, range, tilt);
    }
  }
}

struct Plan2d {
  int nstrip, nseg, rows_per_seg;
  dim3 grid;
};
// sigmoid_sinks: the plan of the soft path, whose sinks do their work wave by wave and want
// many short segments; the hard path's sweeps are measured best as below.
template <typename T>
static Plan2d plan2d(const Shape& s, bool sigmoid_sinks = false) {
  Plan2d p;
  const int H = (int)s.H, W = (int)s.W;
  p.nstrip = (W + kStripOut - 1) / kStripOut;
  const int64_t tubes = (int64_t)p.nstrip * s.batch;
  int64_t nseg;
  if (sigmoid_sinks) {
    // enough wave units to fill 256 CUs several times over, segments of >= 16 rows (24 when
    // that still leaves two rounds of waves: a segment reads five rows more than it puts out)
    nseg = (32768 + tubes - 1) / tubes;
    const int64_t max_seg = tubes * ((H + 23) / 24) >= 8192 ? (H + 23) / 24 : (H + 15) / 16;
    if (nseg > max_seg) nseg = max_seg;
  } else if (tubes * ((H + 15) / 16) <= 1024) {
    // at most one wave per SIMD even with the shortest segments: the call is as long as one
    // wave's march, so the segments are as short as they come
    nseg = (H + 15) / 16;
  } else {
    // Measured (rows per segment against time): a batch of 16 x 4096^2 is flat from 24 to 64
    // rows and loses beyond 96; one 4096^2 image gains 30 % from 24 -> 64, one 2048^2 image
    // 20 % from 16 -> 32, batches of 256^2 ... 512^2 images 25-30 % from 16 -> 32 ... 64.  Aim
    // at about 1536 waves, within 32 ... 64 rows per segment.
    const int64_t want = std::max<int64_t>(1, 1536 / tubes);
    int64_t rows = (H + want - 1) / want;
    rows = (rows + kChunkRows - 1) / kChunkRows * kChunkRows;
    // plenty of tubes (a large batch of small images): up to 128 rows, but two segments per image at least
    // (1024 x 224^2: 0.112 -> 0.085 ms with 2 x 112 rows; 2048 x 128^2 loses 17 % with one segment of 128)
    int64_t longest = 64;
    if (tubes >= 1024) longest = std::max<int64_t>(64, std::min<int64_t>(128, ((H + 1) / 2 + kChunkRows - 1) / kChunkRows * kChunkRows));
    rows = rows < 32 ? 32 : (rows > longest ? longest : rows);
    nseg = (H + rows - 1) / rows;
  }
  if (nseg < 1) nseg = 1;
  // whole chunks per segment; segment + prefetch must stay below 2^31 bytes
  int64_t rows = (H + nseg - 1) / nseg;
  const int64_t gran = kChunkRows;
  rows = (rows + gran - 1) / gran * gran;
  const int64_t row_bytes = (int64_t)W * (int64_t)sizeof(T);
  const int64_t cap = ((((int64_t)1 << 31) / row_bytes - 16) / kChunkRows) * kChunkRows;
  if (rows > cap) rows = cap;
  p.rows_per_seg = (int)rows;
  p.nseg = (int)((H + p.rows_per_seg - 1) / p.rows_per_seg);
  const int units = p.nstrip * p.nseg;
  p.grid = dim3((unsigned)((units + 3) / 4), (unsigned)s.batch);
  return p;
}
// LDS of a block besides the sink's own needs: value rings + queues of the four waves
template <typename Entry>
constexpr size_t ring_bytes2d() {
  return (size_t)4 * kChunkRows * kWave * kNC * sizeof(float) + (size_t)4 * kQueueCap * sizeof(Entry);
}

}  // namespace ecc
