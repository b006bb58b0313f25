// 3D sweep for gfx950: coefficient c(p) (Eq. 3 of the paper), critical vertices handed to a sink
// (LDS histogram, list, or the sigmoid sums of the soft path).
//
// Layout.  A wave owns a tube of 62 output columns (64 lanes: one halo column
// each side) x R output rows (plus one halo row above and below) and marches
// through the planes z.  One plane step loads R+2 rows of 256 bytes, each a
// single coalesced buffer load; values live in registers, nothing is staged in
// LDS.  A vertex is read from HBM once per tube, plus the halo.
//
// Stencil, bit-sliced along z.  "q comes before p" is a strict "<" towards the
// 13 later neighbours of p (+x; the three in the next row; the nine in the next
// plane) and is the sign bit of the float difference q - p (zeros are made +0
// on load).  Every lane shifts each of those sign bits into its own 32-bit
// word, one bit per plane, so a word holds one neighbour relation for 32
// consecutive vertices of the lane's column.  The 13 earlier neighbours need
// no compare: [q before p] = not [p before q], which is the word that q's
// column holds for ITS later neighbour p -- a word of another row (register),
// of a side column (one lane over), or of the plane below (one bit up).
// Vertices outside the grid read as +inf, so every bit that involves them comes
// out as "never before p".  All Boolean work then runs on whole words: 32
// vertices per lane per instruction.
//
// Coefficient.  With a = ring of the 8 in-plane neighbours before p, up / dn =
// rings of the planes above / below, up0 / dn0 = the vertices straight above /
// below:   c = ring(a) - up0 ring(a & up) - dn0 ring(a & dn),
// ring(m) = 1 - #arcs(m), an arc starting at edge neighbour k when
// m_k & ~(m_{k-1} & m_{k-2}).  Hence c = P - Q with
//   P = 1 + arcs(a & up)[up0] + arcs(a & dn)[dn0],   Q = arcs(a) + up0 + dn0,
// both summed with bit-sliced full adders and subtracted the same way.  Only
// vertices with c != 0 (the critical ones) are walked bit by bit, and that walk
// only notes (position, c) in the wave's LDS queue; the queue is drained 64
// entries at a time with every lane busy: the value is re-read there (an L2
// hit) and binned into the block's LDS histogram or appended to the item's list.
//
// A chunk is up to 30 planes; the words keep shifting across chunks, so the bit
// above a chunk's first plane is the last plane of the previous chunk (all ones
// below the grid: "never before p" once complemented).
#pragma once
#include "ecc_device.h"
#include "ecc_internal.h"

#include <type_traits>

namespace ecc {

namespace s3 {

constexpr int kOut = 62;   // output columns per wave
constexpr int kXchWords = 9;  // halo words a wave publishes per chunk
constexpr int kChunk = 30;  // output planes per chunk (even: the two plane buffers swap roles each step)

__device__ __forceinline__ unsigned from_right(unsigned v) {  // lane i <- lane i+1
  return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x130, 0xf, 0xf, true);
}
__device__ __forceinline__ unsigned from_left(unsigned v) {  // lane i <- lane i-1
  return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x138, 0xf, 0xf, true);
}
__device__ __forceinline__ unsigned long long ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }

// w <- (w << 1) | signbit(d)
__device__ __forceinline__ unsigned push(unsigned w, float d) {
  return __builtin_amdgcn_alignbit(w, __float_as_uint(d), 31);
}
// Differences with the left operand taken from the lane to the right / left:
//   dr[i] = q[i+1] - p[i],  dl[i] = q[i-1] - p[i].
// DPP-modified subtractions; lanes without a source lane read 0 (their bits
// belong to halo lanes and are never used).  The s_nop covers the two wait
// states a DPP read needs after a VALU write of its source register.
__device__ __forceinline__ void diff_sides(float q, float p, float& dr, float& dl) {
  asm("s_nop 1\n\t"
      "v_sub_f32_dpp %0, %2, %3 wave_shl:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_sub_f32_dpp %1, %2, %3 wave_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:1"
      : "=&v"(dr), "=&v"(dl)
      : "v"(q), "v"(p));
}
__device__ __forceinline__ float diff_right(float q, float p) {
  float dr;
  asm("s_nop 1\n\t"
      "v_sub_f32_dpp %0, %1, %2 wave_shl:1 row_mask:0xf bank_mask:0xf bound_ctrl:1"
      : "=&v"(dr)
      : "v"(q), "v"(p));
  return dr;
}

__device__ __forceinline__ unsigned xor3(unsigned a, unsigned b, unsigned c) { return a ^ b ^ c; }
__device__ __forceinline__ unsigned maj3(unsigned a, unsigned b, unsigned c) {
  return (a & b) | (c & (a | b));
}

template <typename T> struct Load;
template <> struct Load<float> {
  static __device__ __forceinline__ float get(__amdgpu_buffer_rsrc_t r, unsigned v, unsigned s) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, v, s, 0));
  }
};
template <typename T> struct Load16 {  // two-byte elements, kept as they are until they are converted
  static __device__ __forceinline__ T get(__amdgpu_buffer_rsrc_t r, unsigned v, unsigned s) {
    return __builtin_bit_cast(T, (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(r, v, s, 0));
  }
};
template <> struct Load<uint16_t> : Load16<uint16_t> {};
template <> struct Load<int16_t> : Load16<int16_t> {};
template <> struct Load<F16> : Load16<F16> {};
template <> struct Load<Bf16> : Load16<Bf16> {};
template <> struct Load<uint8_t> {
  static __device__ __forceinline__ uint8_t get(__amdgpu_buffer_rsrc_t r, unsigned v, unsigned s) {
    return (uint8_t)__builtin_amdgcn_raw_buffer_load_b8(r, v, s, 0);
  }
};

// index of the next-plane word for the neighbour (a, b) of a centre
__device__ __forceinline__ constexpr int ui(int a, int b) { return (b + 1) * 3 + (a + 1); }

template <int R>
struct Words {
  unsigned E[R + 2];                          // centre rows 1..R
  unsigned N[R + 2], NE[R + 2], NW[R + 2];    // centre rows 0..R (towards row +1)
  unsigned U[R + 2][9];                       // centre rows 0..R+1 (towards the plane above)
};

// Is the next-plane relation (centre row jc, neighbour row offset b) needed?
template <int R>
__device__ __forceinline__ constexpr bool need_u(int jc, int b) {
  return (jc >= 1 && jc <= R) || (jc == 0 && b == 1) || (jc == R + 1 && b == -1);
}

// Push the next-plane bits of plane v (centres) against plane u.
template <int R>
__device__ __forceinline__ void push_up(Words<R>& w, const float (&v)[R + 2], const float (&u)[R + 2],
                                        bool skip_top, bool skip_bottom) {
#pragma unroll
  for (int jc = 0; jc <= R + 1; ++jc) {
    if (jc == 0 && skip_top) continue;         // wave-uniform: the wave above supplies these words
    if (jc == R + 1 && skip_bottom) continue;  // the wave below supplies them
#pragma unroll
    for (int b = -1; b <= 1; ++b) {
      if (!need_u<R>(jc, b)) continue;
      const int jq = jc + b;
      float dr, dl;
      diff_sides(u[jq], v[jc], dr, dl);
      w.U[jc][ui(0, b)] = push(w.U[jc][ui(0, b)], u[jq] - v[jc]);
      w.U[jc][ui(1, b)] = push(w.U[jc][ui(1, b)], dr);
      w.U[jc][ui(-1, b)] = push(w.U[jc][ui(-1, b)], dl);
    }
  }
}

// Push the in-plane bits of plane v.
template <int R>
__device__ __forceinline__ void push_plane(Words<R>& w, const float (&v)[R + 2], bool skip_top) {
#pragma unroll
  for (int jc = 0; jc <= R; ++jc) {
    if (jc == 0 && skip_top) continue;  // wave-uniform: the wave above supplies these words
    if (jc >= 1) w.E[jc] = push(w.E[jc], diff_right(v[jc], v[jc]));
    float dr, dl;
    diff_sides(v[jc + 1], v[jc], dr, dl);
    w.N[jc] = push(w.N[jc], v[jc + 1] - v[jc]);
    w.NE[jc] = push(w.NE[jc], dr);
    w.NW[jc] = push(w.NW[jc], dl);
  }
}

// Bit-sliced P = 1 + sum of 8 bits (4-bit result), Q = sum of 6 bits (3-bit result),
// c = P - Q as four two's-complement slices (-5 <= c <= 7); returns the word of
// vertices with c != 0.
struct Slices {
  unsigned d0, d1, d2, d3;
};
__device__ __forceinline__ unsigned count_pq(const unsigned (&s)[8], const unsigned (&t)[6], Slices& o) {
  const unsigned x1 = xor3(s[0], s[1], s[2]), c1 = maj3(s[0], s[1], s[2]);
  const unsigned x2 = xor3(s[3], s[4], s[5]), c2 = maj3(s[3], s[4], s[5]);
  const unsigned x3 = ~(s[6] ^ s[7]), c3 = s[6] | s[7];  // third input is the constant 1
  const unsigned p0 = xor3(x1, x2, x3);
  const unsigned c4 = maj3(x1, x2, x3);
  const unsigned y1 = xor3(c1, c2, c3), d1 = maj3(c1, c2, c3);
  const unsigned p1 = y1 ^ c4;
  const unsigned d2 = y1 & c4;
  const unsigned p2 = d1 ^ d2;
  const unsigned p3 = d1 & d2;
  const unsigned u1 = xor3(t[0], t[1], t[2]), e1 = maj3(t[0], t[1], t[2]);
  const unsigned u2 = xor3(t[3], t[4], t[5]), e2 = maj3(t[3], t[4], t[5]);
  const unsigned q0 = u1 ^ u2;
  const unsigned e3 = u1 & u2;
  const unsigned q1 = xor3(e1, e2, e3);
  const unsigned q2 = maj3(e1, e2, e3);
  // P - Q with a borrow chain
  o.d0 = p0 ^ q0;
  const unsigned b0 = ~p0 & q0;
  o.d1 = xor3(p1, q1, b0);
  const unsigned b1 = maj3(~p1, q1, b0);
  o.d2 = xor3(p2, q2, b1);
  const unsigned b2 = maj3(~p2, q2, b1);
  o.d3 = p3 ^ b2;
  return o.d0 | o.d1 | o.d2 | o.d3;
}

// Critical-vertex queue of a tube.  The walk over the critical bits only notes where
// a vertex is (element offset inside its plane; plane counted from the segment's
// first one) and its coefficient; the value is fetched when 64 entries are drained
// together, so the walk stays short and the re-read costs one wait per 64 vertices.
// The directional sweep also keeps the in-plane part of the vertex's tilt.
template <typename Sink>
struct TubeQueue {
  uint2* buf;   // wave-private LDS, kQueueCap entries: (in-plane offset, plane << 8 | c & 0xff)
  float* tbuf;  // wave-private LDS, kQueueCap in-plane tilts (directional sweep only)
  int count;    // wave-uniform
  Sink sink;

  // fetch(in-plane offset, plane, queue slot) -> value of that vertex
  template <typename F>
  __device__ __forceinline__ void drain(int n, const F& fetch) {
    const int lane = threadIdx.x & (kWave - 1);
    float v = 0.f;
    int c = 0;
    uint2 e = make_uint2(0u, 0u);
    if (lane < n) {
      e = buf[lane];
      c = (int)(e.y << 24) >> 24;
      v = fetch(e.x, e.y >> 8, lane);
    }
    sink.take(n, v, c, e.x, e.y >> 8);  // (value, c, in-plane offset, plane of the segment)
  }
  template <bool TILT, typename F>
  __device__ __forceinline__ void push(bool active, unsigned inplane, unsigned zrel, int c, float txy,
                                       const F& fetch) {
    const int lane = threadIdx.x & (kWave - 1);
    const unsigned long long m = __builtin_amdgcn_ballot_w64(active);
    const int idx = count + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32),
                                                           __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
    if (active) {
      buf[idx] = make_uint2(inplane, (zrel << 8) | ((unsigned)c & 0xffu));
      if (TILT) tbuf[idx] = txy;
    }
    count += __builtin_popcountll(m);
    if (count >= kWave) {
      drain(kWave, fetch);
      const int rest = count - kWave;  // < 64
      const int from = lane < rest ? lane + kWave : lane;
      const uint2 e = buf[from];
      const float t = TILT ? tbuf[from] : 0.f;
      if (lane < rest) {
        buf[lane] = e;
        if (TILT) tbuf[lane] = t;
      }
      count = rest;
    }
  }
  template <typename F>
  __device__ __forceinline__ void flush(const F& fetch) {
    if (count > 0) drain(count, fetch);  // wave-uniform
    count = 0;
  }
};

// arcs of the ring m (order E, NE, N, NW, W, SW, S, SE), gated by g
__device__ __forceinline__ void arc_starts(const unsigned (&m)[8], unsigned g, unsigned* out) {
  out[0] = g & m[0] & ~(m[7] & m[6]);
  out[1] = g & m[2] & ~(m[1] & m[0]);
  out[2] = g & m[4] & ~(m[3] & m[2]);
  out[3] = g & m[6] & ~(m[5] & m[4]);
}

// One tube: columns xs .. xs+63 (outputs xs+1 .. xs+62), output rows
// yb .. yb+R-1, output planes z0 .. z1-1.  SAFE: some lane or row of the tube
// lies outside the grid (those read as +inf).
// A SAFE tube may be folded: when the strip is narrow (the ragged last strip of a
// grid), its S = outputs + 2 columns fit into the wave F times, and fold f (lanes
// f*S .. f*S+S-1) takes the same columns for the rows yb0 + f*R .. yb0 + f*R + R-1.
// Lanes that meet at the seam of two folds are halo lanes on both sides, whose
// outputs are dropped, so the folds do not interact.
// TiltT: the field swept is X + t(p) (directional curves), NoTilt: X itself.
template <typename T, int R, typename Sink, bool SAFE, bool SKIP_TOP, bool SKIP_BOTTOM, typename TiltT>
__device__ __forceinline__ void sweep_tube(const T* __restrict__ g, int64_t item_elems, int D, int H,
                                           int W, int xs, int yb0, int z0, int z1,
                                           TubeQueue<Sink>& queue, unsigned* xch, WaveRange& range,
                                           const TiltT& tilt, int S = kWave, int F = 1) {
  constexpr bool skip_top = SKIP_TOP, skip_bottom = SKIP_BOTTOM;
  const int lane = threadIdx.x & (kWave - 1);
  const int fold = SAFE ? lane / S : 0;  // (S = 64, F = 1: one fold, as the tubes inside the grid)
  const int xl = SAFE ? lane - fold * S : lane;
  const int x = xs + xl;
  const int yb = yb0 + fold * R;  // per lane in a folded tube
  const bool inb = !SAFE || (fold < F && x >= 0 && x < W);
  const bool out_lane = xl >= 1 && xl <= S - 2 && inb;

  // The buffer resource is rebuilt for every plane (base: row 0 of the plane,
  // column xs; column 0 for SAFE tubes), so only one plane has to stay below
  // 2^31 bytes.  Planes past the end of the item are not read (zero records).
  const int64_t plane = (int64_t)H * W;
  const T* const item_end = g + item_elems;
  // Tubes inside the grid: lane offset + the rows' offsets (wave-uniform).  SAFE tubes: the
  // lane's own offset of tube row 1 (vb) and of row 0 (v0), rows 2.. by a wave-uniform step;
  // a row or lane outside the grid reads some address inside the item (or beyond its end,
  // which a buffer load answers with 0) and is replaced by the padding value afterwards.
  const unsigned pitch = (unsigned)W * (unsigned)sizeof(T);
  unsigned roff[R + 2];  // tubes inside the grid: byte offset of tube row j inside a plane
  bool okj[R + 2];       // row j of this lane is inside the grid (and so is the lane)
#pragma unroll
  for (int j = 0; j <= R + 1; ++j) {
    const int y = yb - 1 + j;
    okj[j] = inb && y >= 0 && y < H;
    roff[j] = (unsigned)(yb0 - 1 + j) * pitch;  // (not used by SAFE tubes)
  }
  const unsigned vb = SAFE ? (inb ? ((unsigned)yb * (unsigned)W + (unsigned)x) * (unsigned)sizeof(T) : 0u)
                           : (unsigned)lane * (unsigned)sizeof(T);
  const unsigned v0 = (SAFE && vb >= pitch) ? vb - pitch : 0u;
  const T* pnext = g + (int64_t)max(z0 - 1, 0) * plane + (SAFE ? 0 : xs);  // next plane to load
  // the last plane this segment needs: z1 (above its last output plane) or the grid's last one;
  // what the pipeline would fetch beyond it is that plane again (a cache hit, no memory traffic)
  const T* const plast = g + (int64_t)min(z1, D - 1) * plane + (SAFE ? 0 : xs);
  auto load_plane = [&](T (&raw)[R + 2]) {
    const int64_t left = (item_end - pnext) * (int64_t)sizeof(T);
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<T*>(pnext), 0, (int)(left > 0x7fffffff ? 0x7fffffff : (left > 0 ? left : 0)), 0x00020000);
#pragma unroll
    for (int j = 0; j <= R + 1; ++j) {
      if (SAFE) raw[j] = (j == 0) ? Load<T>::get(rsrc, v0, 0u) : Load<T>::get(rsrc, vb, (unsigned)(j - 1) * pitch);
      else raw[j] = Load<T>::get(rsrc, vb, roff[j]);
    }
    if (pnext < plast) pnext += plane;
  };
  // tilt of the vertex (x, row j of the tube, plane z): t = fl(fl(fl(a_x x) + fl(a_y y)) + fl(a_z z));
  // txy[j] is the in-plane part (zero made +0, so that equal values differ by +0)
  float txy[R + 2];
#pragma unroll
  for (int j = 0; j <= R + 1; ++j)
    txy[j] = TiltT::kOn ? add_rn(add_rn(mul_rn(tilt.ax, (float)x), mul_rn(tilt.ay, (float)(yb - 1 + j))), 0.0f)
                        : 0.0f;
  int zfix = max(z0 - 1, 0);  // plane the next call of fix converts
  auto fix = [&](float (&dst)[R + 2], const T (&raw)[R + 2]) {
    const float tz = TiltT::kOn ? mul_rn(tilt.az, (float)zfix) : 0.0f;
    ++zfix;
#pragma unroll
    for (int j = 0; j <= R + 1; ++j) {
      float f = (float)raw[j];
      if (TiltT::kNeg) {  // reversed order (top-cell construction); zeros still +0
        f = 0.0f - f;
        asm volatile("" : "+v"(f));  // opaque: a negated source operand downstream would make -0 of it
      }
      else if (TiltT::kOn) f = add_rn(f, add_rn(txy[j], tz));
      else if (HasNegZero<T>::value) f += 0.0f;  // -0 -> +0 so that equal values differ by +0
      if (SAFE) f = okj[j] ? f : (TiltT::kTop ? -INFINITY : INFINITY);
      dst[j] = f;
    }
  };

  // value of a queued critical vertex: plane zrel of the segment (the launch plan keeps a
  // segment's element offsets below 2^32), in-plane offset inpl
  const T* const seg0 = g + (int64_t)z0 * plane;
  auto fetch = [&](unsigned inpl, unsigned zrel, int slot) {
    float val = (float)seg0[zrel * (unsigned)plane + inpl];
    if (TiltT::kOn && !TiltT::kRaw)
      val = add_rn(val, add_rn(queue.tbuf[slot], mul_rn(tilt.az, (float)(z0 + (int)zrel))));
    return val;
  };

  Words<R> w;
  // Two plane buffers swap the roles "current plane" / "plane above" every step,
  // and two raw buffers swap the roles "next to convert" / "in flight".
  float pa[R + 2], pb[R + 2];
  T rawx[R + 2], rawy[R + 2];
  {
    T r0[R + 2];
    load_plane(r0);
    load_plane(rawx);
    load_plane(rawy);
    fix(pa, r0);
  }
  // bit 0 of the next-plane words <- relations between plane z0-1 and plane z0
#pragma unroll
  for (int jc = 0; jc <= R + 1; ++jc)
#pragma unroll
    for (int q = 0; q < 9; ++q) w.U[jc][q] = TiltT::kTop ? 0u : 1u;  // below the grid: "never before p" after complement (reversed order: always)
  if (z0 > 0) {
    // pa = plane z0-1, rawx = plane z0
    fix(pb, rawx);
#pragma unroll
    for (int j = 0; j <= R + 1; ++j) rawx[j] = rawy[j];
    load_plane(rawy);
    push_up<R>(w, pa, pb, false, false);
#pragma unroll
    for (int j = 0; j <= R + 1; ++j) pa[j] = pb[j];
  }
  // now pa = plane z0; rawx = plane z0+1, rawy = plane z0+2 (in flight)

#pragma unroll
  for (int j = 0; j <= R + 1; ++j) w.E[j] = w.N[j] = w.NE[j] = w.NW[j] = 0u;
  for (int z = z0; z < z1; z += kChunk) {
    const int n = min(kChunk, z1 - z);
    // The words are shift registers that are never cleared: after the n pushes of
    // this chunk, bit i holds plane z+n-1-i, so bit n of a next-plane word still
    // holds the relation of the plane below the chunk's first plane.
    int k = 0;
    auto track = [&](const float (&p)[R + 2]) {
      if (Sink::kTrackRange) {
#pragma unroll
        for (int j = 1; j <= R; ++j) {
          const float v = TiltT::kNeg ? -p[j] : p[j];  // the range is that of the original values
          if (SAFE) range.add_if(v, okj[j]);
          else range.add(v);
        }
      }
    };
    for (; k + 2 <= n; k += 2) {
      fix(pb, rawx);  // plane above pa
      load_plane(rawx);
      track(pa);
      push_plane<R>(w, pa, skip_top);
      push_up<R>(w, pa, pb, skip_top, skip_bottom);
      fix(pa, rawy);  // plane above pb
      load_plane(rawy);
      track(pb);
      push_plane<R>(w, pb, skip_top);
      push_up<R>(w, pb, pa, skip_top, skip_bottom);
    }
    if (k < n) {  // odd tail: only in the last chunk of the segment
      fix(pb, rawx);
      track(pa);
      push_plane<R>(w, pa, skip_top);
      push_up<R>(w, pa, pb, skip_top, skip_bottom);
    }
    // Halo words: the waves of a block own consecutive row groups, so the words a
    // wave would compute for its halo rows are words its neighbours hold for their
    // own first / last row.  Swap them through LDS (double-buffered by chunk
    // parity, one barrier per chunk) instead of computing them twice.
    {
      const int wv = threadIdx.x >> 6;
      unsigned* mine = xch + (((z - z0) / kChunk & 1) * 4 + wv) * (kXchWords * kWave) + lane;
      mine[0 * kWave] = w.N[R];
      mine[1 * kWave] = w.NE[R];
      mine[2 * kWave] = w.NW[R];
      mine[3 * kWave] = w.U[R][ui(-1, 1)];
      mine[4 * kWave] = w.U[R][ui(0, 1)];
      mine[5 * kWave] = w.U[R][ui(1, 1)];
      mine[6 * kWave] = w.U[1][ui(-1, -1)];
      mine[7 * kWave] = w.U[1][ui(0, -1)];
      mine[8 * kWave] = w.U[1][ui(1, -1)];
      __syncthreads();
      if (skip_top) {
        const unsigned* up = mine - kXchWords * kWave;
        w.N[0] = up[0 * kWave];
        w.NE[0] = up[1 * kWave];
        w.NW[0] = up[2 * kWave];
        w.U[0][ui(-1, 1)] = up[3 * kWave];
        w.U[0][ui(0, 1)] = up[4 * kWave];
        w.U[0][ui(1, 1)] = up[5 * kWave];
      }
      if (skip_bottom) {
        const unsigned* dn = mine + kXchWords * kWave;
        w.U[R + 1][ui(-1, -1)] = dn[6 * kWave];
        w.U[R + 1][ui(0, -1)] = dn[7 * kWave];
        w.U[R + 1][ui(1, -1)] = dn[8 * kWave];
      }
    }
    if (z + n >= D) {  // the grid's last plane has nothing above it
#pragma unroll
      for (int jc = 1; jc <= R; ++jc)
#pragma unroll
        for (int q = 0; q < 9; ++q) w.U[jc][q] = TiltT::kTop ? (w.U[jc][q] | 1u) : (w.U[jc][q] & ~1u);
    }
    // plane z+i sits at bit n-1-i of every word; the plane below the chunk at bit n of U
    const unsigned planes = (n >= 32) ? 0xffffffffu : ((1u << n) - 1u);

#pragma unroll
    for (int j = 1; j <= R; ++j) {
      // in-plane ring of row j: E NE N NW W SW S SE
      unsigned a[8];
      a[0] = w.E[j];
      a[1] = w.NE[j];
      a[2] = w.N[j];
      a[3] = w.NW[j];
      a[4] = ~from_left(w.E[j]);
      a[5] = ~from_left(w.NE[j - 1]);
      a[6] = ~w.N[j - 1];
      a[7] = ~from_right(w.NW[j - 1]);
      // plane above: relation of (x+a, j+b, z+1) to p
      unsigned mu[8];
      mu[0] = a[0] & w.U[j][ui(1, 0)];
      mu[1] = a[1] & w.U[j][ui(1, 1)];
      mu[2] = a[2] & w.U[j][ui(0, 1)];
      mu[3] = a[3] & w.U[j][ui(-1, 1)];
      mu[4] = a[4] & w.U[j][ui(-1, 0)];
      mu[5] = a[5] & w.U[j][ui(-1, -1)];
      mu[6] = a[6] & w.U[j][ui(0, -1)];
      mu[7] = a[7] & w.U[j][ui(1, -1)];
      const unsigned up0 = w.U[j][ui(0, 0)];
      // plane below: neighbour (x+a, j+b, z-1) comes before p unless p came before it,
      // which is the word of that neighbour's column towards (-a, -b, +1), one plane down
      unsigned md[8];
      md[0] = a[0] & ~(from_right(w.U[j][ui(-1, 0)]) >> 1);
      md[1] = a[1] & ~(from_right(w.U[j + 1][ui(-1, -1)]) >> 1);
      md[2] = a[2] & ~(w.U[j + 1][ui(0, -1)] >> 1);
      md[3] = a[3] & ~(from_left(w.U[j + 1][ui(1, -1)]) >> 1);
      md[4] = a[4] & ~(from_left(w.U[j][ui(1, 0)]) >> 1);
      md[5] = a[5] & ~(from_left(w.U[j - 1][ui(1, 1)]) >> 1);
      md[6] = a[6] & ~(w.U[j - 1][ui(0, 1)] >> 1);
      md[7] = a[7] & ~(from_right(w.U[j - 1][ui(-1, 1)]) >> 1);
      const unsigned dn0 = ~(w.U[j][ui(0, 0)] >> 1);

      unsigned s[8], t[6];
      arc_starts(mu, up0, &s[0]);
      arc_starts(md, dn0, &s[4]);
      arc_starts(a, 0xffffffffu, &t[0]);
      t[4] = up0;
      t[5] = dn0;
      Slices sl;
      unsigned nz = count_pq(s, t, sl) & planes;
      const bool row_ok = !SAFE || okj[j];
      if (!(out_lane && row_ok)) nz = 0u;
      const unsigned inpl = (unsigned)((yb - 1 + j) * W + x);
      while (ballot(nz != 0)) {
        const bool active = nz != 0;
        const int b = active ? 31 - __clz(nz) : 0;
        nz &= ~(1u << b);
        const unsigned cu = ((sl.d0 >> b) & 1u) | (((sl.d1 >> b) & 1u) << 1) | (((sl.d2 >> b) & 1u) << 2) |
                            (((sl.d3 >> b) & 1u) << 3);
        const int c = (int)(cu ^ 8u) - 8;
        // top cells: (-1)^3 times the vertex coefficient
        queue.template push<(TiltT::kOn && !TiltT::kRaw)>(active, inpl, (unsigned)(z - z0 + n - 1 - b), TiltT::kTop ? -c : c, txy[j],
                                        fetch);
      }
    }
  }
  queue.flush(fetch);
}

}  // namespace s3

// How the tubes of one z segment are numbered.  The strips but the last are full (62
// outputs) and have one unit per row group; the last strip is folded when it is
// narrow (see sweep_tube): F row groups per unit.  Units are padded to multiples of
// four per strip kind, so the four waves of a block are four consecutive row groups
// of one strip.
struct Tiling3 {
  int nstrip, ngroup, ngroup4;  // strips, row groups, row groups padded to a multiple of 4
  int S, F;                     // lanes per fold and folds of a last-strip unit
  int ngroupT, full, units_seg; // units of the last strip, units of the full strips, units per segment
};
__host__ __device__ __forceinline__ Tiling3 make_tiling3(int D, int H, int W, long long batch, int R) {
  Tiling3 t;
  t.nstrip = (W + s3::kOut - 1) / s3::kOut;
  t.ngroup = (H + R - 1) / R;
  t.ngroup4 = (t.ngroup + 3) & ~3;
  const int wt = W - s3::kOut * (t.nstrip - 1);  // outputs of the last strip, 1..62
  t.S = kWave;
  t.F = 1;
  // Folding pays when the launch runs many rounds of waves over the chip (fewer waves, 6 % on
  // 512^3); when every wave is resident at once it only makes the last strip's waves the
  // slowest ones (7 % lost on a 256^3 volume of i.i.d. values), so small launches keep one
  // row group per wave.
  const bool many_rounds = (long long)t.nstrip * t.ngroup * batch * D >= 160000;  // about 1.3 rounds of 30-plane units
  if (many_rounds && wt + 2 <= kWave / 2) {
    t.S = wt + 2;
    t.F = kWave / t.S;
    if (t.F > 8) t.F = 8;
    if (t.F > t.ngroup) t.F = t.ngroup;
    if (t.F == 1) t.S = kWave;
  }
  t.ngroupT = (t.ngroup + t.F - 1) / t.F;
  t.full = (t.nstrip - 1) * t.ngroup4;
  t.units_seg = t.full + ((t.ngroupT + 3) & ~3);
  return t;
}
// unit -> (segment, strip, first row group, is it a last-strip unit, has it any row)
__host__ __device__ __forceinline__ void decode_unit3(const Tiling3& t, int unit, int& seg, int& strip, int& group,
                                                      bool& tail, bool& active) {
  seg = unit / t.units_seg;
  const int r = unit - seg * t.units_seg;
  tail = r >= t.full;
  if (tail) {
    strip = t.nstrip - 1;
    const int gt = r - t.full;
    group = gt * t.F;
    active = gt < t.ngroupT;
  } else {
    strip = r / t.ngroup4;
    group = r - strip * t.ngroup4;
    active = group < t.ngroup;
  }
}

// origin of a wave's unit: first column of the tube (its halo column), first output row, first plane
__host__ __device__ __forceinline__ void unit_origin3(int unit, int D, int H, int W, long long batch,
                                                      int planes_per_seg, int R, int& ox, int& oy, int& oz) {
  const Tiling3 tl = make_tiling3(D, H, W, batch, R);
  int seg, strip, group;
  bool tail, active;
  decode_unit3(tl, unit, seg, strip, group, tail, active);
  ox = strip * s3::kOut - 1;
  oy = group * R;
  oz = seg * planes_per_seg;
}

// Work unit of a wave: (z segment, row group(s), column strip) of one item;
// blockIdx.y is the item; the four waves of a block take consecutive row groups
// of one strip, so their halo rows meet in the CU's vector cache and their halo
// words are swapped through LDS.
template <typename T, int R, typename Sink, typename TiltT>
__device__ __forceinline__ void sweep3d_wave(const T* __restrict__ g, int D, int H, int W, int64_t N,
                                             int nstrip, int ngroup, int nseg, int planes_per_seg,
                                             s3::TubeQueue<Sink>& queue, unsigned* xch, WaveRange& range,
                                             const TiltT& tilt) {
  const Tiling3 tl = make_tiling3(D, H, W, gridDim.y, R);
  const int unit = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform
  int seg, strip, group;
  bool tail, active;
  decode_unit3(tl, unit, seg, strip, group, tail, active);
  const int z0 = seg * planes_per_seg;
  const int z1 = min(z0 + planes_per_seg, D);
  if (active && seg < nseg) {
    const int xs = strip * s3::kOut - 1;
    const int yb = group * R;
    // the four waves of a block are four consecutive row groups of one strip and segment
    const bool skip_top = (unit & 3) != 0;
    const bool skip_bottom = (unit & 3) != 3 && group + 1 < ngroup;
    const bool safe = tail || (xs < 0) || (xs + kWave > W) || (yb == 0) || (yb + R + 1 > H);
    // tubes touching the grid boundary compute their own halo words (one variant fewer)
    if (safe)
      s3::sweep_tube<T, R, Sink, true, false, false, TiltT>(g, N, D, H, W, xs, yb, z0, z1, queue, xch, range, tilt,
                                                            tail ? tl.S : kWave, tail ? tl.F : 1);
    else if (skip_top && skip_bottom)
      s3::sweep_tube<T, R, Sink, false, true, true, TiltT>(g, N, D, H, W, xs, yb, z0, z1, queue, xch, range, tilt);
    else if (skip_top)
      s3::sweep_tube<T, R, Sink, false, true, false, TiltT>(g, N, D, H, W, xs, yb, z0, z1, queue, xch, range, tilt);
    else if (skip_bottom)
      s3::sweep_tube<T, R, Sink, false, false, true, TiltT>(g, N, D, H, W, xs, yb, z0, z1, queue, xch, range, tilt);
    else
      s3::sweep_tube<T, R, Sink, false, false, false, TiltT>(g, N, D, H, W, xs, yb, z0, z1, queue, xch, range, tilt);
  } else {
    // a wave without a row group still meets the block's one barrier per chunk
    for (int z = z0; z < z1; z += s3::kChunk) __syncthreads();
  }
}

constexpr int kXchInts = 2 * 4 * s3::kXchWords * kWave;  // exchange words of a block, in ints

constexpr int kRows3d = 4;

struct Plan3d {
  int nstrip, ngroup, nseg, planes_per_seg;
  dim3 grid;
};
template <typename T>
static Plan3d plan3d(const Shape& s) {
  constexpr int R = kRows3d;
  Plan3d p;
  const int D = (int)s.D, H = (int)s.H, W = (int)s.W;
  const Tiling3 tl = make_tiling3(D, H, W, s.batch, R);
  p.nstrip = tl.nstrip;
  p.ngroup = tl.ngroup;
  const int64_t per_seg = (int64_t)tl.units_seg * s.batch;
  // about 2.5 rounds of waves over the chip on 512^3 (60-plane segments); measured best
  // between the ragged last round of fewer, longer segments and the three extra planes
  // every segment reads
  int64_t nseg = (16384 + per_seg - 1) / per_seg;
  const int64_t max_seg = (D + s3::kChunk - 1) / s3::kChunk;
  if (nseg > max_seg) nseg = max_seg;
  if (nseg < 1) nseg = 1;
  // whole chunks per segment; a segment's element offsets stay below 2^32 and its plane
  // count below 2^24 (what the critical-vertex queue stores)
  int64_t planes = ((D + nseg - 1) / nseg + s3::kChunk - 1) / s3::kChunk * s3::kChunk;
  // A small launch, whose one-chunk segments leave wave slots empty (256 CUs x 4 SIMDs x 4 waves),
  // takes shorter segments, down to 12 planes, until the slots are filled: each wave's march is
  // the critical path of the call (256^3 uint16: 73 -> 66 us with 20-plane segments).
  if (per_seg * max_seg < 4096) {
    int64_t want = (4096 + per_seg - 1) / per_seg;
    int64_t pl = (D + want - 1) / want;
    pl = (pl + 1) & ~(int64_t)1;
    if (pl < 12) pl = 12;
    if (pl < planes) planes = pl;
  }
  int64_t fit = (((int64_t)1 << 32) - 1) / ((int64_t)H * W);
  if (fit > (1 << 24) - 1) fit = (1 << 24) - 1;
  fit = fit / s3::kChunk * s3::kChunk;  // >= one chunk: a supported plane has fewer than 2^27 elements
  if (planes > fit) planes = fit;
  p.planes_per_seg = (int)planes;
  p.nseg = (int)((D + p.planes_per_seg - 1) / p.planes_per_seg);
  const int64_t units = (int64_t)p.nseg * tl.units_seg;
  p.grid = dim3((unsigned)(units / 4), (unsigned)s.batch);
  return p;
}
constexpr size_t kFixedLds3d = (size_t)4 * kQueueCap * (sizeof(uint2) + sizeof(float)) + (size_t)kXchInts * 4;


}  // namespace ecc
