// Soft ECC, state kept between the forward and the backward pass (shared by the 2D and the 3D
// kernels): layout of the state buffer, and the walk over a unit's saved list that yields
// grad_X (Eq. 8 of the paper contracted with the upstream gradient).
#pragma once
#include "ecc_device.h"
#include "ecc_internal.h"

namespace ecc {

// ---- state saved by the forward pass for the backward pass -----------------------------------
// Header as ecc_internal.h describes it, followed by a generation number: every saving forward
// pass raises it by one (its reduction kernel does, after the sweep), and a unit that runs out
// of room writes the generation it belongs to into its item's overflow word.  An item's lists
// are usable when the header matches the shape and that word is not the current generation --
// so nothing in the state ever needs clearing, whatever it held before.
struct StateView {
  SoftStateHeader* hdr;
  unsigned* gen;       // generation of the lists the state holds
  unsigned* overflow;  // [batch]: generation in which a unit of the item last ran out of room
  unsigned* counts;    // [batch][units]: critical vertices each unit found (may exceed cap)
  SavedEntry* lists;   // [batch][units][cap]
};
static inline size_t align256(size_t n) { return (n + 255) / 256 * 256; }
static inline StateView state_view(void* state, int64_t batch, size_t units) {
  char* b = static_cast<char*>(state);
  StateView v;
  v.hdr = reinterpret_cast<SoftStateHeader*>(b);
  v.gen = reinterpret_cast<unsigned*>(b + 128);
  v.overflow = reinterpret_cast<unsigned*>(b + 256);
  v.counts = reinterpret_cast<unsigned*>(b + 256 + align256((size_t)batch * 4));
  v.lists = reinterpret_cast<SavedEntry*>(b + 256 + align256((size_t)batch * 4) + align256((size_t)batch * units * 4));
  return v;
}
static inline size_t state_bytes(int64_t batch, size_t units, unsigned cap) {
  return 256 + align256((size_t)batch * 4) + align256((size_t)batch * units * 4) +
         (size_t)batch * units * cap * sizeof(SavedEntry);
}
__device__ __forceinline__ bool state_usable(const StateView& v, const SoftStateHeader& e, int item) {
  const SoftStateHeader h = *v.hdr;
  return h.magic == e.magic && h.D == e.D && h.H == e.H && h.W == e.W && h.batch == e.batch && h.nstrip == e.nstrip &&
         h.nseg == e.nseg && h.rows_per_seg == e.rows_per_seg && h.units == e.units && h.tiltc == e.tiltc &&
         h.cap == e.cap && v.overflow[item] != *v.gen;
}

constexpr int kSavedLanes = 8;  // lanes per entry
struct StagedEntry {
  float yh, yl, c;
  int idx;
};
__device__ __forceinline__ float soft_dsig(float tau, float yh, float yl, float kneg) {  // sigma (1 - sigma)
  const float ex = soft_exp_neg((tau - yh) - yl, kneg);
  const float s = __builtin_amdgcn_rcpf(1.0f + ex);
  return ex * s * s;
}

// One block (256 threads) walks one unit's list, 256 entries at a time: entries whose sigmoids
// are all saturated are dropped (grad_X stays 0 there, see soft_sat_bounds), the others are
// packed into an LDS stage and get eight lanes each -- every lane sums an eighth of the
// thresholds, three lane swaps add the eight partial sums.
// first: entry number threadIdx.x of the list, requested by the caller ahead of time; stau / sg:
// thresholds and upstream gradient in LDS; stage: 256 entries, skept: 4 ints of LDS.
__device__ __forceinline__ void saved_lists_to_grad(const SavedEntry* __restrict__ list, unsigned cnt_raw, unsigned cap,
                                                    const SavedEntry& first, const float* stau, const float* sg, int T,
                                                    float kneg, float lambda, float sat_lo, float sat_hi,
                                                    float* __restrict__ gx, int64_t N, StagedEntry* stage, int* skept) {
  const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
  // (<= cap when the forward pass wrote it: the item did not overflow; clamped all the same, and
  // positions are checked below, so that a state that was never written cannot lead out of bounds)
  const unsigned cnt = min(cnt_raw, cap);
  const int q = lane & (kSavedLanes - 1), slot = threadIdx.x / kSavedLanes;  // 32 entries per pass
  for (unsigned e0 = 0; e0 < cnt; e0 += 256) {
    bool keep = false;
    StagedEntry mine;
    if (e0 + threadIdx.x < cnt) {
      const SavedEntry en = e0 == 0 ? first : list[e0 + threadIdx.x];
      mine.yh = (float)en.y;
      mine.yl = (float)(en.y - (double)mine.yh);
      mine.c = (float)en.c;
      mine.idx = en.idx;
      keep = mine.yh > sat_lo && mine.yh < sat_hi;
    }
    const unsigned long long m = __builtin_amdgcn_ballot_w64(keep);
    if (lane == 0) skept[wv] = __builtin_popcountll(m);
    __syncthreads();  // (also: the previous round's readers of the stage are done)
    int base = 0, kept = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      if (w < wv) base += skept[w];
      kept += skept[w];
    }
    const int pos = base + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
    if (keep) stage[pos] = mine;
    __syncthreads();
    for (int b = 0; b < kept; b += 256 / kSavedLanes) {
      const bool on = b + slot < kept;
      const StagedEntry en = stage[on ? b + slot : 0];
      float g0 = 0.0f, g1 = 0.0f;  // two independent chains
      int j = q;
      for (; j + kSavedLanes < T; j += 2 * kSavedLanes) {
        g0 += sg[j] * soft_dsig(stau[j], en.yh, en.yl, kneg);
        g1 += sg[j + kSavedLanes] * soft_dsig(stau[j + kSavedLanes], en.yh, en.yl, kneg);
      }
      if (j < T) g0 += sg[j] * soft_dsig(stau[j], en.yh, en.yl, kneg);
      float gd = g0 + g1;
      gd += dpp_move<0xB1, 0xf>(gd);   // quad_perm [1,0,3,2]
      gd += dpp_move<0x4E, 0xf>(gd);   // quad_perm [2,3,0,1]
      gd += dpp_move<0x141, 0xf>(gd);  // row_half_mirror: the other quad of the eight
      if (on && q == 0 && (unsigned)en.idx < (unsigned)N) gx[en.idx] = -lambda * en.c * gd;
    }
  }
}

}  // namespace ecc
