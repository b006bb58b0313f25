// Hard Euler Characteristic Curve of small and mid-sized float32 inputs without a range, in two or three launches.
//
// Below a few hundred thousand vertices a call is bound by its chain of dependent launches
// (clear, sweep with the range, bin, gated second sweep, scan: five links of 4 to 5 us each),
// not by the stencil.  Here the chain has two links and nothing has to be cleared first:
//   stage  : one thread per vertex (Eq. 3 of the paper, neighbours through the caches); every
//            block packs its critical vertices (value, c) into a list of its own and leaves the
//            list's length and the minimum / maximum of its values in a header of its own;
//   finish : one block per item: the batch's range from the headers, the threshold table and a
//            histogram in LDS, the item's lists binned into it, the prefix sum, the int64 curve
//            written out.
// Binning, thresholds and conventions are those of the large-input kernels (ecc_device.h).
// One block per item has to get through all of the item's critical vertices (white noise, 60 %
// critical: 256^2 in 34 us against 63 us through the five-launch flow; 512^2 would take 94 us
// against 75 us), so items of more than 2^16 vertices take three launches instead: the stage
// blocks also clear the global histogram, the second kernel runs with several blocks per item,
// each binning a share of the item's lists and adding its histogram to the global one, and the
// scan is a launch of its own.  With the thresholds known up front (integer levels, a caller's
// range) the large-input flow has three launches and is as quick.
#include "ecc_device.h"
#include "ecc_internal.h"

namespace ecc {

constexpr int kStageBlock = 256, kFinishBlock = 1024, kFewThreads = 256;
constexpr int64_t kSmallTotal = (int64_t)1 << 18;  // vertices in the whole batch
constexpr int64_t kSmallItem = (int64_t)1 << 16;   // vertices in an item that one finishing block takes
constexpr unsigned kSmallShares = 16;              // finishing blocks per larger item
constexpr int64_t kSmallBatch = 64;                // items (larger batches: the mid-sized flow below)
constexpr int kSmallBins = 4096;

typedef ListHead SmallHead;

struct SmallPlan {
  int per_thread;       // vertices per thread of a stage block
  int per_block;        // vertices (and list room) per stage block
  unsigned per_item;    // stage blocks per item
  unsigned blocks;      // stage blocks in all
  size_t head_bytes;    // headers, a multiple of 256 bytes
};

static SmallPlan small_plan(const Shape& s) {
  SmallPlan p;
  const int64_t total = s.N * s.batch;
  int64_t pt = (total + 131071) / 131072;  // up to 512 blocks of 256 or 512 vertices (measured best at 512^2)
  p.per_thread = (int)(pt < 1 ? 1 : (pt > 4 ? 4 : pt));
  p.per_block = kStageBlock * p.per_thread;
  p.per_item = (unsigned)((s.N + p.per_block - 1) / p.per_block);
  p.blocks = p.per_item * (unsigned)s.batch;
  p.head_bytes = ((size_t)p.blocks * sizeof(SmallHead) + 255) / 256 * 256;
  return p;
}

bool small_supported(const Shape& s, int bins) {
  return s.N * s.batch <= kSmallTotal && s.batch <= kSmallBatch && bins <= kSmallBins;
}

// headers and lists, placed behind the threshold table
size_t small_workspace_bytes(const Shape& s) {
  const SmallPlan p = small_plan(s);
  return p.head_bytes + (size_t)p.blocks * p.per_block * sizeof(uint2);
}

template <int ND, int CONV>
__global__ __launch_bounds__(kStageBlock) void small_stage_kernel(const float* __restrict__ grid, int D, int H, int W,
                                                                  int N, int per_thread,
                                                                  SmallHead* __restrict__ heads,
                                                                  uint2* __restrict__ entries,
                                                                  unsigned long long* __restrict__ hist, int bins) {
  constexpr bool TOP = (CONV & kConvTop) != 0, SUPER = (CONV & kConvSuper) != 0;
  __shared__ unsigned s_count, s_min, s_max;
  if (threadIdx.x == 0) {
    s_count = 0u;
    s_min = 0xffffffffu;
    s_max = 0u;
  }
  __syncthreads();
  if (hist)  // (three-launch form) the item's global histogram, cleared by the item's blocks together
    for (int b = blockIdx.x * kStageBlock + threadIdx.x; b < bins; b += gridDim.x * kStageBlock)
      hist[(int64_t)blockIdx.y * bins + b] = 0ull;
  const float* g = grid + (int64_t)blockIdx.y * N;
  const unsigned blk = blockIdx.y * gridDim.x + blockIdx.x;
  uint2* out = entries + (size_t)blk * (size_t)(kStageBlock * per_thread);
  const int base = (int)blockIdx.x * kStageBlock * per_thread;
  const int lane = threadIdx.x & (kWave - 1);
  unsigned kmin = 0xffffffffu, kmax = 0u;
  for (int k = 0; k < per_thread; ++k) {
    const int i = base + k * kStageBlock + (int)threadIdx.x;
    int c = 0;
    float v = 0.0f;
    if (i < N) {
      const int x = i % W, r = i / W;
      const int y = r % H, z = r / H;
      c = coeff_at<float, ND, TOP, TOP != SUPER>(g, D, H, W, z, y, x);
      if (TOP && ND == 3) c = -c;
      v = g[i];
      const unsigned key = float_key(v);
      kmin = min(kmin, key);
      kmax = max(kmax, key);
    }
    const unsigned long long m = __builtin_amdgcn_ballot_w64(c != 0);
    if (m != 0ull) {  // wave-uniform
      unsigned at = 0u;
      if (lane == 0) at = atomicAdd(&s_count, (unsigned)__builtin_popcountll(m));
      at = (unsigned)__builtin_amdgcn_readfirstlane((int)at);
      const unsigned pos = __builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
      if (c != 0) out[at + pos] = make_uint2(__float_as_uint(v), (unsigned)c);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    kmin = min(kmin, (unsigned)__shfl_xor((int)kmin, o));
    kmax = max(kmax, (unsigned)__shfl_xor((int)kmax, o));
  }
  if (lane == 0) {
    atomicMin(&s_min, kmin);
    atomicMax(&s_max, kmax);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    SmallHead h;
    h.count = s_count;
    h.min_key = s_min;
    h.max_key = s_max;
    h.pad = 0u;
    heads[blk] = h;
  }
}

// The batch's range from all the heads, for launches with so many heads that every finishing
// block reading all of them would cost more than this extra launch.
__global__ __launch_bounds__(kFinishBlock) void small_range_kernel(const SmallHead* __restrict__ heads, unsigned blocks,
                                                                   HardHeader* __restrict__ hdr) {
  __shared__ unsigned s_min, s_max;
  if (threadIdx.x == 0) {
    s_min = 0xffffffffu;
    s_max = 0u;
  }
  __syncthreads();
  unsigned kmin = 0xffffffffu, kmax = 0u;
  for (unsigned b = threadIdx.x; b < blocks; b += kFinishBlock) {
    const SmallHead h = heads[b];
    kmin = min(kmin, h.min_key);
    kmax = max(kmax, h.max_key);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    kmin = min(kmin, (unsigned)__shfl_xor((int)kmin, o));
    kmax = max(kmax, (unsigned)__shfl_xor((int)kmax, o));
  }
  if ((threadIdx.x & (kWave - 1)) == 0 && kmin <= kmax) {
    atomicMin(&s_min, kmin);
    atomicMax(&s_max, kmax);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    hdr->min_key = s_min;
    hdr->max_key = s_max;
  }
}

// BLOCK: threads of a block (1024, or 256 for batches of many small items).
// ALONE: one block per item, which also scans and writes the curve.  Otherwise block (x, item) takes
// the x-th share of the item's lists and adds its histogram to the global one (`curve`, cleared
// by the stage kernel); the scan is a launch of its own.
template <bool ALONE, int BLOCK>
__global__ __launch_bounds__(BLOCK) void small_finish_kernel(const SmallHead* __restrict__ heads,
                                                                    const uint2* __restrict__ entries,
                                                                    unsigned per_item, unsigned blocks, int per_block,
                                                                    int bins, int super,
                                                                    HardHeader* __restrict__ hdr,
                                                                    float* __restrict__ table,
                                                                    long long* __restrict__ curve) {
  extern __shared__ int lhist[];
  float* ltable = reinterpret_cast<float*>(lhist + bins);
  __shared__ unsigned s_min, s_max;
  __shared__ long long wsum[BLOCK / kWave];
  __shared__ unsigned wcnt[BLOCK / kWave];
  __shared__ unsigned off[BLOCK + 1];  // exclusive prefix sums of the lists' lengths
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
  const unsigned item = ALONE ? blockIdx.x : blockIdx.y;
  // this block's lists: all of the item's, or lists l0 .. l0 + nl of it
  const unsigned share = ALONE ? per_item : (per_item + gridDim.x - 1) / gridDim.x;
  const unsigned l0 = ALONE ? 0u : min(per_item, blockIdx.x * share), nl = min(share, per_item - l0);
  // length of this block's list number tid (requested before anything waits on memory)
  const unsigned n_mine = tid < (int)nl ? min(heads[item * per_item + l0 + tid].count, (unsigned)per_block) : 0u;
  const bool first = item == 0 && (ALONE || blockIdx.x == 0);
  // the batch's range: every stage block's header (blocks = 0: small_range_kernel has left it in hdr)
  if (tid == 0) {
    s_min = blocks ? 0xffffffffu : hdr->min_key;
    s_max = blocks ? 0u : hdr->max_key;
  }
  __syncthreads();
  {
    unsigned kmin = 0xffffffffu, kmax = 0u;
    for (unsigned b = tid; b < blocks; b += BLOCK) {
      const SmallHead h = heads[b];
      kmin = min(kmin, h.min_key);
      kmax = max(kmax, h.max_key);
    }
    if (kmin <= kmax) {
      atomicMin(&s_min, kmin);
      atomicMax(&s_max, kmax);
    }
  }
  __syncthreads();
  const double lo_d = (double)key_float(s_min), hi_d = (double)key_float(s_max);
  const float lo = __double2float_rn(lo_d), scale = bin_scale(bins, lo_d, hi_d);
  for (int b = tid; b < bins; b += BLOCK) {
    lhist[b] = 0;
    const float t = super ? threshold_lower_at(b, bins, lo_d, hi_d) : threshold_at(b, bins, lo_d, hi_d);
    ltable[b] = t;
    if (first) table[b] = t;
  }
  if (first && tid == 0) {  // the header as the other flows leave it
    hdr->min_key = s_min;
    hdr->max_key = s_max;
    hdr->lo = lo;
    hdr->scale = scale;
    hdr->overflow = 0u;
  }
  // The item's lists as one sequence: list l holds the entries off[l] .. off[l + 1] of it.  The
  // counts were requested at the top; the sequence is cut into one contiguous piece per wave, a
  // wave walks its piece up to 4 x 64 entries at a time (loads that do not wait for one another), and a
  // lane finds the list of its next entry by stepping on from the list of its last one.
  {
    unsigned inc = n_mine;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const unsigned up = (unsigned)__shfl_up((int)inc, o);
      if (lane >= o) inc += up;
    }
    if (lane == kWave - 1) wcnt[wv] = inc;
    __syncthreads();  // also: histogram cleared, table built
    unsigned before = 0u;
    for (int w = 0; w < wv; ++w) before += wcnt[w];
    off[tid + 1] = before + inc;
    if (tid == 0) off[0] = 0u;
  }
  __syncthreads();
  const unsigned total = off[BLOCK];
  constexpr unsigned kWaves = BLOCK / kWave, kDeep = 4;
  const unsigned piece = ((total + kWaves - 1) / kWaves + kWave - 1) / kWave * kWave;
  const unsigned begin = min(total, (unsigned)wv * piece), end = min(total, begin + piece);
  unsigned l = 0u;  // the last list that starts at or before `begin`
  if (begin < end) {
#pragma unroll
    for (unsigned step = BLOCK / 2; step > 0; step >>= 1)
      if (off[l + step] <= begin) l += step;
  }
  const uint2* mine = entries + ((size_t)item * per_item + l0) * (size_t)per_block;
  for (unsigned f0 = begin + lane; f0 < end + lane; f0 += kWave * kDeep) {  // (wave-uniform trip count)
    uint2 e[kDeep];
    bool ok[kDeep];
#pragma unroll
    for (unsigned q = 0; q < kDeep; ++q) {
      const unsigned f = f0 + q * kWave;
      ok[q] = f < end;
      e[q] = make_uint2(0u, 0u);
      if (ok[q]) {
        while (off[l + 1] <= f) ++l;  // off[l] <= f < off[l + 1]
        e[q] = mine[(size_t)l * (size_t)per_block + (f - off[l])];
      }
    }
#pragma unroll
    for (unsigned q = 0; q < kDeep; ++q) {
      if (ok[q]) {
        const float v = __uint_as_float(e[q].x);
        const int b = super ? bin_super_from_table(v, ltable, bins, lo, scale)
                            : bin_from_table(v, ltable, bins, lo, scale);
        if (b < bins) atomicAdd(&lhist[b], (int)e[q].y);
      }
    }
  }
  __syncthreads();
  if constexpr (!ALONE) {
    unsigned long long* out = reinterpret_cast<unsigned long long*>(curve) + (int64_t)item * bins;
    for (int b = tid; b < bins; b += BLOCK) {
      const int v = lhist[b];
      if (v != 0) atomicAdd(&out[b], (unsigned long long)(long long)v);
    }
    return;
  }
  // inclusive prefix sum over the bins (suffix sum for superlevel sets: the mirrored index)
  const int per = (bins + BLOCK - 1) / BLOCK;
  const int b0 = min(tid * per, bins), b1 = min(b0 + per, bins);
  long long s = 0;
  for (int b = b0; b < b1; ++b) s += (long long)lhist[super ? bins - 1 - b : b];
  long long inc = s;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const long long up = __shfl_up(inc, o);
    if (lane >= o) inc += up;
  }
  if (lane == kWave - 1) wsum[wv] = inc;
  __syncthreads();
  long long run = inc - s;  // exclusive prefix within the wave
  for (int w = 0; w < wv; ++w) run += wsum[w];
  long long* out = curve + (int64_t)item * bins;
  for (int b = b0; b < b1; ++b) {
    const int k = super ? bins - 1 - b : b;
    run += (long long)lhist[k];
    out[k] = run;
  }
}

// `small`: the workspace behind the threshold table
hipError_t launch_hard_small(const float* grid, const Shape& s, int bins, int64_t* curve, HardHeader* hdr, float* table,
                             void* small, hipStream_t st, int conv) {
  const SmallPlan p = small_plan(s);
  SmallHead* heads = static_cast<SmallHead*>(small);
  uint2* entries = reinterpret_cast<uint2*>(static_cast<char*>(small) + p.head_bytes);
  const dim3 g(p.per_item, (unsigned)s.batch);
  const bool alone = s.N <= kSmallItem;
  unsigned long long* hist = reinterpret_cast<unsigned long long*>(curve);
  profile_mark(st, false);
#define ECC_GO(ND, CV)                                                                                       \
  hipLaunchKernelGGL((small_stage_kernel<ND, CV>), g, dim3(kStageBlock), 0, st, grid, (int)s.D, (int)s.H,     \
                     (int)s.W, (int)s.N, p.per_thread, heads, entries, alone ? nullptr : hist, bins)
#define ECC_CONV(ND)                   \
  switch (conv) {                      \
    case 1: ECC_GO(ND, 1); break;      \
    case 2: ECC_GO(ND, 2); break;      \
    case 3: ECC_GO(ND, 3); break;      \
    default: ECC_GO(ND, 0); break;     \
  }
  if (s.ndim == 2) { ECC_CONV(2); } else { ECC_CONV(3); }
#undef ECC_CONV
#undef ECC_GO
  profile_mark(st, true);
  const size_t lds = (size_t)bins * (sizeof(int) + sizeof(float));
  const int super = (conv & kConvSuper) ? 1 : 0;
  if (alone) {
    hipLaunchKernelGGL((small_finish_kernel<true, kFinishBlock>), dim3((unsigned)s.batch), dim3(kFinishBlock), lds, st,
                       heads, entries, p.per_item, p.blocks, p.per_block, bins, super, hdr, table,
                       reinterpret_cast<long long*>(curve));
  } else {
    hipLaunchKernelGGL((small_finish_kernel<false, kFinishBlock>), dim3(kSmallShares, (unsigned)s.batch),
                       dim3(kFinishBlock), lds, st, heads, entries, p.per_item, p.blocks, p.per_block, bins, super, hdr,
                       table, reinterpret_cast<long long*>(curve));
    launch_scan(curve, s, bins, super, st);
  }
  return hipGetLastError();
}

// ---- mid-sized grids: the strip / tube sweep with a list per block ----------------------------
// The five-launch flow clears counters first and keeps a gated second sweep in case a shared list
// overflows.  Here every block of the sweep has a list with room for all of its vertices and a
// head of its own, so nothing is cleared and nothing can overflow; the finishing kernel above (a
// share of the lists per block) and the scan follow.  The price is workspace: 8 bytes per vertex.
// Measured against the five launches (1024 bins, smoothed fields): 32 x 512^2 54 -> 35 us, 16 x 1024^2
// 74 -> 52 us, 8 x 4096^2 199 -> 179 us, 2 x 8192^2 196 -> 175 us, 16 x 4096^2 313 -> 301 us, but the
// smoother fields of the 16 x 4096^2 benchmark batch 254 -> 257 us (8 of them 153 -> 152, 4 of them
// 95 -> 81); volumes 2 x 256^3 82 -> 73 us, 4 x 256^3 118 -> 121 us, 512^3 205 -> 216 us (the lists of
// the blocks lie far apart in a workspace of 8 bytes per vertex): hence the limits.
constexpr int64_t kMidTotal2d = (int64_t)1 << 27, kMidTotal3d = (int64_t)1 << 25;  // vertices in the whole batch
constexpr int64_t kMidBatch = 4096;
constexpr int64_t kMidFinishBlocks = 512;          // finishing blocks in all, about (8 to 128 per item)
constexpr unsigned kMidHeads = 4096;             // more heads than this: a launch of its own reduces the range
constexpr unsigned kMidBlocks = 65536;           // sweep blocks in all

static bool mid_plan(const Shape& s, int dtype, unsigned& per_item, unsigned& cap) {
  if (s.ndim == 2 && sweep2d_supported(s, 1)) {
    per_item = sweep2d_list_blocks(s, dtype);
    cap = sweep2d_block_vertices(s, dtype);
  } else if (sweep3d_supported(s, 1)) {
    if (dtype != 2) return false;  // (the tube sweep's list kernels take float32 here)
    per_item = sweep3d_list_blocks(s);
    cap = sweep3d_block_vertices(s);
  } else {
    return false;
  }
  cap = (cap + 63u) / 64u * 64u;
  return true;
}

// dtype: float32, float16 or bfloat16 (the types whose range is found on the device)
bool mid_supported(const Shape& s, int bins, int dtype) {
  const int64_t most = s.ndim == 2 ? kMidTotal2d : kMidTotal3d;
  if (!(dtype == 2 || dtype == 3 || dtype == 6) || bins > kSmallBins || s.N * s.batch > most || s.batch > kMidBatch)
    return false;
  unsigned per_item, cap;
  if (!mid_plan(s, dtype, per_item, cap)) return false;
  return (int64_t)per_item * s.batch <= kMidBlocks && per_item <= 64u * kFinishBlock;
}

size_t mid_workspace_bytes(const Shape& s, int dtype) {
  unsigned per_item, cap;
  if (!mid_plan(s, dtype, per_item, cap)) return 0;
  const size_t blocks = (size_t)per_item * s.batch;
  return (blocks * sizeof(ListHead) + 255) / 256 * 256 + blocks * cap * sizeof(float2);
}

hipError_t launch_hard_mid(const void* grid, const Shape& s, int dtype, int bins, int64_t* curve, HardHeader* hdr,
                           float* table, void* room, hipStream_t st, int conv, const DirArgs* dir) {
  unsigned per_item, cap;
  mid_plan(s, dtype, per_item, cap);
  const unsigned blocks = per_item * (unsigned)s.batch;
  ListArgs la;
  la.heads = static_cast<ListHead*>(room);
  la.lists = reinterpret_cast<float2*>(static_cast<char*>(room) + ((size_t)blocks * sizeof(ListHead) + 255) / 256 * 256);
  la.cap = cap;
  la.counters = nullptr;
  la.nsub = 1;
  la.hdr = hdr;
  la.zero_hist = reinterpret_cast<unsigned long long*>(curve);
  la.bins = bins;
  profile_mark(st, false);
  if (s.ndim == 2) launch_sweep2d_list(grid, dtype, s, la, st, dir, conv);
  else launch_sweep3d_list(grid, dtype, s, la, st, dir, conv);
  profile_mark(st, true);
  const int super = (conv & kConvSuper) ? 1 : 0;
  const size_t lds = (size_t)bins * (sizeof(int) + sizeof(float));
  const uint2* entries = reinterpret_cast<const uint2*>(la.lists);
  long long* out = reinterpret_cast<long long*>(curve);
  if (s.N <= kSmallItem && per_item <= (unsigned)kFewThreads) {
    // Items one block can finish alone, prefix sum included: no third launch.  Every finishing block
    // would read every head for the range; from about 16 MB of that on a launch of its own is cheaper.
    const bool range_first = (int64_t)blocks * s.batch > ((int64_t)1 << 20);
    if (range_first) hipLaunchKernelGGL(small_range_kernel, dim3(1), dim3(kFinishBlock), 0, st, la.heads, blocks, hdr);
    if (s.batch >= 64 && s.N <= 4096)  // many small items: small blocks
      hipLaunchKernelGGL((small_finish_kernel<true, kFewThreads>), dim3((unsigned)s.batch), dim3(kFewThreads), lds, st,
                         la.heads, entries, per_item, range_first ? 0u : blocks, (int)cap, bins, super, hdr, table, out);
    else
      hipLaunchKernelGGL((small_finish_kernel<true, kFinishBlock>), dim3((unsigned)s.batch), dim3(kFinishBlock), lds, st,
                         la.heads, entries, per_item, range_first ? 0u : blocks, (int)cap, bins, super, hdr, table, out);
    return hipGetLastError();
  }
  // finishing blocks per item: about 8 lists each (1024 at most), up to 128 blocks; a lone item gets 16 at least
  unsigned shares = (per_item + 7u) / 8u;
  const unsigned least = s.batch >= 16 ? 1u : 16u / (unsigned)s.batch;
  unsigned most = (unsigned)(kMidFinishBlocks / s.batch);  // about this many finishing blocks in all
  most = most < 8u ? 8u : (most > 128u ? 128u : most);
  shares = shares < least ? least : (shares > most ? most : shares);
  if (shares * kFinishBlock < per_item) shares = (per_item + kFinishBlock - 1) / kFinishBlock;  // (1024 lists a block at most)
  const bool range_first = blocks > kMidHeads || (int64_t)blocks * shares * s.batch > ((int64_t)1 << 20);
  if (range_first) hipLaunchKernelGGL(small_range_kernel, dim3(1), dim3(kFinishBlock), 0, st, la.heads, blocks, hdr);
  hipLaunchKernelGGL((small_finish_kernel<false, kFinishBlock>), dim3(shares, (unsigned)s.batch), dim3(kFinishBlock), lds, st,
                     la.heads, entries, per_item, range_first ? 0u : blocks, (int)cap, bins, super, hdr, table, out);
  launch_scan(curve, s, bins, super, st);
  return hipGetLastError();
}

}  // namespace ecc
