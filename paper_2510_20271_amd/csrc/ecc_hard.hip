// Hard Euler Characteristic Curve on gfx950: range pass, threshold table,
// coefficient + LDS-privatised histogram sweep, global merge, prefix scan.
//
// Steps (Eq. 3 of the paper; Methods, "full sweep" kernel):
//   range   : batch-global min/max of a float grid (only when no range given)
//   prepare : threshold table t_b and zeroed global histogram
//   sweep   : c(p) for every vertex, hist_block[bin(X(p))] += c(p) in LDS,
//             block histogram merged into the global one with 64-bit atomics
//   scan    : inclusive prefix sum of each item's histogram -> int64 curve
#include "ecc_device.h"
#include "ecc_internal.h"

#include <algorithm>
#include <cstdlib>
#include <atomic>
#include <mutex>

namespace ecc {

constexpr int kBlock = 256;

// ---------------------------------------------------------------------------
// range pass
// ---------------------------------------------------------------------------
// resets the header and the list counters; hist (may be null): zeroed too
__global__ void init_header_kernel(HardHeader* h, unsigned* counters, int ncounters,
                                   unsigned long long* hist, int64_t hist_len) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  if (i == 0) {
    h->min_key = 0xffffffffu;
    h->max_key = 0u;
    h->overflow = 0u;
  }
  if (counters)
    for (int64_t k = i; k < ncounters; k += stride) counters[k] = 0u;
  if (hist)
    for (int64_t k = i; k < hist_len; k += stride) hist[k] = 0ull;
}

__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}

__global__ __launch_bounds__(kBlock) void minmax_f32_kernel(const float* __restrict__ g, int64_t n,
                                                            HardHeader* h) {
  float lo = INFINITY, hi = -INFINITY;
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  const int64_t n4 = n >> 2;
  const float4* g4 = reinterpret_cast<const float4*>(g);
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n4; i += stride) {
    float4 v = g4[i];
    lo = fminf(fminf(lo, v.x), fminf(v.y, fminf(v.z, v.w)));
    hi = fmaxf(fmaxf(hi, v.x), fmaxf(v.y, fmaxf(v.z, v.w)));
  }
  for (int64_t i = (n4 << 2) + (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) {
    float v = g[i];
    lo = fminf(lo, v);
    hi = fmaxf(hi, v);
  }
  lo = wave_min(lo);
  hi = wave_max(hi);
  __shared__ float slo[kBlock / kWave], shi[kBlock / kWave];
  const int wv = threadIdx.x / kWave, ln = threadIdx.x % kWave;
  if (ln == 0) { slo[wv] = lo; shi[wv] = hi; }
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int k = 1; k < kBlock / kWave; ++k) { lo = fminf(lo, slo[k]); hi = fmaxf(hi, shi[k]); }
    if (lo <= hi) {
      atomicMin(&h->min_key, float_key(lo));
      atomicMax(&h->max_key, float_key(hi));
    }
  }
}

// ---------------------------------------------------------------------------
// thresholds + zeroed histogram
// ---------------------------------------------------------------------------
// t_b = float32(lo + (b+1)(hi-lo)/B) in float64 with every operation rounded
// on its own (no contraction), t_{B-1} = float32(hi); lower != 0: the lower edges
// of the same bins (superlevel curves).
__global__ void prepare_kernel(HardHeader* h, float* __restrict__ table, int bins, int from_device,
                               double lo_host, double hi_host, unsigned long long* hist,
                               int64_t hist_len, int lower) {
  double lo, hi;
  if (from_device) {
    lo = (double)key_float(h->min_key);
    hi = (double)key_float(h->max_key);
  } else {
    lo = lo_host;
    hi = hi_host;
  }
  const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t b = tid; b < bins; b += stride)
    table[b] = lower ? threshold_lower_at((int)b, bins, lo, hi) : threshold_at((int)b, bins, lo, hi);
  for (int64_t i = tid; i < hist_len; i += stride) hist[i] = 0ull;
  if (tid == 0) {
    h->lo = __double2float_rn(lo);
    h->scale = bin_scale(bins, lo, hi);
  }
}

// ---------------------------------------------------------------------------
// generic sweep: one thread per vertex, neighbours read through the caches
// ---------------------------------------------------------------------------
// CONV: kConvTop (top-cell construction: outside first, (-1)^d times the vertex formula) and /
// or kConvSuper (superlevel sets: descending order, lower bin edges); the order the stencil
// runs on is reversed when exactly one of the two is set
template <typename T, int ND, bool LEVELS, int CONV>
__global__ __launch_bounds__(kBlock) void sweep_generic_kernel(
    const T* __restrict__ grid, int64_t D, int64_t H, int64_t W, int64_t N, int bins,
    const HardHeader* __restrict__ hdr, const float* __restrict__ table,
    unsigned long long* __restrict__ hist) {
  extern __shared__ int lhist[];
  for (int b = threadIdx.x; b < bins; b += kBlock) lhist[b] = 0;
  __syncthreads();
  const T* g = grid + (int64_t)blockIdx.y * N;
  float lo = 0.f, scale = 0.f;
  if (!LEVELS) { lo = hdr->lo; scale = hdr->scale; }
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < N; i += stride) {
    const int64_t x = i % W;
    const int64_t r = i / W;
    const int64_t y = r % H;
    const int64_t z = r / H;
    constexpr bool TOP = (CONV & kConvTop) != 0, SUPER = (CONV & kConvSuper) != 0;
    int c = coeff_at<T, ND, TOP, TOP != SUPER>(g, D, H, W, z, y, x);
    if (TOP && ND == 3) c = -c;
    if (c != 0) {
      const T v = g[i];
      int b;
      if (LEVELS) b = bin_levels<SUPER>(as_float(v), bins);
      else b = bin_table<SUPER>(as_float(v), table, bins, lo, scale);
      if (b < bins) atomicAdd(&lhist[b], c);
    }
  }
  __syncthreads();
  unsigned long long* out = hist + (int64_t)blockIdx.y * bins;
  for (int b = threadIdx.x; b < bins; b += kBlock) {
    const int v = lhist[b];
    if (v != 0) atomicAdd(&out[b], (unsigned long long)(long long)v);
  }
}

// ---------------------------------------------------------------------------
// single-pass mode: bin the lists of critical vertices once the range is known
// ---------------------------------------------------------------------------
// Every block builds the threshold table from the range the sweep found (LDS);
// block (0, 0) also leaves it, with the factor of the bin guess, in the
// workspace for the histogram-mode sweep that runs if a list overflowed.
// lower != 0: superlevel curves (lower bin edges, bin = last threshold <= value).
// Few, large blocks: every block ends by adding its histogram to the global one, and atomics on
// one address queue up behind each other (256 blocks per item cost 10 us there, 32 cost one).
constexpr int kBinBlock = 1024;
__global__ __launch_bounds__(kBinBlock) void binlist_kernel(ListArgs la, float* __restrict__ table, int bins,
                                                         unsigned long long* __restrict__ hist, int lower) {
  extern __shared__ int lhist[];
  float* ltable = reinterpret_cast<float*>(lhist + bins);
  // Wave w of block x (16 waves) takes the sub-lists 16x + w, 16x + w + 16 gridDim.x, ... of item y.  What it
  // needs from memory is requested in as few dependent steps as possible: the fill counts of all
  // its sub-lists at once (lane k holds the k-th), then the first 256 entries of its first
  // sub-list, both before the header is looked at and the table is built.
  const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
  const unsigned sl0 = blockIdx.x * (kBinBlock / kWave) + wv, step = gridDim.x * (kBinBlock / kWave);
  unsigned mycount = 0;
  {
    const unsigned sl = sl0 + (unsigned)lane * step;
    if (sl < la.nsub) mycount = min(la.counters[blockIdx.y * la.nsub + sl], la.cap);
  }
  const unsigned n0 = sl0 < la.nsub ? (unsigned)__builtin_amdgcn_readlane((int)mycount, 0) : 0u;
  float2 e0[4];
  {
    const float2* list = la.lists + (size_t)(blockIdx.y * la.nsub + (sl0 < la.nsub ? sl0 : 0u)) * la.cap;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const unsigned i = q * kWave + lane;
      e0[q] = i < n0 ? list[i] : make_float2(0.f, 0.f);
    }
  }
  const double lo_d = (double)key_float(la.hdr->min_key), hi_d = (double)key_float(la.hdr->max_key);
  const float lo = __double2float_rn(lo_d), scale = bin_scale(bins, lo_d, hi_d);
  const bool first = blockIdx.x == 0 && blockIdx.y == 0;
  const bool overflow = la.hdr->overflow != 0u;  // the two-pass sweep that follows does the work
  if (overflow && !first) return;
  for (int b = threadIdx.x; b < bins; b += kBinBlock) {
    const float t = lower ? threshold_lower_at(b, bins, lo_d, hi_d) : threshold_at(b, bins, lo_d, hi_d);
    ltable[b] = t;
    lhist[b] = 0;
    if (first) table[b] = t;
  }
  if (first && threadIdx.x == 0) {
    la.hdr->lo = lo;
    la.hdr->scale = scale;
  }
  if (overflow) return;
  __syncthreads();  // histogram cleared, table built
  auto bin_four = [&](const float2 (&e)[4], unsigned i0, unsigned n) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (i0 + q * kWave + lane < n) {
        const int b = lower ? bin_super_from_table(e[q].x, ltable, bins, lo, scale)
                            : bin_from_table(e[q].x, ltable, bins, lo, scale);
        if (b < bins) atomicAdd(&lhist[b], __float_as_int(e[q].y));
      }
    }
  };
  for (unsigned sl = sl0, k = 0; sl < la.nsub; sl += step, ++k) {
    unsigned n;
    if (k < (unsigned)kWave) {
      n = (unsigned)__builtin_amdgcn_readlane((int)mycount, (int)k);
    } else {  // (more than 64 sub-lists per wave: small launches only)
      n = min(la.counters[blockIdx.y * la.nsub + sl], la.cap);
    }
    const float2* list = la.lists + (size_t)(blockIdx.y * la.nsub + sl) * la.cap;
    unsigned i0 = 0;
    if (k == 0) {
      bin_four(e0, 0, n);
      i0 = 4 * kWave;
    }
    for (; i0 < n; i0 += 4 * kWave) {
      float2 e[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const unsigned i = i0 + q * kWave + lane;
        e[q] = i < n ? list[i] : make_float2(0.f, 0.f);
      }
      bin_four(e, i0, n);
    }
  }
  __syncthreads();
  unsigned long long* out = hist + (int64_t)blockIdx.y * bins;
  for (int b = threadIdx.x; b < bins; b += kBinBlock) {
    const int v = lhist[b];
    if (v != 0) atomicAdd(&out[b], (unsigned long long)(long long)v);
  }
}

// ---------------------------------------------------------------------------
// inclusive prefix sum, one block per batch item, in place (int64); suffix != 0:
// inclusive suffix sum instead (superlevel curves: a point of bin b is in the sets
// of the thresholds 0 .. b), which is the prefix sum over the mirrored index
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void scan_kernel(long long* __restrict__ curve, int bins, int suffix) {
  long long* c = curve + (int64_t)blockIdx.x * bins;
  auto at = [&](int b) -> long long& { return c[suffix ? bins - 1 - b : b]; };
  const int per = (bins + kBlock - 1) / kBlock;
  const int b0 = threadIdx.x * per;
  const int b1 = min(b0 + per, bins);
  long long s = 0;
  for (int b = b0; b < b1; ++b) s += at(b);
  __shared__ long long part[kBlock];
  part[threadIdx.x] = s;
  __syncthreads();
  // Hillis-Steele over the 256 thread sums
  for (int o = 1; o < kBlock; o <<= 1) {
    long long add = (threadIdx.x >= o) ? part[threadIdx.x - o] : 0;
    __syncthreads();
    part[threadIdx.x] += add;
    __syncthreads();
  }
  long long run = part[threadIdx.x] - s;  // exclusive prefix of this thread's span
  for (int b = b0; b < b1; ++b) {
    run += at(b);
    at(b) = run;
  }
}

void launch_scan(int64_t* curve, const Shape& s, int bins, int suffix, hipStream_t st) {
  hipLaunchKernelGGL(scan_kernel, dim3((unsigned)s.batch), dim3(kBlock), 0, st, reinterpret_cast<long long*>(curve), bins,
                     suffix);
}

// ---------------------------------------------------------------------------
// coefficient map (inspection / tests)
// ---------------------------------------------------------------------------
template <typename T, int ND>
__global__ __launch_bounds__(kBlock) void coeff_kernel(const T* __restrict__ grid, int64_t D,
                                                       int64_t H, int64_t W, int64_t N,
                                                       int8_t* __restrict__ out) {
  const T* g = grid + (int64_t)blockIdx.y * N;
  int8_t* o = out + (int64_t)blockIdx.y * N;
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < N; i += stride) {
    const int64_t x = i % W;
    const int64_t r = i / W;
    o[i] = (int8_t)coeff_at<T, ND>(g, D, H, W, r / H, r % H, x);
  }
}

// ---------------------------------------------------------------------------
// sweep-kernel timing with HIP events on the caller's stream
// ---------------------------------------------------------------------------
namespace {
std::mutex g_prof_mutex;
std::atomic<bool> g_prof_on{false};
struct Profile {
  bool on = false;
  int cap = 0, used = 0;
  hipEvent_t* ev = nullptr;  // 2 per launch
} g_prof;
}  // namespace

hipError_t profile_begin(int max_launches) {
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  if (g_prof.on) return hipErrorInvalidValue;
  g_prof.ev = new hipEvent_t[2 * (size_t)max_launches];
  for (int i = 0; i < 2 * max_launches; ++i) {
    hipError_t e = hipEventCreate(&g_prof.ev[i]);
    if (e != hipSuccess) {
      for (int k = 0; k < i; ++k) (void)hipEventDestroy(g_prof.ev[k]);
      delete[] g_prof.ev;
      g_prof.ev = nullptr;
      return e;
    }
  }
  g_prof.cap = max_launches;
  g_prof.used = 0;
  g_prof.on = true;
  g_prof_on.store(true, std::memory_order_release);
  return hipSuccess;
}

void profile_mark(hipStream_t st, bool after) {
  if (!g_prof_on.load(std::memory_order_acquire)) return;  // the usual case: nothing is being recorded
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  if (!g_prof.on || g_prof.used >= g_prof.cap) return;
  (void)hipEventRecord(g_prof.ev[2 * g_prof.used + (after ? 1 : 0)], st);
  if (after) ++g_prof.used;
}

hipError_t profile_end(float* mean_ms, int* launches) {
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  if (!g_prof.on) return hipErrorInvalidValue;
  hipError_t rc = hipSuccess;
  double sum = 0.0;
  for (int i = 0; i < g_prof.used; ++i) {
    float ms = 0.f;
    hipError_t e = hipEventSynchronize(g_prof.ev[2 * i + 1]);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, g_prof.ev[2 * i], g_prof.ev[2 * i + 1]);
    if (e != hipSuccess) rc = e;
    sum += ms;
  }
  *launches = g_prof.used;
  *mean_ms = g_prof.used ? (float)(sum / g_prof.used) : 0.f;
  for (int i = 0; i < 2 * g_prof.cap; ++i) (void)hipEventDestroy(g_prof.ev[i]);
  delete[] g_prof.ev;
  g_prof = Profile();
  g_prof_on.store(false, std::memory_order_release);
  return rc;
}

// ---------------------------------------------------------------------------
// host launchers
// ---------------------------------------------------------------------------
// Workspace: header | threshold table | list counters [batch] | lists [batch][cap].
// The lists (single-pass mode for float grids without a range) hold one entry
// of 8 bytes per critical vertex; room for one vertex in eight.
static size_t table_bytes(int bins) { return (((size_t)bins * sizeof(float) + 255) / 256) * 256; }
// Lists of an item: room for one vertex in eight (for every vertex when the item
// has fewer than 8192), split into a power-of-two number of sub-lists of at
// least kMinSubListCap entries each (a single shorter one for tiny items).
static int64_t list_entries(const Shape& s) {
  const int64_t all = (s.N + 63) / 64 * 64;
  const int64_t eighth = s.N / 8;
  return eighth >= 8192 ? eighth : (all < 8192 ? all : 8192);
}
static unsigned list_nsub(const Shape& s) {
  unsigned n = 1;
  while (n < kMaxSubLists && list_entries(s) / (2 * n) >= (int64_t)kMinSubListCap) n *= 2;
  return n;
}
static unsigned list_cap(const Shape& s) {  // entries per sub-list
  int64_t cap = (list_entries(s) / list_nsub(s) + 63) / 64 * 64;
  if (cap > (int64_t)1 << 30) cap = (int64_t)1 << 30;
  return (unsigned)cap;
}
static size_t counter_bytes(const Shape& s) { return (((size_t)s.batch * list_nsub(s) * 4 + 255) / 256) * 256; }
size_t hard_workspace_min_bytes(const Shape& s, int bins) {
  const size_t lists = counter_bytes(s) + (size_t)s.batch * list_nsub(s) * list_cap(s) * sizeof(float2);
  const size_t small = small_supported(s, bins) ? small_workspace_bytes(s) : 0;
  return kTableOffset + table_bytes(bins) + std::max(lists, small);
}
// with room for a list per block of the sweep (mid-sized float grids; the launch plans of the
// four-byte and the two-byte types differ)
size_t hard_workspace_bytes(const Shape& s, int bins) {
  size_t mid = 0;
  for (int dtype : {2, 3})
    if (mid_supported(s, bins, dtype)) mid = std::max(mid, kTableOffset + table_bytes(bins) + mid_workspace_bytes(s, dtype));
  return std::max(hard_workspace_min_bytes(s, bins), mid);
}

static int blocks_for(int64_t N) {
  int64_t nb = (N + kBlock - 1) / kBlock;
  return (int)(nb < 1 ? 1 : (nb > 4096 ? 4096 : nb));
}

template <typename T>
static void launch_sweep_generic(const void* grid, const Shape& s, bool levels, int bins,
                                 const HardHeader* hdr, const float* table,
                                 unsigned long long* hist, hipStream_t st, int conv) {
  dim3 g(blocks_for(s.N), (unsigned)s.batch);
  size_t lds = (size_t)bins * sizeof(int);
  const T* p = static_cast<const T*>(grid);
#define ECC_GO(ND, LV, CV)                                                                        \
  hipLaunchKernelGGL((sweep_generic_kernel<T, ND, LV, CV>), g, dim3(kBlock), lds, st, p, s.D, s.H, \
                     s.W, s.N, bins, hdr, table, hist)
#define ECC_CONV(ND, LV)                 \
  switch (conv) {                        \
    case 1: ECC_GO(ND, LV, 1); break;    \
    case 2: ECC_GO(ND, LV, 2); break;    \
    case 3: ECC_GO(ND, LV, 3); break;    \
    default: ECC_GO(ND, LV, 0); break;   \
  }
  if (s.ndim == 2) { if (levels) { ECC_CONV(2, true); } else { ECC_CONV(2, false); } }
  else             { if (levels) { ECC_CONV(3, true); } else { ECC_CONV(3, false); } }
#undef ECC_CONV
#undef ECC_GO
}

hipError_t launch_hard(const void* grid, const Shape& s, int dtype, int bins, bool have_range,
                       double lo, double hi, int64_t* curve, void* ws, hipStream_t st, const DirArgs* dir,
                       int conv, float* f32_scratch, bool roomy) {
  const int super = (conv & kConvSuper) ? 1 : 0;
  HardHeader* hdr = static_cast<HardHeader*>(ws);
  char* wsb = static_cast<char*>(ws);
  float* table = reinterpret_cast<float*>(wsb + kTableOffset);
  unsigned long long* hist = reinterpret_cast<unsigned long long*>(curve);
  const bool is_float = (dtype == 2 || dtype == 3 || dtype == 5 || dtype == 6);  // float32 / 16 / 64, bfloat16
  const bool levels = !have_range && !is_float;
  const bool device_range = !have_range && is_float;
  const int64_t total = s.N * s.batch;
  // test aid (ecc_debug_force): every shape through the plain one-thread-per-vertex sweep, and / or
  // the separate range pass for float grids without a range
  const bool force_generic = (forced_paths() & kForceGeneric) != 0;
  const bool two_pass = (forced_paths() & kForceTwoPass) != 0;
  // With the thresholds known up front, inputs of up to 2^16 vertices are quicker through
  // the one-thread-per-vertex sweep: a strip / tube wave marching alone is bound by its own
  // instruction latency (256^2 uint8: 11.7 against 19.5 us).
  const bool tiny = !device_range && total <= (1 << 16);
  // (a directional call comes here only for shapes the strip / tube sweeps take)
  const bool fast2d = (dir || (!force_generic && !tiny)) && sweep2d_supported(s, bins);
  const bool fast3d = (dir || (!force_generic && !tiny)) && !fast2d && sweep3d_supported(s, bins);
  // Small float grids without a range: the whole call in two launches.
  if (device_range && !dir && forced_paths() == 0u && small_supported(s, bins)) {
    if (dtype >= 3) {
      hipError_t e = launch_convert(grid, dtype, total, f32_scratch, st);
      if (e != hipSuccess) return e;
      grid = f32_scratch;
    }
    return launch_hard_small(static_cast<const float*>(grid), s, bins, curve, hdr, table,
                             wsb + kTableOffset + table_bytes(bins), st, conv);
  }
  // Mid-sized float grids without a range: the sweep with a list per block, three launches.
  if (device_range && roomy && forced_paths() == 0u && (fast2d || fast3d) && mid_supported(s, bins, dtype))
    return launch_hard_mid(grid, s, dtype, bins, curve, hdr, table, wsb + kTableOffset + table_bytes(bins), st, conv, dir);
  // Element types beyond uint8 / uint16 / float32.  The strip / tube sweeps load float16, bfloat16
  // and int16 as they are (all three widen to float32 exactly); the other kernels, and int32 /
  // float64 everywhere, get a float32 copy rounded to nearest even.
  if (dtype >= 3) {
    const bool native = (dtype == 3 || dtype == 6 || dtype == 7) && (fast2d || fast3d) && !(device_range && two_pass);
    if (!native) {
      hipError_t e = launch_convert(grid, dtype, total, f32_scratch, st);
      if (e != hipSuccess) return e;
      grid = f32_scratch;
      dtype = 2;
    }
  }
  const int64_t hist_len = s.batch * bins;
  int prep_blocks = (int)((hist_len + kBlock - 1) / kBlock);
  prep_blocks = prep_blocks > 1024 ? 1024 : prep_blocks;

  if (device_range && (fast2d || fast3d) && (!two_pass || dir)) {
    // Single pass over the grid: the sweep finds the critical vertices and the
    // range together; the few critical vertices are binned afterwards.  If a list
    // overflows (more than one vertex in eight critical), the histogram-mode sweep
    // that follows runs instead (it is a no-op otherwise).
    ListArgs la = {};  // (heads = null: shared sub-lists)
    la.hdr = hdr;
    la.counters = reinterpret_cast<unsigned*>(wsb + kTableOffset + table_bytes(bins));
    la.lists = reinterpret_cast<float2*>(wsb + kTableOffset + table_bytes(bins) + counter_bytes(s));
    // no more sub-lists than blocks that append to them (a block uses one sub-list);
    // the room of the unused ones goes to the others
    const unsigned blocks = fast2d ? sweep2d_list_blocks(s, dtype) : sweep3d_list_blocks(s);
    la.nsub = list_nsub(s);
    la.cap = list_cap(s);
    while (la.nsub > 1 && la.nsub > blocks) {
      la.nsub /= 2;
      la.cap *= 2;
    }
    int64_t ib = (std::max<int64_t>(s.batch * la.nsub, hist_len) + 255) / 256;
    ib = ib > 1024 ? 1024 : ib;
    hipLaunchKernelGGL(init_header_kernel, dim3((unsigned)ib), dim3(256), 0, st, hdr, la.counters,
                       (int)(s.batch * la.nsub), hist, hist_len);
    profile_mark(st, false);
    if (fast2d) launch_sweep2d_list(grid, dtype, s, la, st, dir, conv);
    else launch_sweep3d_list(grid, dtype, s, la, st, dir, conv);
    profile_mark(st, true);
    // a wave per sub-list, but no more than about 512 blocks in all and 32 to 64 per item (every block
    // ends with one atomic per non-empty bin on the item's histogram)
    int64_t nblk = ((int64_t)la.nsub + kBinBlock / kWave - 1) / (kBinBlock / kWave);
    const int64_t most = std::min<int64_t>(64, std::max<int64_t>(32, 512 / s.batch));
    nblk = nblk > most ? most : (nblk < 1 ? 1 : nblk);
    hipLaunchKernelGGL(binlist_kernel, dim3((unsigned)nblk, (unsigned)s.batch), dim3(kBinBlock),
                       (size_t)bins * 2 * sizeof(int), st, la, table, bins, hist, super);
    if (fast2d) launch_sweep2d(grid, s, dtype, false, bins, hdr, table, hist, st, &hdr->overflow, dir, conv);
    else launch_sweep3d(grid, s, dtype, false, bins, hdr, table, hist, st, &hdr->overflow, dir, conv);
    hipLaunchKernelGGL(scan_kernel, dim3((unsigned)s.batch), dim3(kBlock), 0, st,
                       reinterpret_cast<long long*>(curve), bins, super);
    return hipGetLastError();
  }

  if (device_range) {
    hipLaunchKernelGGL(init_header_kernel, dim3(1), dim3(64), 0, st, hdr, (unsigned*)nullptr, 0,
                       (unsigned long long*)nullptr, (int64_t)0);
    int nb = (int)((total / 4 + kBlock - 1) / kBlock);
    nb = nb < 1 ? 1 : (nb > 2048 ? 2048 : nb);
    hipLaunchKernelGGL(minmax_f32_kernel, dim3(nb), dim3(kBlock), 0, st,
                       static_cast<const float*>(grid), total, hdr);
  }
  hipLaunchKernelGGL(prepare_kernel, dim3(prep_blocks), dim3(kBlock), 0, st, hdr, table, bins,
                     device_range ? 1 : 0, lo, hi, hist, hist_len, super);
  profile_mark(st, false);
  if (fast2d) {
    launch_sweep2d(grid, s, dtype, levels, bins, hdr, table, hist, st, nullptr, dir, conv);
  } else if (fast3d) {
    launch_sweep3d(grid, s, dtype, levels, bins, hdr, table, hist, st, nullptr, dir, conv);
  } else
  switch (dtype) {
    case 0: launch_sweep_generic<uint8_t>(grid, s, levels, bins, hdr, table, hist, st, conv); break;
    case 1: launch_sweep_generic<uint16_t>(grid, s, levels, bins, hdr, table, hist, st, conv); break;
    default: launch_sweep_generic<float>(grid, s, levels, bins, hdr, table, hist, st, conv); break;
  }
  profile_mark(st, true);
  hipLaunchKernelGGL(scan_kernel, dim3((unsigned)s.batch), dim3(kBlock), 0, st,
                     reinterpret_cast<long long*>(curve), bins, super);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// directional curves: hard ECC of the tilted fields X + alpha <u_k, p>
// ---------------------------------------------------------------------------
// Shapes the strip / tube sweeps do not take: the tilted fields are written out
// (one per direction and item) and go through the plain path.
__global__ __launch_bounds__(kBlock) void tilt_kernel(const float* __restrict__ grid, int64_t D, int64_t H,
                                                      int64_t W, int64_t N, DirArgs dir,
                                                      float* __restrict__ out) {
  const int d = blockIdx.y / dir.batch, item = blockIdx.y - d * dir.batch;
  const Tilt t = load_tilt(dir, d);
  const float* g = grid + (int64_t)item * N;
  float* o = out + (int64_t)blockIdx.y * N;
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < N; i += stride) {
    const int64_t x = i % W, r = i / W, y = r % H, z = r / H;
    float tt = add_rn(mul_rn(t.ax, (float)x), mul_rn(t.ay, (float)y));
    if (dir.ndim == 3) tt = add_rn(tt, mul_rn(t.az, (float)z));
    o[i] = add_rn(g[i], tt);
  }
}

static bool dir_fused(const Shape& sv, int bins, bool have_range) {
  const bool tiny = have_range && sv.N * sv.batch <= (1 << 16);
  return !tiny && (sweep2d_supported(sv, bins) || sweep3d_supported(sv, bins));
}

// sv: the shape with batch = directions x items
size_t hard_dir_workspace_bytes(const Shape& sv, int bins) {
  size_t n = hard_workspace_bytes(sv, bins);
  if (!dir_fused(sv, bins, true) || !dir_fused(sv, bins, false))
    n += (((size_t)sv.N * sv.batch * sizeof(float) + 255) / 256) * 256;
  return n;
}

hipError_t launch_hard_dir(const float* grid, const Shape& sv, const float* u, float alpha, int batch,
                           int bins, bool have_range, double lo, double hi, int64_t* curve, void* ws,
                           hipStream_t st) {
  DirArgs dir;
  dir.u = u;
  dir.alpha = alpha;
  dir.batch = batch;
  dir.ndim = sv.ndim;
  if (dir_fused(sv, bins, have_range))
    return launch_hard(grid, sv, 2, bins, have_range, lo, hi, curve, ws, st, &dir);
  float* tilted = reinterpret_cast<float*>(static_cast<char*>(ws) + hard_workspace_bytes(sv, bins));
  hipLaunchKernelGGL(tilt_kernel, dim3(blocks_for(sv.N), (unsigned)sv.batch), dim3(kBlock), 0, st, grid, sv.D,
                     sv.H, sv.W, sv.N, dir, tilted);
  return launch_hard(tilted, sv, 2, bins, have_range, lo, hi, curve, ws, st, nullptr);
}

// ---------------------------------------------------------------------------
// further element types: rounded to float32 (to nearest even) into the workspace
// ---------------------------------------------------------------------------
template <typename S> __device__ __forceinline__ float to_f32(S v) { return (float)v; }
template <> __device__ __forceinline__ float to_f32<Bf16>(Bf16 v) { return (float)v; }

template <typename S>
__global__ __launch_bounds__(kBlock) void convert_kernel(const S* __restrict__ src, int64_t n,
                                                         float* __restrict__ dst) {
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) dst[i] = to_f32<S>(src[i]);
}

// ---------------------------------------------------------------------------
// NaN / Inf census (the sweeps need finite values and do not check)
// ---------------------------------------------------------------------------
__global__ void clear_u64_kernel(unsigned long long* p) { *p = 0ull; }

// EXP: the exponent field's mask in the element's bit pattern (all ones: NaN or Inf)
template <typename U, U EXP>
__global__ __launch_bounds__(kBlock) void count_nonfinite_kernel(const U* __restrict__ bits, int64_t n,
                                                                 unsigned long long* __restrict__ count) {
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  unsigned bad = 0;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) bad += (bits[i] & EXP) == EXP;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) bad += __shfl_xor(bad, o);
  if ((threadIdx.x & (kWave - 1)) == 0 && bad) atomicAdd(count, (unsigned long long)bad);
}

hipError_t launch_count_nonfinite(const void* grid, int64_t n, int dtype, unsigned long long* count, hipStream_t st) {
  hipLaunchKernelGGL(clear_u64_kernel, dim3(1), dim3(1), 0, st, count);
  int64_t nb = (n + kBlock - 1) / kBlock;
  nb = nb > 8192 ? 8192 : nb;
#define ECC_GO(U, EXP)                                                                                     \
  hipLaunchKernelGGL((count_nonfinite_kernel<U, EXP>), dim3((unsigned)nb), dim3(kBlock), 0, st,            \
                     static_cast<const U*>(grid), n, count)
  switch (dtype) {
    case 2: ECC_GO(uint32_t, 0x7f800000u); break;             // float32
    case 3: ECC_GO(uint16_t, (uint16_t)0x7c00u); break;       // float16
    case 5: ECC_GO(uint64_t, 0x7ff0000000000000ull); break;   // float64
    case 6: ECC_GO(uint16_t, (uint16_t)0x7f80u); break;       // bfloat16
    default: break;                                           // integer types: nothing to count
  }
#undef ECC_GO
  return hipGetLastError();
}

hipError_t launch_convert(const void* grid, int dtype, int64_t n, float* out, hipStream_t st) {
  int64_t nb = (n + kBlock - 1) / kBlock;
  nb = nb < 1 ? 1 : (nb > 16384 ? 16384 : nb);
#define ECC_GO(S) \
  hipLaunchKernelGGL(convert_kernel<S>, dim3((unsigned)nb), dim3(kBlock), 0, st, static_cast<const S*>(grid), n, out)
  switch (dtype) {
    case 3: ECC_GO(_Float16); break;
    case 4: ECC_GO(int32_t); break;
    case 5: ECC_GO(double); break;
    case 6: ECC_GO(Bf16); break;
    default: ECC_GO(int16_t); break;
  }
#undef ECC_GO
  return hipGetLastError();
}

// out[0..n) = 0, any alignment
__global__ __launch_bounds__(kBlock) void clear_i8_kernel(int8_t* __restrict__ out, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  const int64_t tid = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const int64_t lead = min<int64_t>(n, (int64_t)((16 - (reinterpret_cast<uintptr_t>(out) & 15)) & 15));
  const int64_t n16 = (n - lead) / 16;
  uint4* body = reinterpret_cast<uint4*>(out + lead);
  for (int64_t i = tid; i < n16; i += stride) body[i] = make_uint4(0u, 0u, 0u, 0u);
  for (int64_t i = tid; i < lead; i += stride) out[i] = 0;
  for (int64_t i = lead + n16 * 16 + tid; i < n; i += stride) out[i] = 0;
}

// Shapes the strip / tube sweeps take go through them (the map is cleared, the sweep writes the
// critical vertices), so that the map shows the stencil every timed path runs; the rest, and
// every shape under ECC_FORCE_GENERIC, through the one-thread-per-vertex kernel.
hipError_t launch_coeff(const void* grid, const Shape& s, int dtype, int8_t* c_out, hipStream_t st) {
  const bool force_generic = (forced_paths() & kForceGeneric) != 0;
  const bool fast2d = !force_generic && sweep2d_supported(s, 1);
  const bool fast3d = !force_generic && !fast2d && sweep3d_supported(s, 1);
  if (fast2d || fast3d) {
    const int64_t total = s.N * s.batch;
    int64_t nb = (total / 16 + kBlock - 1) / kBlock;
    nb = nb < 1 ? 1 : (nb > 4096 ? 4096 : nb);
    hipLaunchKernelGGL(clear_i8_kernel, dim3((unsigned)nb), dim3(kBlock), 0, st, c_out, total);
    if (fast2d) launch_coeff2d(grid, s, dtype, c_out, st);
    else launch_coeff3d(grid, s, dtype, c_out, st);
    return hipGetLastError();
  }
  dim3 g(blocks_for(s.N), (unsigned)s.batch);
#define ECC_GO(T, ND)                                                                          \
  hipLaunchKernelGGL((coeff_kernel<T, ND>), g, dim3(kBlock), 0, st, static_cast<const T*>(grid), \
                     s.D, s.H, s.W, s.N, c_out)
  if (s.ndim == 2) {
    if (dtype == 0) ECC_GO(uint8_t, 2); else if (dtype == 1) ECC_GO(uint16_t, 2); else ECC_GO(float, 2);
  } else {
    if (dtype == 0) ECC_GO(uint8_t, 3); else if (dtype == 1) ECC_GO(uint16_t, 3); else ECC_GO(float, 3);
  }
#undef ECC_GO
  return hipGetLastError();
}

}  // namespace ecc
