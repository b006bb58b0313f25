// Hard ECC, 3D: kernels and launchers around the tube sweep of ecc_sweep3d.h.
#include "ecc_sweep3d.h"

#include <type_traits>

namespace ecc {

// Histogram mode; run_if (may be null): do nothing unless *run_if != 0.
template <typename T, int R, bool LEVELS, bool TLDS, int MODE>
__global__ __launch_bounds__(256) void sweep3d_kernel(
    const T* __restrict__ grid, int D, int H, int W, int64_t N, int bins, int nstrip, int ngroup,
    int nseg, int planes_per_seg, const HardHeader* __restrict__ hdr,
    const float* __restrict__ table, unsigned long long* __restrict__ hist,
    const unsigned* __restrict__ run_if, DirArgs dir) {
  if (run_if && *run_if == 0) return;
  extern __shared__ int smem[];
  // [2][4 waves][9][64] exchange words, [4 waves] queues (entries, tilts), histogram, table
  unsigned* xch = reinterpret_cast<unsigned*>(smem);
  uint2* qbuf = reinterpret_cast<uint2*>(smem + kXchInts) + (threadIdx.x >> 6) * kQueueCap;
  float* tbuf = reinterpret_cast<float*>(smem + kXchInts + 4 * kQueueCap * 2) + (threadIdx.x >> 6) * kQueueCap;
  int* lhist = smem + kXchInts + 4 * kQueueCap * 3;
  float* ltable = reinterpret_cast<float*>(lhist + bins);
  for (int b = threadIdx.x; b < bins; b += 256) {
    lhist[b] = 0;
    if (TLDS) ltable[b] = table[b];
  }
  __syncthreads();
  s3::TubeQueue<HistSink<LEVELS, mode_is_super(MODE)>> queue;
  queue.buf = qbuf;
  queue.tbuf = tbuf;
  queue.count = 0;
  queue.sink.lhist = lhist;
  queue.sink.table = TLDS ? ltable : table;
  queue.sink.bins = bins;
  queue.sink.lo = LEVELS ? 0.f : hdr->lo;
  queue.sink.scale = LEVELS ? 0.f : hdr->scale;
  WaveRange range;
  if constexpr (MODE == kTilted) {
    const int d = blockIdx.y / dir.batch, item = blockIdx.y - d * dir.batch;
    sweep3d_wave<T, R>(grid + (int64_t)item * N, D, H, W, N, nstrip, ngroup, nseg, planes_per_seg, queue, xch,
                       range, load_tilt(dir, d));
  } else {
    sweep3d_wave<T, R>(grid + (int64_t)blockIdx.y * N, D, H, W, N, nstrip, ngroup, nseg, planes_per_seg,
                       queue, xch, range, typename ModeTransform<MODE>::type());
  }
  __syncthreads();
  unsigned long long* out = hist + (int64_t)blockIdx.y * bins;
  for (int b = threadIdx.x; b < bins; b += 256) {
    const int v = lhist[b];
    if (v != 0) atomicAdd(&out[b], (unsigned long long)(long long)v);
  }
}

// Single-pass mode: critical vertices to the item's list, min / max to the header.
template <typename T, int R, int MODE>
__global__ __launch_bounds__(256) void sweep3d_list_kernel(const T* __restrict__ grid, int D, int H, int W,
                                                           int64_t N, int nstrip, int ngroup, int nseg,
                                                           int planes_per_seg, ListArgs la, DirArgs dir) {
  extern __shared__ int smem[];
  unsigned* xch = reinterpret_cast<unsigned*>(smem);
  uint2* qbuf = reinterpret_cast<uint2*>(smem + kXchInts) + (threadIdx.x >> 6) * kQueueCap;
  s3::TubeQueue<ListSink> queue;
  queue.buf = qbuf;
  queue.tbuf = reinterpret_cast<float*>(smem + kXchInts + 4 * kQueueCap * 2) + (threadIdx.x >> 6) * kQueueCap;
  queue.count = 0;
  __shared__ unsigned own[4];  // list per block: fill count, least / greatest key, overflow (never raised)
  if (la.heads) {              // (block-uniform)
    block_list_begin(la, queue.sink, own);
  } else {
    const unsigned sub = blockIdx.y * la.nsub + (blockIdx.x & (la.nsub - 1u));
    queue.sink.list = la.lists + (size_t)sub * la.cap;
    queue.sink.counter = la.counters + sub;
    queue.sink.overflow = &la.hdr->overflow;
  }
  queue.sink.cap = la.cap;
  WaveRange range;
  if constexpr (MODE == kTilted) {
    const int d = blockIdx.y / dir.batch, item = blockIdx.y - d * dir.batch;
    sweep3d_wave<T, R>(grid + (int64_t)item * N, D, H, W, N, nstrip, ngroup, nseg, planes_per_seg, queue, xch,
                       range, load_tilt(dir, d));
  } else {
    sweep3d_wave<T, R>(grid + (int64_t)blockIdx.y * N, D, H, W, N, nstrip, ngroup, nseg, planes_per_seg,
                       queue, xch, range, typename ModeTransform<MODE>::type());
  }
  if (la.heads) block_list_end(la, range, own);
  else range.commit(la.hdr);
}

// LV: the type also comes with one bin per level (uint8 / uint16 grids without a range)
template <typename T, bool LV = false>
static void launch3d_t(const void* grid, const Shape& s, bool levels, int bins, const HardHeader* hdr,
                       const float* table, unsigned long long* hist, hipStream_t st,
                       const unsigned* run_if, const DirArgs* dir, int conv) {
  constexpr int R = kRows3d;
  const Plan3d pl = plan3d<T>(s);
  const bool tlds = !levels && (size_t)bins * 8 + kFixedLds3d <= 60 * 1024;
  const size_t lds = kFixedLds3d + (size_t)bins * (tlds ? 8 : 4);
  const T* p = static_cast<const T*>(grid);
  const DirArgs none = {nullptr, 0.f, 1, 3};
#define ECC_GO(LV, TL, TI)                                                                                  \
  hipLaunchKernelGGL((sweep3d_kernel<T, R, LV, TL, TI>), pl.grid, dim3(256), lds, st, p, (int)s.D, (int)s.H, \
                     (int)s.W, s.N, bins, pl.nstrip, pl.ngroup, pl.nseg, pl.planes_per_seg, hdr, table,      \
                     hist, run_if, dir ? *dir : none)
  if constexpr (std::is_same<T, float>::value) {
    if (dir) {  // directional call: float grids, thresholds from a range
      if (tlds) ECC_GO(false, true, kTilted);
      else ECC_GO(false, false, kTilted);
      return;
    }
  }
#define ECC_MODE(M)                                  \
  do {                                               \
    if constexpr (LV) {                              \
      if (levels) { ECC_GO(true, false, M); break; } \
    }                                                \
    if (tlds) ECC_GO(false, true, M);                \
    else ECC_GO(false, false, M);                    \
  } while (0)
  switch (mode_of_conv(conv)) {
    case kTopCells: ECC_MODE(kTopCells); break;
    case kSuper: ECC_MODE(kSuper); break;
    case kTopSuper: ECC_MODE(kTopSuper); break;
    default: ECC_MODE(kPlain); break;
  }
#undef ECC_MODE
#undef ECC_GO
}

template <typename T>
static void launch3d_list_t(const void* grid, const Shape& s, const ListArgs& la, hipStream_t st, const DirArgs* dir,
                            int conv) {
  const Plan3d pl = plan3d<T>(s);
  const DirArgs none = {nullptr, 0.f, 1, 3};
  const T* p = static_cast<const T*>(grid);
#define ECC_LIST(M, DIR)                                                                                  \
  hipLaunchKernelGGL((sweep3d_list_kernel<T, kRows3d, M>), pl.grid, dim3(256), kFixedLds3d, st, p,   \
                     (int)s.D, (int)s.H, (int)s.W, s.N, pl.nstrip, pl.ngroup, pl.nseg, pl.planes_per_seg, la, \
                     DIR)
  if constexpr (std::is_same<T, float>::value) {
    if (dir) {
      ECC_LIST(kTilted, *dir);
      return;
    }
  }
  switch (mode_of_conv(conv)) {
    case kTopCells: ECC_LIST(kTopCells, none); break;
    case kSuper: ECC_LIST(kSuper, none); break;
    case kTopSuper: ECC_LIST(kTopSuper, none); break;
    default: ECC_LIST(kPlain, none); break;
  }
#undef ECC_LIST
}

// dtype: float32, float16 or bfloat16 (the floating types whose range is found on the device)
void launch_sweep3d_list(const void* grid, int dtype, const Shape& s, const ListArgs& la, hipStream_t st,
                         const DirArgs* dir, int conv) {
  switch (dtype) {
    case 3: launch3d_list_t<F16>(grid, s, la, st, nullptr, conv); break;
    case 6: launch3d_list_t<Bf16>(grid, s, la, st, nullptr, conv); break;
    default: launch3d_list_t<float>(grid, s, la, st, dir, conv); break;
  }
}

unsigned sweep3d_list_blocks(const Shape& s) { return plan3d<float>(s).grid.x; }
unsigned sweep3d_block_vertices(const Shape& s) {
  // four wave units of at most 62 columns x 4 rows (a folded unit: several row groups of fewer columns) x the segment's planes
  return 4u * (unsigned)s3::kOut * (unsigned)kRows3d * (unsigned)plan3d<float>(s).planes_per_seg;
}

bool sweep3d_supported(const Shape& s, int bins) {
  // 32-bit element offsets inside a chunk of up to 31 planes (and so one plane stays far
  // below the 2^31 bytes a buffer resource can span)
  return bins <= 10240 && s.ndim == 3 && s.D >= 2 && s.W >= 8 && s.W <= (1 << 22) && s.H <= (1 << 22) &&
         s.H * s.W * 32 < ((int64_t)1 << 32) && s.D <= (1 << 30);
}

void launch_sweep3d(const void* grid, const Shape& s, int dtype, bool levels, int bins,
                    const HardHeader* hdr, const float* table, unsigned long long* hist,
                    hipStream_t st, const unsigned* run_if, const DirArgs* dir, int conv) {
  switch (dtype) {
    case 0: launch3d_t<uint8_t, true>(grid, s, levels, bins, hdr, table, hist, st, run_if, nullptr, conv); break;
    case 1: launch3d_t<uint16_t, true>(grid, s, levels, bins, hdr, table, hist, st, run_if, nullptr, conv); break;
    case 3: launch3d_t<F16>(grid, s, false, bins, hdr, table, hist, st, run_if, nullptr, conv); break;
    case 6: launch3d_t<Bf16>(grid, s, false, bins, hdr, table, hist, st, run_if, nullptr, conv); break;
    case 7: launch3d_t<int16_t>(grid, s, false, bins, hdr, table, hist, st, run_if, nullptr, conv); break;
    default: launch3d_t<float>(grid, s, levels, bins, hdr, table, hist, st, run_if, dir, conv); break;
  }
}

// Coefficient map through the tube sweep: the critical vertices' c(p) written to an int8 map
// that the caller has cleared.  The same stencil, order and tie-break as every other
// tube-sweep kernel, made visible vertex by vertex.
struct CoeffSink3d {
  static constexpr bool kTrackRange = false;
  int8_t* out;    // this item's map
  int64_t plane;  // H * W
  int oz;         // first plane of the wave's segment
  __device__ __forceinline__ void take(int n, float, int c, unsigned inpl, unsigned zrel) {
    const int lane = threadIdx.x & (kWave - 1);
    if (lane < n) out[(int64_t)(oz + (int)zrel) * plane + inpl] = (int8_t)c;
  }
};

template <typename T, int R>
__global__ __launch_bounds__(256) void coeff3d_kernel(const T* __restrict__ grid, int D, int H, int W, int64_t N,
                                                      int nstrip, int ngroup, int nseg, int planes_per_seg,
                                                      int8_t* __restrict__ out) {
  extern __shared__ int smem[];
  unsigned* xch = reinterpret_cast<unsigned*>(smem);
  s3::TubeQueue<CoeffSink3d> queue;
  queue.buf = reinterpret_cast<uint2*>(smem + kXchInts) + (threadIdx.x >> 6) * kQueueCap;
  queue.tbuf = reinterpret_cast<float*>(smem + kXchInts + 4 * kQueueCap * 2) + (threadIdx.x >> 6) * kQueueCap;
  queue.count = 0;
  queue.sink.out = out + (int64_t)blockIdx.y * N;
  queue.sink.plane = (int64_t)H * W;
  const int unit = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int ox, oy;
  unit_origin3(unit, D, H, W, gridDim.y, planes_per_seg, R, ox, oy, queue.sink.oz);
  WaveRange range;
  sweep3d_wave<T, R>(grid + (int64_t)blockIdx.y * N, D, H, W, N, nstrip, ngroup, nseg, planes_per_seg, queue, xch,
                     range, NoTilt());
}

template <typename T>
static void launch_coeff3d_t(const void* grid, const Shape& s, int8_t* out, hipStream_t st) {
  const Plan3d pl = plan3d<T>(s);
  hipLaunchKernelGGL((coeff3d_kernel<T, kRows3d>), pl.grid, dim3(256), kFixedLds3d, st, static_cast<const T*>(grid),
                     (int)s.D, (int)s.H, (int)s.W, s.N, pl.nstrip, pl.ngroup, pl.nseg, pl.planes_per_seg, out);
}

void launch_coeff3d(const void* grid, const Shape& s, int dtype, int8_t* out, hipStream_t st) {
  switch (dtype) {
    case 0: launch_coeff3d_t<uint8_t>(grid, s, out, st); break;
    case 1: launch_coeff3d_t<uint16_t>(grid, s, out, st); break;
    default: launch_coeff3d_t<float>(grid, s, out, st); break;
  }
}

}  // namespace ecc
