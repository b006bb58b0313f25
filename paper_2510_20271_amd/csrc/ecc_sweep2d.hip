// Hard ECC, 2D: kernels and launchers around the strip sweep of ecc_sweep2d.h.
#include "ecc_sweep2d.h"

#include <type_traits>

namespace ecc {

// Histogram mode: critical vertices are binned into the block's LDS histogram,
// which is merged into the global one at the end.  run_if (may be null): the
// kernel does nothing unless *run_if != 0 (fallback of the single-pass mode).
// MODE (SweepMode): kTilted is a directional launch (blockIdx.y = direction * batch + item,
// tilted field), kTopCells the top-cell construction, kSuper / kTopSuper the two
// constructions on superlevel sets.
template <typename T, bool LEVELS, bool TLDS, int MODE>
__global__ __launch_bounds__(256) void sweep2d_kernel(
    const T* __restrict__ grid, int H, int W, int64_t N, int bins, int nstrip, int nseg, int rows_per_seg,
    const HardHeader* __restrict__ hdr, const float* __restrict__ table,
    unsigned long long* __restrict__ hist, const unsigned* __restrict__ run_if, DirArgs dir) {
  if (run_if && *run_if == 0) return;
  extern __shared__ int smem[];
  // [4 waves][kChunkRows][64][kNC] floats of value ring, [4 waves] queues, histogram, table
  const int wv = threadIdx.x >> 6;
  float* ring = reinterpret_cast<float*>(smem) + wv * (kChunkRows * kWave * kNC);
  float2* qbuf = reinterpret_cast<float2*>(smem + 4 * kChunkRows * kWave * kNC) + wv * kQueueCap;
  int* lhist = smem + 4 * kChunkRows * kWave * kNC + 4 * kQueueCap * 2;
  float* ltable = reinterpret_cast<float*>(lhist + bins);
  for (int b = threadIdx.x; b < bins; b += 256) {
    lhist[b] = 0;
    if (TLDS) ltable[b] = table[b];
  }
  __syncthreads();
  WaveQueue<HistSink<LEVELS, mode_is_super(MODE)>> queue;
  queue.buf = qbuf;
  queue.count = 0;
  queue.sink.lhist = lhist;
  queue.sink.table = TLDS ? ltable : table;
  queue.sink.bins = bins;
  queue.sink.lo = LEVELS ? 0.f : hdr->lo;
  queue.sink.scale = LEVELS ? 0.f : hdr->scale;
  WaveRange range;
  if constexpr (MODE == kTilted) {
    const int d = blockIdx.y / dir.batch, item = blockIdx.y - d * dir.batch;
    sweep2d_wave<T>(grid + (int64_t)item * N, H, W, N, nstrip, nseg, rows_per_seg, queue, ring, range,
                    load_tilt(dir, d));
  } else {
    sweep2d_wave<T>(grid + (int64_t)blockIdx.y * N, H, W, N, nstrip, nseg, rows_per_seg, queue, ring, range,
                    typename ModeTransform<MODE>::type());
  }
  __syncthreads();
  unsigned long long* out = hist + (int64_t)blockIdx.y * bins;
  for (int b = threadIdx.x; b < bins; b += 256) {
    const int v = lhist[b];
    if (v != 0) atomicAdd(&out[b], (unsigned long long)(long long)v);
  }
}

// Single-pass mode: critical vertices (value, c) go to the item's list in the
// workspace and the wave's min / max to the header; the bins are assigned later,
// once the batch-global range is known.
template <typename T, int MODE>
__global__ __launch_bounds__(256) void sweep2d_list_kernel(const T* __restrict__ grid, int H, int W,
                                                           int64_t N, int nstrip, int nseg,
                                                           int rows_per_seg, ListArgs la, DirArgs dir) {
  extern __shared__ int smem[];
  const int wv = threadIdx.x >> 6;
  float* ring = reinterpret_cast<float*>(smem) + wv * (kChunkRows * kWave * kNC);
  float2* qbuf = reinterpret_cast<float2*>(smem + 4 * kChunkRows * kWave * kNC) + wv * kQueueCap;
  WaveQueue<ListSink> queue;
  queue.buf = qbuf;
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
    sweep2d_wave<T>(grid + (int64_t)item * N, H, W, N, nstrip, nseg, rows_per_seg, queue, ring, range,
                    load_tilt(dir, d));
  } else {
    sweep2d_wave<T>(grid + (int64_t)blockIdx.y * N, H, W, N, nstrip, nseg, rows_per_seg, queue, ring, range,
                    typename ModeTransform<MODE>::type());
  }
  if (la.heads) block_list_end(la, range, own);
  else range.commit(la.hdr);
}

constexpr size_t kRingBytes2d = ring_bytes2d<float2>();

// LV: the type also comes with one bin per level (uint8 / uint16 grids without a range)
template <typename T, bool LV = false>
static void launch2d_t(const void* grid, const Shape& s, bool levels, int bins, const HardHeader* hdr,
                       const float* table, unsigned long long* hist, hipStream_t st,
                       const unsigned* run_if, const DirArgs* dir, int conv) {
  const Plan2d pl = plan2d<T>(s);
  const bool tlds = !levels && (size_t)bins * 8 + kRingBytes2d <= 64 * 1024;
  const size_t lds = kRingBytes2d + (size_t)bins * (tlds ? 8 : 4);
  const T* p = static_cast<const T*>(grid);
  const DirArgs none = {nullptr, 0.f, 1, 2};
#define ECC_GO(LV, TL, TI)                                                                                \
  hipLaunchKernelGGL((sweep2d_kernel<T, LV, TL, TI>), pl.grid, dim3(256), lds, st, p, (int)s.H, (int)s.W, \
                     s.N, bins, pl.nstrip, pl.nseg, pl.rows_per_seg, hdr, table, hist, run_if,           \
                     dir ? *dir : none)
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
static void launch2d_list_t(const void* grid, const Shape& s, const ListArgs& la, hipStream_t st, const DirArgs* dir,
                            int conv) {
  const Plan2d pl = plan2d<T>(s);
  const DirArgs none = {nullptr, 0.f, 1, 2};
  const T* p = static_cast<const T*>(grid);
#define ECC_LIST(M, DIR)                                                                                 \
  hipLaunchKernelGGL((sweep2d_list_kernel<T, M>), pl.grid, dim3(256), kRingBytes2d, st, p, (int)s.H, \
                     (int)s.W, s.N, pl.nstrip, pl.nseg, pl.rows_per_seg, la, DIR)
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
void launch_sweep2d_list(const void* grid, int dtype, const Shape& s, const ListArgs& la, hipStream_t st,
                         const DirArgs* dir, int conv) {
  switch (dtype) {
    case 3: launch2d_list_t<F16>(grid, s, la, st, nullptr, conv); break;
    case 6: launch2d_list_t<Bf16>(grid, s, la, st, nullptr, conv); break;
    default: launch2d_list_t<float>(grid, s, la, st, dir, conv); break;
  }
}

unsigned sweep2d_block_vertices(const Shape& s, int dtype) {
  const Plan2d pl = dtype == 2 ? plan2d<float>(s) : plan2d<F16>(s);
  return 4u * (unsigned)kStripOut * (unsigned)pl.rows_per_seg;  // four wave units of 248 columns x the segment's rows
}

unsigned sweep2d_list_blocks(const Shape& s, int dtype) {
  return dtype == 2 ? plan2d<float>(s).grid.x : plan2d<F16>(s).grid.x;
}

bool sweep2d_supported(const Shape& s, int bins) {
  // value ring (32 KiB) + queues (4 KiB) + histogram must fit the 64 KiB of LDS a block may ask for
  return bins <= 7168 && s.D == 1 && s.W >= 8 && s.W <= (1 << 22) && s.H <= (1 << 30);
}

void launch_sweep2d(const void* grid, const Shape& s, int dtype, bool levels, int bins,
                    const HardHeader* hdr, const float* table, unsigned long long* hist,
                    hipStream_t st, const unsigned* run_if, const DirArgs* dir, int conv) {
  switch (dtype) {
    case 0: launch2d_t<uint8_t, true>(grid, s, levels, bins, hdr, table, hist, st, run_if, nullptr, conv); break;
    case 1: launch2d_t<uint16_t, true>(grid, s, levels, bins, hdr, table, hist, st, run_if, nullptr, conv); break;
    case 3: launch2d_t<F16>(grid, s, false, bins, hdr, table, hist, st, run_if, nullptr, conv); break;
    case 6: launch2d_t<Bf16>(grid, s, false, bins, hdr, table, hist, st, run_if, nullptr, conv); break;
    case 7: launch2d_t<int16_t>(grid, s, false, bins, hdr, table, hist, st, run_if, nullptr, conv); break;
    default: launch2d_t<float>(grid, s, levels, bins, hdr, table, hist, st, run_if, dir, conv); break;
  }
}

// Coefficient map through the strip sweep: the critical vertices' c(p) written to an int8
// map that the caller has cleared (every other vertex has c = 0).  The same stencil, order
// and tie-break as every other strip-sweep kernel, made visible vertex by vertex.
struct CoeffSink2d {
  typedef int4 Entry;  // (column, row, c, -)
  static constexpr bool kTrackRange = false;
  static constexpr bool kZeroFill = false;
  int8_t* out;  // this item's map
  int W;
  static __device__ __forceinline__ Entry make(float, int c, int col, int row) { return make_int4(col, row, c, 0); }
  __device__ __forceinline__ void consume(const Entry* buf, int n) {
    const int lane = threadIdx.x & (kWave - 1);
    if (lane >= n) return;
    const Entry e = buf[lane];
    out[(int64_t)e.y * W + e.x] = (int8_t)e.z;
  }
};

template <typename T>
__global__ __launch_bounds__(256) void coeff2d_kernel(const T* __restrict__ grid, int H, int W, int64_t N,
                                                      int nstrip, int nseg, int rows_per_seg,
                                                      int8_t* __restrict__ out) {
  extern __shared__ int smem[];
  const int wv = threadIdx.x >> 6;
  float* ring = reinterpret_cast<float*>(smem) + wv * (kChunkRows * kWave * kNC);
  int4* qbuf = reinterpret_cast<int4*>(smem + 4 * kChunkRows * kWave * kNC) + wv * kQueueCap;
  WaveQueue<CoeffSink2d> queue;
  queue.buf = qbuf;
  queue.count = 0;
  queue.sink.out = out + (int64_t)blockIdx.y * N;
  queue.sink.W = W;
  WaveRange range;
  sweep2d_wave<T>(grid + (int64_t)blockIdx.y * N, H, W, N, nstrip, nseg, rows_per_seg, queue, ring, range, NoTilt());
}

template <typename T>
static void launch_coeff2d_t(const void* grid, const Shape& s, int8_t* out, hipStream_t st) {
  const Plan2d pl = plan2d<T>(s);
  hipLaunchKernelGGL((coeff2d_kernel<T>), pl.grid, dim3(256), ring_bytes2d<int4>(), st, static_cast<const T*>(grid),
                     (int)s.H, (int)s.W, s.N, pl.nstrip, pl.nseg, pl.rows_per_seg, out);
}

void launch_coeff2d(const void* grid, const Shape& s, int dtype, int8_t* out, hipStream_t st) {
  switch (dtype) {
    case 0: launch_coeff2d_t<uint8_t>(grid, s, out, st); break;
    case 1: launch_coeff2d_t<uint16_t>(grid, s, out, st); break;
    default: launch_coeff2d_t<float>(grid, s, out, st); break;
  }
}

}  // namespace ecc
