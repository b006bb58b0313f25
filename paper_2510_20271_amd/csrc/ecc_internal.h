// Host-side internal interface between the C-ABI layer (ecc_api.hip) and the
// kernel launchers (ecc_hard.hip, ecc_soft.hip).  Arguments are already
// validated when these are called.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace ecc {

struct Shape {
  int ndim;          // 2 or 3
  int64_t D, H, W;   // D == 1 for 2D
  int64_t N;         // D*H*W
  int64_t batch;
};

// ---- hard path ------------------------------------------------------------
// convention bits (`conv` below): bit 0 top-cell construction (grid points are squares /
// cubes) instead of the vertex one, bit 1 superlevel sets instead of sublevel sets
constexpr int kConvTop = 1, kConvSuper = 2;
size_t hard_workspace_bytes(const Shape& s, int bins);
struct DirArgs;  // directional launch (tilted field, blockIdx.y over directions x items); null: plain
// dtype: any ecc_dtype code; f32_scratch: room for a float32 copy of the grid (codes 3..7 only)
// roomy: ws holds hard_workspace_bytes(); otherwise hard_workspace_min_bytes() (no list per block)
size_t hard_workspace_min_bytes(const Shape& s, int bins);
hipError_t launch_hard(const void* grid, const Shape& s, int dtype, int bins, bool have_range,
                       double lo, double hi, int64_t* curve, void* ws, hipStream_t st,
                       const DirArgs* dir = nullptr, int conv = 0, float* f32_scratch = nullptr, bool roomy = true);
// directional curves; sv: the shape with batch = directions x items, batch: items per direction
size_t hard_dir_workspace_bytes(const Shape& sv, int bins);
hipError_t launch_hard_dir(const float* grid, const Shape& sv, const float* u, float alpha, int batch,
                           int bins, bool have_range, double lo, double hi, int64_t* curve, void* ws,
                           hipStream_t st);
// element types beyond uint8 / uint16 / float32 (codes 3..7 of ecc_dtype): n elements rounded to float32
hipError_t launch_convert(const void* grid, int dtype, int64_t n, float* out, hipStream_t st);
hipError_t launch_coeff(const void* grid, const Shape& s, int dtype, int8_t* c_out, hipStream_t st);
// *count = number of NaN / Inf among n elements of type `dtype` (any ecc_dtype code)
hipError_t launch_count_nonfinite(const void* grid, int64_t n, int dtype, unsigned long long* count, hipStream_t st);
// the coefficient map through the strip / tube sweep (the map must have been cleared)
void launch_coeff2d(const void* grid, const Shape& s, int dtype, int8_t* c_out, hipStream_t st);
void launch_coeff3d(const void* grid, const Shape& s, int dtype, int8_t* c_out, hipStream_t st);

// Paths forced by ecc_debug_force (bits ECC_FORCE_* of include/ecc.h); 0 in normal operation.
constexpr unsigned kForceGeneric = 1u, kForceTwoPass = 2u, kForceSoftTiles = 4u, kForceNoSmall = 8u;
unsigned forced_paths();

// fast sweeps (one wave per column strip / tube, bit-sliced stencil)
struct HardHeader;
// small float32 inputs without a range: the whole call in two launches (ecc_small.hip);
// `small`: small_workspace_bytes(s) bytes behind the threshold table
bool small_supported(const Shape& s, int bins);
size_t small_workspace_bytes(const Shape& s);
void launch_scan(int64_t* curve, const Shape& s, int bins, int suffix, hipStream_t st);  // in-place prefix / suffix sums
// Mid-sized float grids without a range: the strip / tube sweep with a list per block, then the
// finishing kernel of the small flow and the scan (three launches, nothing cleared beforehand).
// `room`: mid_workspace_bytes() bytes behind the threshold table.
bool mid_supported(const Shape& s, int bins, int dtype);
size_t mid_workspace_bytes(const Shape& s, int dtype);
// dir (may be null): a directional call, s.batch = directions x items
hipError_t launch_hard_mid(const void* grid, const Shape& s, int dtype, int bins, int64_t* curve, HardHeader* hdr,
                           float* table, void* room, hipStream_t st, int conv, const DirArgs* dir);
hipError_t launch_hard_small(const float* grid, const Shape& s, int bins, int64_t* curve, HardHeader* hdr, float* table,
                             void* small, hipStream_t st, int conv);
// single-pass mode: per-item lists of critical vertices (value, c) in the workspace
// what a block that keeps a list of its own leaves behind (nothing has to be cleared for it)
struct ListHead {
  unsigned count;             // critical vertices the block found
  unsigned min_key, max_key;  // float_key of the least / greatest value the block saw
  unsigned pad;
};
struct ListArgs {
  float2* lists;       // [batch][nsub][cap]
  unsigned* counters;  // [batch][nsub]
  unsigned cap;        // entries per sub-list
  unsigned nsub;       // sub-lists per item, a power of two
  HardHeader* hdr;
  // Lists per block (heads != null): block (x, y) of the sweep appends to lists[(y gridDim.x + x) cap ..],
  // which has room for every vertex the block owns, and leaves its count and value range in
  // heads[y gridDim.x + x]; counters, nsub and hdr are unused.  The item's blocks also clear its
  // histogram zero_hist[y bins ..].
  ListHead* heads;
  unsigned long long* zero_hist;
  int bins;
};
bool sweep2d_supported(const Shape& s, int bins);
void launch_sweep2d(const void* grid, const Shape& s, int dtype, bool levels, int bins,
                    const HardHeader* hdr, const float* table, unsigned long long* hist,
                    hipStream_t st, const unsigned* run_if, const DirArgs* dir = nullptr, int conv = 0);
void launch_sweep2d_list(const void* grid, int dtype, const Shape& s, const ListArgs& la, hipStream_t st,
                         const DirArgs* dir = nullptr, int conv = 0);
unsigned sweep2d_list_blocks(const Shape& s, int dtype);  // blocks per item of that launch
unsigned sweep2d_block_vertices(const Shape& s, int dtype);  // most vertices a block of that launch owns

bool sweep3d_supported(const Shape& s, int bins);
void launch_sweep3d(const void* grid, const Shape& s, int dtype, bool levels, int bins,
                    const HardHeader* hdr, const float* table, unsigned long long* hist,
                    hipStream_t st, const unsigned* run_if, const DirArgs* dir = nullptr, int conv = 0);
void launch_sweep3d_list(const void* grid, int dtype, const Shape& s, const ListArgs& la, hipStream_t st,
                         const DirArgs* dir = nullptr, int conv = 0);
unsigned sweep3d_list_blocks(const Shape& s);
unsigned sweep3d_block_vertices(const Shape& s);

// ---- sweep-kernel timing (measurement aid) ----------------------------------
hipError_t profile_begin(int max_launches);
hipError_t profile_end(float* mean_ms, int* launches);
void profile_mark(hipStream_t st, bool after);  // no-op unless recording

// ---- soft path ------------------------------------------------------------
// tiltc: c(p) is the coefficient of the tilted field X + alpha <u,p> (formed as the
// directional hard curves form it) instead of the coefficient of X
size_t soft_workspace_bytes(const Shape& s, int T);
hipError_t launch_soft_fwd(const float* grid, const Shape& s, const float* u, float alpha,
                           const float* tau, int T, float lambda, float* chi, void* ws,
                           hipStream_t st, bool tiltc = false);
hipError_t launch_soft_bwd(const float* grid, const Shape& s, const float* u, float alpha,
                           const float* tau, int T, float lambda, const float* g, float* grad_X,
                           float* dtau, float* du, void* ws, hipStream_t st, bool tiltc = false);

void launch_clear_f32(float* p, int64_t n, hipStream_t st);  // p[0..n) = 0 (fill kernel)

// ---- soft path with state saved for the backward pass --------------------------------
// The forward pass leaves the critical vertices it found -- (y = X(p) + alpha <u,p>, position,
// c(p)) -- in a caller-owned state buffer, one list per wave unit of its sweep (filled in sweep
// order without atomics, so the contents are the same on every run), with the per-unit counts
// and a header naming the shape and plan.  The backward pass for grad_X then runs over those
// lists alone: no second sweep of the grid.  Layout: header | overflow flags [batch] | counts
// [batch][units] | entries [batch][units][cap].
struct SavedEntry {
  double y;  // X(p) + alpha <u,p>
  int idx;   // linear index of p inside its item
  int c;
};
struct SoftStateHeader {
  unsigned magic;
  int D, H, W, batch, nstrip, nseg, rows_per_seg, units, tiltc;  // (3D: rows_per_seg holds the planes per segment)
  unsigned cap;  // entries per unit
};
constexpr unsigned kSoftStateMagic = 0x45434353u;
size_t soft_state_bytes(const Shape& s);  // 256 when no shape-specific state is kept
// chi always; dtau / du may be null.  state: soft_state_bytes(s) bytes.
hipError_t launch_soft_fwd_save(const float* grid, const Shape& s, const float* u, float alpha, const float* tau,
                                int T, float lambda, float* chi, float* dtau, float* du, void* state, void* ws,
                                hipStream_t st, bool tiltc);
hipError_t launch_soft_bwd_saved(const float* grid, const Shape& s, const float* u, float alpha, const float* tau,
                                 int T, float lambda, const float* gup, float* grad_X, const void* state, void* ws,
                                 hipStream_t st, bool tiltc);
// fused 2D implementation of the two (shapes soft2d_supported takes)
size_t soft2d_state_bytes(const Shape& s);
void launch_soft2d_fwd_save(const float* grid, const Shape& s, const float* u, float alpha, const float* tau, int T,
                            float lambda, float* chi, float* dtau, float* du, void* state, void* ws, hipStream_t st,
                            bool tiltc);
void launch_soft2d_bwd_saved(const float* grid, const Shape& s, const float* u, float alpha, const float* tau, int T,
                             float lambda, const float* gup, float* grad_X, const void* state, hipStream_t st,
                             bool tiltc);

// fused 3D implementation of the two (volumes of fewer than 2^31 vertices that soft3d_supported takes)
bool soft3d_state_supported(const Shape& s, int T);
size_t soft3d_state_bytes(const Shape& s);
void launch_soft3d_fwd_save(const float* grid, const Shape& s, const float* u, float alpha, const float* tau, int T,
                            float lambda, float* chi, float* dtau, float* du, void* state, void* ws, hipStream_t st,
                            bool tiltc);
void launch_soft3d_bwd_saved(const float* grid, const Shape& s, const float* u, float alpha, const float* tau, int T,
                             float lambda, const float* gup, float* grad_X, const void* state, hipStream_t st,
                             bool tiltc);

// fused 2D soft path (strip sweep + sigmoid sinks)
bool soft2d_supported(const Shape& s, int T);
size_t soft2d_workspace_bytes(const Shape& s, int T);
void launch_soft2d_fwd(const float* grid, const Shape& s, const float* u, float alpha, const float* tau,
                       int T, float lambda, float* chi, void* ws, hipStream_t st, bool tiltc = false);
void launch_soft2d_bwd(const float* grid, const Shape& s, const float* u, float alpha, const float* tau,
                       int T, float lambda, const float* gup, float* grad_X, float* dtau, float* du,
                       void* ws, hipStream_t st, bool tiltc = false);

// fused 3D soft path (tube sweep + sigmoid sinks)
bool soft3d_supported(const Shape& s, int T);
size_t soft3d_workspace_bytes(const Shape& s, int T);
void launch_soft3d_fwd(const float* grid, const Shape& s, const float* u, float alpha, const float* tau,
                       int T, float lambda, float* chi, void* ws, hipStream_t st, bool tiltc = false);
void launch_soft3d_bwd(const float* grid, const Shape& s, const float* u, float alpha, const float* tau,
                       int T, float lambda, const float* gup, float* grad_X, float* dtau, float* du,
                       void* ws, hipStream_t st, bool tiltc = false);

}  // namespace ecc
