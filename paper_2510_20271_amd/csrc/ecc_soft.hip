// Soft single-direction ECC on gfx950: forward (Eq. 6 of the paper) and the
// analytic derivatives (Eq. 8-10 of its appendix).
//
// Every term of Eq. 6 and Eq. 8-10 carries the integer factor c(p), so only
// vertices with c(p) != 0 contribute.  A block takes a tile of consecutive
// vertices, computes c(p) with the same stencil as the hard path, compacts the
// critical vertices (c != 0) into an LDS list in a fixed order, and then
// evaluates the sigmoid only on list x thresholds pairs:
//   - threshold-major loops (one thread per tau_j, running over the list)
//     give the sums over p of Eq. 6 / Eq. 9 / Eq. 10 without any cross-lane
//     reduction;
//   - a vertex-major loop (one thread per list entry, running over tau_j)
//     gives the contraction of Eq. 8 with the upstream gradient.
// Block partials go to the workspace and are combined by a second kernel in a
// fixed order in float64, so results are run-to-run identical.
//
// The sigmoid argument z = tau_j - X(p) - alpha <u,p> is formed in float64 and
// rounded once; exp2 and reciprocal run on the float32 transcendental unit.
#include "ecc_device.h"
#include "ecc_internal.h"

#include <algorithm>
#include <cstdlib>

namespace ecc {

constexpr int kSoftBlock = 256;
constexpr int kPerThread = 8;
constexpr int kTile = kSoftBlock * kPerThread;  // vertices per block

struct SoftList {
  double y[kTile];         // X(p) + alpha <u,p>
  float c[kTile];          // c(p) as float
  unsigned short loc[kTile];  // position of p inside the tile
};

__device__ __forceinline__ float exp_neg(float z, float kneg) {
  // exp(-lambda z) = 2^(kneg z); clamped so the result stays finite
  return __builtin_amdgcn_exp2f(fminf(kneg * z, 126.0f));
}

// Fill the list for this block's tile.  Returns the number of entries.  When
// zero_out != nullptr, vertices with c == 0 get 0 written there.  rel (may be
// null) receives the coordinates relative to the tile's first vertex.
// TILTC: c(p) is the coefficient of the tilted field (as the directional hard curves
// form it) instead of the field's own.
template <int ND, bool TILTC>
__device__ __forceinline__ int build_list(const float* __restrict__ g, int64_t D, int64_t H,
                                          int64_t W, int64_t N, int64_t tile0,
                                          const float* __restrict__ u, float alpha, SoftList& L,
                                          float (*rel)[kTile], float* __restrict__ zero_out,
                                          int* scratch /* kSoftBlock/64 + 1 ints */) {
  const int tid = threadIdx.x;
  int cs[kPerThread];
  int n = 0;
  Tilt tilt;
  if (TILTC) {
    const DirArgs da = {u, alpha, 1, ND};
    tilt = load_tilt(da, 0);
  }
#pragma unroll
  for (int k = 0; k < kPerThread; ++k) {
    const int64_t i = tile0 + k * kSoftBlock + tid;
    int c = 0;
    if (i < N) {
      const int64_t x = i % W, r = i / W;
      if (TILTC) c = coeff_tilted_at<ND>(g, tilt, D, H, W, r / H, r % H, x);
      else c = coeff_at<float, ND>(g, D, H, W, r / H, r % H, x);
      if (c == 0 && zero_out) zero_out[i] = 0.0f;
    }
    cs[k] = c;
    n += (c != 0);
  }
  // exclusive scan of n over the block: wave scan + wave totals
  int incl = n;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    int t = __shfl_up(incl, o);
    if ((tid & (kWave - 1)) >= o) incl += t;
  }
  const int wv = tid / kWave;
  if ((tid & (kWave - 1)) == kWave - 1) scratch[wv] = incl;
  __syncthreads();
  int base = 0, total = 0;
#pragma unroll
  for (int w = 0; w < kSoftBlock / kWave; ++w) {
    const int t = scratch[w];
    if (w < wv) base += t;
    total += t;
  }
  int pos = base + incl - n;
  const double ux = (double)u[0], uy = (double)u[1], uz = (ND == 3) ? (double)u[2] : 0.0;
  const int64_t x0 = tile0 % W, r0 = tile0 / W, y0 = r0 % H, z0 = r0 / H;
#pragma unroll
  for (int k = 0; k < kPerThread; ++k) {
    if (cs[k] != 0) {
      const int64_t i = tile0 + k * kSoftBlock + tid;
      const int64_t x = i % W, r = i / W, y = r % H, z = r / H;
      double dot = ux * (double)x + uy * (double)y;
      if (ND == 3) dot += uz * (double)z;
      L.y[pos] = (double)g[i] + (double)alpha * dot;
      L.c[pos] = (float)cs[k];
      L.loc[pos] = (unsigned short)(k * kSoftBlock + tid);
      if (rel) {
        rel[0][pos] = (float)(x - x0);
        rel[1][pos] = (float)(y - y0);
        if (ND == 3) rel[2][pos] = (float)(z - z0);
      }
      ++pos;
    }
  }
  __syncthreads();
  return total;
}

// ---------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------
template <int ND, bool TILTC>
__global__ __launch_bounds__(kSoftBlock) void soft_fwd_kernel(
    const float* __restrict__ grid, int64_t D, int64_t H, int64_t W, int64_t N,
    const float* __restrict__ u, float alpha, const float* __restrict__ tau, int T, float kneg,
    float* __restrict__ partial) {
  __shared__ SoftList L;
  __shared__ float red[kSoftBlock];
  __shared__ int scratch[kSoftBlock / kWave + 1];
  const float* g = grid + (int64_t)blockIdx.y * N;
  const int64_t tile0 = (int64_t)blockIdx.x * kTile;
  const int cnt = build_list<ND, TILTC>(g, D, H, W, N, tile0, u, alpha, L, nullptr, nullptr, scratch);
  float* out = partial + ((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * T;
  const int tid = threadIdx.x;
  for (int jc = 0; jc < T; jc += kSoftBlock) {
    const int Tc = min(kSoftBlock, T - jc);
    const int nparts = kSoftBlock / Tc;
    const int part = tid / Tc, jl = tid - part * Tc;
    float acc = 0.0f;
    if (part < nparts) {
      const double tj = (double)tau[jc + jl];
      for (int e = part; e < cnt; e += nparts) {
        const float z = (float)(tj - L.y[e]);
        const float ex = exp_neg(z, kneg);
        acc += L.c[e] * __builtin_amdgcn_rcpf(1.0f + ex);
      }
    }
    red[tid] = acc;
    __syncthreads();
    if (tid < Tc) {
      float s = 0.0f;
      for (int p = 0; p < nparts; ++p) s += red[p * Tc + tid];
      out[jc + tid] = s;
    }
    __syncthreads();
  }
}

__global__ void soft_fwd_reduce_kernel(const float* __restrict__ partial, int ntiles, int T,
                                       int64_t total /* batch*T */, float* __restrict__ chi) {
  const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= total) return;
  const int64_t item = k / T;
  const int j = (int)(k - item * T);
  const float* p = partial + item * ntiles * (int64_t)T + j;
  double s = 0.0;
  int t = 0;
  for (; t + 8 <= ntiles; t += 8) {  // eight loads in flight, added in tile order
    float v[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) v[q] = p[(int64_t)(t + q) * T];
#pragma unroll
    for (int q = 0; q < 8; ++q) s += (double)v[q];
  }
  for (; t < ntiles; ++t) s += (double)p[(int64_t)t * T];
  chi[k] = (float)s;
}

// ---------------------------------------------------------------------------
// backward
// ---------------------------------------------------------------------------
template <int ND, bool TILTC>
__global__ __launch_bounds__(kSoftBlock) void soft_bwd_kernel(
    const float* __restrict__ grid, int64_t D, int64_t H, int64_t W, int64_t N,
    const float* __restrict__ u, float alpha, const float* __restrict__ tau, int T, float kneg,
    float lambda, const float* __restrict__ gup /* [batch][T] or null */,
    float* __restrict__ grad_X /* or null */, float* __restrict__ partial /* or null */) {
  __shared__ SoftList L;
  __shared__ float rel[ND][kTile];
  __shared__ float red[1 + ND][kSoftBlock];
  __shared__ int scratch[kSoftBlock / kWave + 1];
  const float* g = grid + (int64_t)blockIdx.y * N;
  const int64_t tile0 = (int64_t)blockIdx.x * kTile;
  float* gx = grad_X ? grad_X + (int64_t)blockIdx.y * N : nullptr;
  const int cnt = build_list<ND, TILTC>(g, D, H, W, N, tile0, u, alpha, L, rel, gx, scratch);
  const int tid = threadIdx.x;

  if (gx) {  // Eq. 8 contracted with the upstream gradient, one thread per critical vertex
    const float* gj = gup ? gup + (int64_t)blockIdx.y * T : nullptr;
    for (int e = tid; e < cnt; e += kSoftBlock) {
      const double ye = L.y[e];
      float acc = 0.0f;
      for (int j = 0; j < T; ++j) {
        const float z = (float)((double)tau[j] - ye);
        const float ex = exp_neg(z, kneg);
        const float s = __builtin_amdgcn_rcpf(1.0f + ex);
        const float d = ex * s * s;  // sigma (1 - sigma)
        acc += (gj ? gj[j] : 1.0f) * d;
      }
      gx[tile0 + L.loc[e]] = -lambda * L.c[e] * acc;
    }
  }

  if (partial) {  // Eq. 9 and Eq. 10, one thread per threshold
    float* out = partial + ((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * (int64_t)T * 4;
    for (int jc = 0; jc < T; jc += kSoftBlock) {
      const int Tc = min(kSoftBlock, T - jc);
      const int nparts = kSoftBlock / Tc;
      const int part = tid / Tc, jl = tid - part * Tc;
      float a0 = 0.0f, a[ND];
#pragma unroll
      for (int k = 0; k < ND; ++k) a[k] = 0.0f;
      if (part < nparts) {
        const double tj = (double)tau[jc + jl];
        for (int e = part; e < cnt; e += nparts) {
          const float z = (float)(tj - L.y[e]);
          const float ex = exp_neg(z, kneg);
          const float s = __builtin_amdgcn_rcpf(1.0f + ex);
          const float cd = L.c[e] * (ex * s * s);
          a0 += cd;
#pragma unroll
          for (int k = 0; k < ND; ++k) a[k] += cd * rel[k][e];
        }
      }
      red[0][tid] = a0;
#pragma unroll
      for (int k = 0; k < ND; ++k) red[1 + k][tid] = a[k];
      __syncthreads();
      if (tid < Tc) {
#pragma unroll
        for (int q = 0; q < 1 + ND; ++q) {
          float s = 0.0f;
          for (int p = 0; p < nparts; ++p) s += red[q][p * Tc + tid];
          out[(int64_t)(jc + tid) * 4 + q] = s;
        }
      }
      __syncthreads();
    }
  }
}

// dchi_dtau = lambda * sum A0;  dchi_du_k = -alpha lambda * sum (o_k A0 + A_k),
// o = coordinates of the tile's first vertex.
__global__ void soft_bwd_reduce_kernel(const float* __restrict__ partial, int ntiles, int T,
                                       int64_t total, int nd, int64_t H, int64_t W, float alpha,
                                       float lambda, float* __restrict__ dtau,
                                       float* __restrict__ du) {
  const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= total) return;
  const int64_t item = k / T;
  const int j = (int)(k - item * T);
  const float* p = partial + (item * ntiles * (int64_t)T + j) * 4;
  double s0 = 0.0, s[3] = {0.0, 0.0, 0.0};
  auto add = [&](int t, const float4& e) {
    const int64_t i0 = (int64_t)t * kTile;
    const int64_t r0 = i0 / W;
    const double o[3] = {(double)(i0 % W), (double)(r0 % H), (double)(r0 / H)};
    const float q[3] = {e.y, e.z, e.w};
    const double a0 = (double)e.x;
    s0 += a0;
    for (int c = 0; c < nd; ++c) s[c] += o[c] * a0 + (double)q[c];
  };
  const float4* p4 = reinterpret_cast<const float4*>(p);
  int t = 0;
  for (; t + 8 <= ntiles; t += 8) {  // eight loads in flight, added in tile order
    float4 v[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) v[q] = p4[(int64_t)(t + q) * T];
#pragma unroll
    for (int q = 0; q < 8; ++q) add(t + q, v[q]);
  }
  for (; t < ntiles; ++t) add(t, p4[(int64_t)t * T]);
  if (dtau) dtau[k] = (float)((double)lambda * s0);
  if (du)
    for (int c = 0; c < nd; ++c) du[k * nd + c] = (float)(-(double)alpha * (double)lambda * s[c]);
}

// ---------------------------------------------------------------------------
// grad_X of the fused paths is zero away from the critical vertices: cleared by a
// fill kernel of its own (a captured graph may hold it, unlike a memset node)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void clear_f32_kernel(float4* __restrict__ p, int64_t n4, float* __restrict__ tail,
                                                        int ntail) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  if (blockIdx.x == 0 && (int)threadIdx.x < ntail) tail[threadIdx.x] = 0.f;
}

void launch_clear_f32(float* p, int64_t total, hipStream_t st) {
  // p is only known to be 4-byte aligned: whole float4s from the first 16-byte boundary on,
  // the few elements before and after by the first threads (two launches at most)
  const uintptr_t a = reinterpret_cast<uintptr_t>(p);
  int64_t lead = (int64_t)(((16 - (a & 15)) & 15) / 4);
  if (lead > total) lead = total;
  const int64_t n4 = (total - lead) / 4;
  const int64_t rest = total - lead - n4 * 4;
  int64_t nb = (n4 + 255) / 256;
  nb = nb < 1 ? 1 : (nb > 4096 ? 4096 : nb);
  if (lead)
    hipLaunchKernelGGL(clear_f32_kernel, dim3(1), dim3(256), 0, st, (float4*)nullptr, (int64_t)0, p, (int)lead);
  hipLaunchKernelGGL(clear_f32_kernel, dim3((unsigned)nb), dim3(256), 0, st, reinterpret_cast<float4*>(p + lead), n4,
                     p + lead + n4 * 4, (int)rest);
}

// ---------------------------------------------------------------------------
// host launchers
// ---------------------------------------------------------------------------
static int64_t tiles_of(const Shape& s) { return (s.N + kTile - 1) / kTile; }

size_t soft_workspace_bytes(const Shape& s, int T) {
  const size_t a = (size_t)256 + (size_t)s.batch * (size_t)tiles_of(s) * (size_t)T * 4 * sizeof(float);
  const size_t b = soft2d_workspace_bytes(s, T), c = soft3d_workspace_bytes(s, T);
  return std::max(a, std::max(b, c));
}

// test aid (ecc_debug_force): the tile kernels of this file for every shape
static bool use_soft2d(const Shape& s, int T) {
  return !(forced_paths() & kForceSoftTiles) && soft2d_supported(s, T);
}

static bool use_soft3d(const Shape& s, int T) {
  return !(forced_paths() & kForceSoftTiles) && soft3d_supported(s, T);
}

static float kneg_of(float lambda) { return (float)(-(double)lambda * 1.4426950408889634); }

hipError_t launch_soft_fwd(const float* grid, const Shape& s, const float* u, float alpha,
                           const float* tau, int T, float lambda, float* chi, void* ws,
                           hipStream_t st, bool tiltc) {
  if (use_soft2d(s, T)) {
    launch_soft2d_fwd(grid, s, u, alpha, tau, T, lambda, chi, ws, st, tiltc);
    return hipGetLastError();
  }
  if (use_soft3d(s, T)) {
    launch_soft3d_fwd(grid, s, u, alpha, tau, T, lambda, chi, ws, st, tiltc);
    return hipGetLastError();
  }
  float* partial = static_cast<float*>(ws);
  const int ntiles = (int)tiles_of(s);
  dim3 g((unsigned)ntiles, (unsigned)s.batch);
#define ECC_GO(ND, TC)                                                                                  \
  hipLaunchKernelGGL((soft_fwd_kernel<ND, TC>), g, dim3(kSoftBlock), 0, st, grid, s.D, s.H, s.W, s.N, u, \
                     alpha, tau, T, kneg_of(lambda), partial)
  if (s.ndim == 2) { if (tiltc) ECC_GO(2, true); else ECC_GO(2, false); }
  else             { if (tiltc) ECC_GO(3, true); else ECC_GO(3, false); }
#undef ECC_GO
  const int64_t total = s.batch * T;
  hipLaunchKernelGGL(soft_fwd_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                     st, partial, ntiles, T, total, chi);
  return hipGetLastError();
}

hipError_t launch_soft_bwd(const float* grid, const Shape& s, const float* u, float alpha,
                           const float* tau, int T, float lambda, const float* gup, float* grad_X,
                           float* dtau, float* du, void* ws, hipStream_t st, bool tiltc) {
  if (use_soft2d(s, T)) {
    launch_soft2d_bwd(grid, s, u, alpha, tau, T, lambda, gup, grad_X, dtau, du, ws, st, tiltc);
    return hipGetLastError();
  }
  if (use_soft3d(s, T)) {
    launch_soft3d_bwd(grid, s, u, alpha, tau, T, lambda, gup, grad_X, dtau, du, ws, st, tiltc);
    return hipGetLastError();
  }
  float* partial = (dtau || du) ? static_cast<float*>(ws) : nullptr;
  const int ntiles = (int)tiles_of(s);
  dim3 g((unsigned)ntiles, (unsigned)s.batch);
#define ECC_GO(ND, TC)                                                                                  \
  hipLaunchKernelGGL((soft_bwd_kernel<ND, TC>), g, dim3(kSoftBlock), 0, st, grid, s.D, s.H, s.W, s.N, u, \
                     alpha, tau, T, kneg_of(lambda), lambda, gup, grad_X, partial)
  if (s.ndim == 2) { if (tiltc) ECC_GO(2, true); else ECC_GO(2, false); }
  else             { if (tiltc) ECC_GO(3, true); else ECC_GO(3, false); }
#undef ECC_GO
  if (partial) {
    const int64_t total = s.batch * T;
    hipLaunchKernelGGL(soft_bwd_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       st, partial, ntiles, T, total, s.ndim, s.H, s.W, alpha, lambda, dtau, du);
  }
  return hipGetLastError();
}

// ---- forward pass that saves its critical vertices, backward pass that reuses them ---------------
size_t soft_state_bytes(const Shape& s) { return s.ndim == 3 ? soft3d_state_bytes(s) : soft2d_state_bytes(s); }

hipError_t launch_soft_fwd_save(const float* grid, const Shape& s, const float* u, float alpha, const float* tau,
                                int T, float lambda, float* chi, float* dtau, float* du, void* state, void* ws,
                                hipStream_t st, bool tiltc) {
  if (use_soft2d(s, T)) {
    launch_soft2d_fwd_save(grid, s, u, alpha, tau, T, lambda, chi, dtau, du, state, ws, st, tiltc);
    return hipGetLastError();
  }
  if (use_soft3d(s, T) && soft3d_state_supported(s, T)) {
    launch_soft3d_fwd_save(grid, s, u, alpha, tau, T, lambda, chi, dtau, du, state, ws, st, tiltc);
    return hipGetLastError();
  }
  // other shapes keep no state: the forward pass, then the threshold / direction sums of the backward one
  hipError_t e = launch_soft_fwd(grid, s, u, alpha, tau, T, lambda, chi, ws, st, tiltc);
  if (e == hipSuccess && (dtau || du))
    e = launch_soft_bwd(grid, s, u, alpha, tau, T, lambda, nullptr, nullptr, dtau, du, ws, st, tiltc);
  return e;
}

hipError_t launch_soft_bwd_saved(const float* grid, const Shape& s, const float* u, float alpha, const float* tau,
                                 int T, float lambda, const float* gup, float* grad_X, const void* state, void* ws,
                                 hipStream_t st, bool tiltc) {
  if (use_soft2d(s, T)) {
    launch_soft2d_bwd_saved(grid, s, u, alpha, tau, T, lambda, gup, grad_X, state, st, tiltc);
    return hipGetLastError();
  }
  if (use_soft3d(s, T) && soft3d_state_supported(s, T)) {
    launch_soft3d_bwd_saved(grid, s, u, alpha, tau, T, lambda, gup, grad_X, state, st, tiltc);
    return hipGetLastError();
  }
  return launch_soft_bwd(grid, s, u, alpha, tau, T, lambda, gup, grad_X, nullptr, nullptr, ws, st, tiltc);
}

}  // namespace ecc
