// C ABI of libecc_hip: argument validation (host only, before any HIP call),
// error strings, dispatch to the kernel launchers.
#include "../../include/ecc.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>

#include <atomic>
#include <mutex>

#include "ecc_internal.h"

// Scratch of ecc_hard_static: device memory that belongs to the library, one copy per GPU,
// held until the process ends.  In host code the name is only a handle for
// hipGetSymbolAddress; kernels are given the address that call returns.
static __device__ __align__(256) unsigned char scratch[ECC_STATIC_SCRATCH_BYTES];

namespace {

std::atomic<unsigned> g_forced{0u};

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};  // address of `scratch` on each device, looked up once

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

constexpr int64_t kMaxBatch = 65535;            // batch rides on gridDim.y
constexpr int64_t kMaxVertices = (int64_t)1 << 40;

// Fills `s`; returns ECC_OK or an error status with the message set.
int make_shape(int ndim, const int64_t* dims, int64_t batch, ecc::Shape* s) {
  if (ndim != 2 && ndim != 3) return fail(ECC_ERR_INVALID_ARG, "ndim must be 2 or 3, got %d", ndim);
  if (!dims) return fail(ECC_ERR_INVALID_ARG, "dims is NULL");
  if (batch < 1) return fail(ECC_ERR_INVALID_ARG, "batch must be >= 1, got %lld", (long long)batch);
  int64_t n = 1;
  for (int k = 0; k < ndim; ++k) {
    if (dims[k] < 1)
      return fail(ECC_ERR_INVALID_ARG, "dims[%d] must be >= 1, got %lld", k, (long long)dims[k]);
    if (dims[k] > kMaxVertices / n)
      return fail(ECC_ERR_UNSUPPORTED, "grid has more than 2^40 vertices");
    n *= dims[k];
  }
  if (batch > kMaxBatch)
    return fail(ECC_ERR_UNSUPPORTED, "batch %lld exceeds %lld", (long long)batch, (long long)kMaxBatch);
  if (batch > kMaxVertices / n) return fail(ECC_ERR_UNSUPPORTED, "batch * vertices exceeds 2^40");
  s->ndim = ndim;
  s->D = ndim == 3 ? dims[0] : 1;
  s->H = dims[ndim - 2];
  s->W = dims[ndim - 1];
  s->N = n;
  s->batch = batch;
  return ECC_OK;
}

int check_dtype(int dtype) {
  if (dtype != ECC_U8 && dtype != ECC_U16 && dtype != ECC_F32)
    return fail(ECC_ERR_INVALID_ARG, "unknown dtype %d (this entry point takes ECC_U8, ECC_U16, ECC_F32)", dtype);
  return ECC_OK;
}
// the hard curves also take the element types that are rounded to float32 first
bool converted_dtype(int dtype) { return dtype >= ECC_F16 && dtype <= ECC_I16; }
bool integer_dtype(int dtype) { return dtype == ECC_U8 || dtype == ECC_U16 || dtype == ECC_I32 || dtype == ECC_I16; }
size_t dtype_size(int dtype) {
  switch (dtype) {
    case ECC_U8: return 1;
    case ECC_U16: case ECC_F16: case ECC_BF16: case ECC_I16: return 2;
    case ECC_F64: return 8;
    default: return 4;
  }
}
size_t convert_bytes(const ecc::Shape& s, int dtype) {
  return converted_dtype(dtype) ? (((size_t)s.N * s.batch * sizeof(float) + 255) / 256) * 256 : 0;
}

int device_status(hipError_t e, const char* what) {
  if (e == hipSuccess) return ECC_OK;
  return fail(ECC_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

int check_soft_common(const float* grid, const float* u, float alpha, const float* tau, int T,
                      float lambda) {
  if (!grid) return fail(ECC_ERR_INVALID_ARG, "grid is NULL");
  if (!u) return fail(ECC_ERR_INVALID_ARG, "u is NULL");
  if (!tau) return fail(ECC_ERR_INVALID_ARG, "tau is NULL");
  if (T < 1) return fail(ECC_ERR_INVALID_ARG, "T must be >= 1, got %d", T);
  if (T > ECC_MAX_THRESHOLDS)
    return fail(ECC_ERR_UNSUPPORTED, "T %d exceeds ECC_MAX_THRESHOLDS %d", T, ECC_MAX_THRESHOLDS);
  if (!(lambda > 0.0f) || !std::isfinite(lambda))
    return fail(ECC_ERR_INVALID_ARG, "lambda must be finite and > 0");
  if (!std::isfinite(alpha)) return fail(ECC_ERR_INVALID_ARG, "alpha must be finite");
  if ((reinterpret_cast<uintptr_t>(grid) | reinterpret_cast<uintptr_t>(u) | reinterpret_cast<uintptr_t>(tau)) & 3)
    return fail(ECC_ERR_INVALID_ARG, "grid / u / tau is not 4-byte aligned");
  return ECC_OK;
}
int check_f32_out(const void* p, const char* name) {
  if (reinterpret_cast<uintptr_t>(p) & 3) return fail(ECC_ERR_INVALID_ARG, "%s is not 4-byte aligned", name);
  return ECC_OK;
}

int check_workspace(void* ws, size_t have, size_t need) {
  if (!ws) return fail(ECC_ERR_WORKSPACE, "workspace is NULL (need %zu bytes)", need);
  if (have < need) return fail(ECC_ERR_WORKSPACE, "workspace has %zu bytes, need %zu", have, need);
  if (reinterpret_cast<uintptr_t>(ws) & 255)
    return fail(ECC_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  return ECC_OK;
}

}  // namespace

namespace ecc {
unsigned forced_paths() { return g_forced.load(std::memory_order_relaxed); }
}  // namespace ecc

extern "C" {

unsigned ecc_debug_force(unsigned mask) {
  return g_forced.exchange(mask & (ECC_FORCE_GENERIC | ECC_FORCE_TWO_PASS | ECC_FORCE_SOFT_TILES | ECC_FORCE_NO_SMALL),
                           std::memory_order_relaxed);
}

const char* ecc_last_error(void) { return g_err; }

const char* ecc_version(void) { return "libecc_hip 0.1 (gfx950)"; }

size_t ecc_workspace_bytes(int ndim, const int64_t* dims, int64_t batch, int bins_or_T) {
  ecc::Shape s;
  if (make_shape(ndim, dims, batch, &s) != ECC_OK) return 0;
  if (bins_or_T < 1) {
    fail(ECC_ERR_INVALID_ARG, "bins_or_T must be >= 1");
    return 0;
  }
  size_t a = ecc::hard_workspace_bytes(s, bins_or_T);
  size_t b = ecc::soft_workspace_bytes(s, bins_or_T);
  return a > b ? a : b;
}

size_t ecc_workspace_bytes_dtype(int ndim, const int64_t* dims, int64_t batch, ecc_dtype dtype, int bins) {
  ecc::Shape s;
  if (make_shape(ndim, dims, batch, &s) != ECC_OK) return 0;
  if (!converted_dtype(dtype) && check_dtype(dtype) != ECC_OK) return 0;
  const size_t base = ecc_workspace_bytes(ndim, dims, batch, bins);
  return base ? base + convert_bytes(s, dtype) : 0;
}

// The current device's copy of `scratch`: looked up with hipGetSymbolAddress on the first call
// on that device (no allocation: the array is part of the loaded code object).
static int static_scratch(const char* who, void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return device_status(e, who);
  if (dev < 0 || dev >= kMaxDevices) return fail(ECC_ERR_UNSUPPORTED, "%s: device index %d beyond %d", who, dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return device_status(e, who);
    if (!p) return fail(ECC_ERR_DEVICE, "%s: hipGetSymbolAddress returned NULL", who);
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return ECC_OK;
}

// use_static: the workspace is the library's static scratch (workspace / workspace_bytes ignored)
static int hard_common(int conv, const char* who, const void* grid, int ndim, const int64_t* dims, int64_t batch, int dtype, int bins,
             const double* range, int64_t* curve, void* workspace, size_t workspace_bytes,
             void* hip_stream, bool use_static = false) {
  ecc::Shape s;
  int rc = make_shape(ndim, dims, batch, &s);
  if (rc != ECC_OK) return rc;
  if (!converted_dtype(dtype) && (rc = check_dtype(dtype)) != ECC_OK) return rc;
  if (!grid) return fail(ECC_ERR_INVALID_ARG, "grid is NULL");
  if (!curve) return fail(ECC_ERR_INVALID_ARG, "curve is NULL");
  if (bins < 1) return fail(ECC_ERR_INVALID_ARG, "bins must be >= 1, got %d", bins);
  if (bins > ECC_MAX_BINS)
    return fail(ECC_ERR_UNSUPPORTED, "bins %d exceeds ECC_MAX_BINS %d", bins, ECC_MAX_BINS);
  double lo = 0.0, hi = 0.0;
  if (range) {
    lo = range[0];
    hi = range[1];
    if (!std::isfinite(lo) || !std::isfinite(hi) || lo > hi)
      return fail(ECC_ERR_RANGE, "range must be finite with lo <= hi");
  }
  if (reinterpret_cast<uintptr_t>(grid) % dtype_size(dtype))
    return fail(ECC_ERR_INVALID_ARG, "grid is not aligned to its element size");
  if (reinterpret_cast<uintptr_t>(curve) % 8)
    return fail(ECC_ERR_INVALID_ARG, "curve is not 8-byte aligned");
  // the static scratch may hold the smaller workspace only: then no list per block of the sweep
  size_t base_bytes = ecc::hard_workspace_bytes(s, bins);
  bool roomy = true;
  if (use_static && base_bytes + convert_bytes(s, dtype) > (size_t)ECC_STATIC_SCRATCH_BYTES) {
    base_bytes = ecc::hard_workspace_min_bytes(s, bins);
    roomy = false;
  }
  if (use_static) {
    const size_t need = base_bytes + convert_bytes(s, dtype);
    if (need > (size_t)ECC_STATIC_SCRATCH_BYTES)
      return fail(ECC_ERR_UNSUPPORTED, "%s: this call needs %zu bytes of scratch, the static buffer has %zu "
                  "(use ecc_hard with a workspace)", who, need, (size_t)ECC_STATIC_SCRATCH_BYTES);
    if ((rc = static_scratch(who, &workspace)) != ECC_OK) return rc;
  } else if ((rc = check_workspace(workspace, workspace_bytes, base_bytes + convert_bytes(s, dtype))) != ECC_OK) {
    return rc;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (converted_dtype(dtype)) {
    // room for a float32 copy behind the path's own workspace (the strip / tube sweeps read float16,
    // bfloat16 and int16 directly and leave it unused); one bin per level (integer types without a
    // range) is the equal-width table over (-1, B-1], or the lower edges of the one over [0, B) for
    // superlevel sets
    float* f32 = reinterpret_cast<float*>(static_cast<char*>(workspace) + base_bytes);
    bool have_range = range != nullptr;
    if (!have_range && integer_dtype(dtype)) {
      have_range = true;
      const bool super = (conv & ecc::kConvSuper) != 0;
      lo = super ? 0.0 : -1.0;
      hi = super ? (double)bins : (double)bins - 1.0;
    }
    return device_status(ecc::launch_hard(grid, s, dtype, bins, have_range, lo, hi, curve, workspace, st, nullptr,
                                          conv, f32, roomy),
                         who);
  }
  return device_status(ecc::launch_hard(grid, s, dtype, bins, range != nullptr, lo, hi, curve, workspace, st,
                                        nullptr, conv, nullptr, roomy),
                       who);
}

int ecc_hard(const void* grid, int ndim, const int64_t* dims, int64_t batch, ecc_dtype dtype, int bins,
             const double* range, int64_t* curve, void* workspace, size_t workspace_bytes,
             void* hip_stream) {
  return hard_common(0, "ecc_hard", grid, ndim, dims, batch, dtype, bins, range, curve, workspace, workspace_bytes,
                     hip_stream);
}

int ecc_hard_static(const void* grid, int ndim, const int64_t* dims, int64_t batch, ecc_dtype dtype, int bins,
                    const double* range, int64_t* curve, void* hip_stream) {
  return hard_common(0, "ecc_hard_static", grid, ndim, dims, batch, dtype, bins, range, curve, nullptr, 0, hip_stream,
                     true);
}

int ecc_hard_top(const void* grid, int ndim, const int64_t* dims, int64_t batch, ecc_dtype dtype, int bins,
                 const double* range, int64_t* curve, void* workspace, size_t workspace_bytes,
                 void* hip_stream) {
  return hard_common(ecc::kConvTop, "ecc_hard_top", grid, ndim, dims, batch, dtype, bins, range, curve, workspace, workspace_bytes,
                     hip_stream);
}

int ecc_hard_ex(const void* grid, int ndim, const int64_t* dims, int64_t batch, ecc_dtype dtype, int construction,
                int filtration, int bins, const double* range, int64_t* curve, void* workspace,
                size_t workspace_bytes, void* hip_stream) {
  if (construction != ECC_VERTEX && construction != ECC_TOPCELL)
    return fail(ECC_ERR_INVALID_ARG, "construction must be ECC_VERTEX or ECC_TOPCELL, got %d", construction);
  if (filtration != ECC_SUBLEVEL && filtration != ECC_SUPERLEVEL)
    return fail(ECC_ERR_INVALID_ARG, "filtration must be ECC_SUBLEVEL or ECC_SUPERLEVEL, got %d", filtration);
  const int conv = (construction == ECC_TOPCELL ? ecc::kConvTop : 0) | (filtration == ECC_SUPERLEVEL ? ecc::kConvSuper : 0);
  return hard_common(conv, "ecc_hard_ex", grid, ndim, dims, batch, dtype, bins, range, curve, workspace,
                     workspace_bytes, hip_stream);
}

size_t ecc_workspace_bytes_dir(int ndim, const int64_t* dims, int64_t batch, int ndir, int bins) {
  ecc::Shape s;
  if (make_shape(ndim, dims, batch, &s) != ECC_OK) return 0;
  if (bins < 1 || ndir < 1 || (int64_t)ndir * batch > kMaxBatch) {
    fail(ECC_ERR_INVALID_ARG, "bins and ndir must be >= 1 and ndir * batch <= %lld", (long long)kMaxBatch);
    return 0;
  }
  s.batch = (int64_t)ndir * batch;
  return ecc::hard_dir_workspace_bytes(s, bins);
}

int ecc_hard_dir(const float* grid, int ndim, const int64_t* dims, int64_t batch, const float* u, int ndir,
                 float alpha, int bins, const double* range, int64_t* curve, void* workspace,
                 size_t workspace_bytes, void* hip_stream) {
  ecc::Shape s;
  int rc = make_shape(ndim, dims, batch, &s);
  if (rc != ECC_OK) return rc;
  if (!grid) return fail(ECC_ERR_INVALID_ARG, "grid is NULL");
  if (!u) return fail(ECC_ERR_INVALID_ARG, "u is NULL");
  if (!curve) return fail(ECC_ERR_INVALID_ARG, "curve is NULL");
  if (ndir < 1) return fail(ECC_ERR_INVALID_ARG, "ndir must be >= 1, got %d", ndir);
  if ((int64_t)ndir * batch > kMaxBatch)
    return fail(ECC_ERR_UNSUPPORTED, "ndir * batch = %lld exceeds %lld", (long long)ndir * (long long)batch,
                (long long)kMaxBatch);
  if (!std::isfinite(alpha)) return fail(ECC_ERR_INVALID_ARG, "alpha must be finite");
  if (bins < 1) return fail(ECC_ERR_INVALID_ARG, "bins must be >= 1, got %d", bins);
  if (bins > ECC_MAX_BINS)
    return fail(ECC_ERR_UNSUPPORTED, "bins %d exceeds ECC_MAX_BINS %d", bins, ECC_MAX_BINS);
  double lo = 0.0, hi = 0.0;
  if (range) {
    lo = range[0];
    hi = range[1];
    if (!std::isfinite(lo) || !std::isfinite(hi) || lo > hi)
      return fail(ECC_ERR_RANGE, "range must be finite with lo <= hi");
  }
  if (reinterpret_cast<uintptr_t>(grid) % 4 || reinterpret_cast<uintptr_t>(u) % 4)
    return fail(ECC_ERR_INVALID_ARG, "grid / u is not 4-byte aligned");
  if (reinterpret_cast<uintptr_t>(curve) % 8)
    return fail(ECC_ERR_INVALID_ARG, "curve is not 8-byte aligned");
  ecc::Shape sv = s;
  sv.batch = (int64_t)ndir * batch;
  if ((rc = check_workspace(workspace, workspace_bytes, ecc::hard_dir_workspace_bytes(sv, bins))) != ECC_OK)
    return rc;
  return device_status(ecc::launch_hard_dir(grid, sv, u, alpha, (int)batch, bins, range != nullptr, lo, hi,
                                            curve, workspace, static_cast<hipStream_t>(hip_stream)),
                       "ecc_hard_dir");
}

int ecc_coeff(const void* grid, int ndim, const int64_t* dims, int64_t batch, ecc_dtype dtype,
              int8_t* c_out, void* hip_stream) {
  ecc::Shape s;
  int rc = make_shape(ndim, dims, batch, &s);
  if (rc != ECC_OK) return rc;
  if ((rc = check_dtype(dtype)) != ECC_OK) return rc;
  if (!grid) return fail(ECC_ERR_INVALID_ARG, "grid is NULL");
  if (!c_out) return fail(ECC_ERR_INVALID_ARG, "c_out is NULL");
  const size_t esz = dtype == ECC_U8 ? 1 : dtype == ECC_U16 ? 2 : 4;
  if (reinterpret_cast<uintptr_t>(grid) % esz)
    return fail(ECC_ERR_INVALID_ARG, "grid is not aligned to its element size");
  return device_status(
      ecc::launch_coeff(grid, s, dtype, c_out, static_cast<hipStream_t>(hip_stream)), "ecc_coeff");
}

static int soft_fwd_common(const char* who, bool tiltc, const float* grid, int ndim, const int64_t* dims,
                           int64_t batch, const float* u, float alpha, const float* tau, int T, float lambda,
                           float* chi, void* workspace, size_t workspace_bytes, void* hip_stream) {
  ecc::Shape s;
  int rc = make_shape(ndim, dims, batch, &s);
  if (rc != ECC_OK) return rc;
  if ((rc = check_soft_common(grid, u, alpha, tau, T, lambda)) != ECC_OK) return rc;
  if (!chi) return fail(ECC_ERR_INVALID_ARG, "chi is NULL");
  if ((rc = check_f32_out(chi, "chi")) != ECC_OK) return rc;
  if ((rc = check_workspace(workspace, workspace_bytes, ecc::soft_workspace_bytes(s, T))) != ECC_OK)
    return rc;
  return device_status(ecc::launch_soft_fwd(grid, s, u, alpha, tau, T, lambda, chi, workspace,
                                            static_cast<hipStream_t>(hip_stream), tiltc),
                       who);
}

static int soft_bwd_common(const char* who, bool tiltc, const float* grid, int ndim, const int64_t* dims,
                           int64_t batch, const float* u, float alpha, const float* tau, int T, float lambda,
                           const float* grad_chi, float* grad_X, float* dchi_dtau, float* dchi_du,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
  ecc::Shape s;
  int rc = make_shape(ndim, dims, batch, &s);
  if (rc != ECC_OK) return rc;
  if ((rc = check_soft_common(grid, u, alpha, tau, T, lambda)) != ECC_OK) return rc;
  if (!grad_X && !dchi_dtau && !dchi_du)
    return fail(ECC_ERR_INVALID_ARG, "all three outputs are NULL");
  if ((rc = check_f32_out(grad_chi, "grad_chi")) != ECC_OK || (rc = check_f32_out(grad_X, "grad_X")) != ECC_OK ||
      (rc = check_f32_out(dchi_dtau, "dchi_dtau")) != ECC_OK || (rc = check_f32_out(dchi_du, "dchi_du")) != ECC_OK)
    return rc;
  if ((rc = check_workspace(workspace, workspace_bytes, ecc::soft_workspace_bytes(s, T))) != ECC_OK)
    return rc;
  return device_status(
      ecc::launch_soft_bwd(grid, s, u, alpha, tau, T, lambda, grad_chi, grad_X, dchi_dtau, dchi_du,
                           workspace, static_cast<hipStream_t>(hip_stream), tiltc),
      who);
}

size_t ecc_soft_state_bytes(int ndim, const int64_t* dims, int64_t batch) {
  ecc::Shape s;
  if (make_shape(ndim, dims, batch, &s) != ECC_OK) return 0;
  return ecc::soft_state_bytes(s);
}

int ecc_soft_fwd_save(const float* grid, int ndim, const int64_t* dims, int64_t batch, const float* u, float alpha,
                      const float* tau, int T, float lambda, int tilted, float* chi, float* dchi_dtau,
                      float* dchi_du, void* state, size_t state_bytes, void* workspace, size_t workspace_bytes,
                      void* hip_stream) {
  ecc::Shape s;
  int rc = make_shape(ndim, dims, batch, &s);
  if (rc != ECC_OK) return rc;
  if ((rc = check_soft_common(grid, u, alpha, tau, T, lambda)) != ECC_OK) return rc;
  if (!chi) return fail(ECC_ERR_INVALID_ARG, "chi is NULL");
  if ((rc = check_f32_out(chi, "chi")) != ECC_OK || (rc = check_f32_out(dchi_dtau, "dchi_dtau")) != ECC_OK ||
      (rc = check_f32_out(dchi_du, "dchi_du")) != ECC_OK)
    return rc;
  if (!state || state_bytes < ecc::soft_state_bytes(s) || (reinterpret_cast<uintptr_t>(state) & 255))
    return fail(ECC_ERR_WORKSPACE, "state must be 256-byte aligned and hold ecc_soft_state_bytes() = %zu bytes",
                ecc::soft_state_bytes(s));
  if ((rc = check_workspace(workspace, workspace_bytes, ecc::soft_workspace_bytes(s, T))) != ECC_OK) return rc;
  return device_status(ecc::launch_soft_fwd_save(grid, s, u, alpha, tau, T, lambda, chi, dchi_dtau, dchi_du, state,
                                                 workspace, static_cast<hipStream_t>(hip_stream), tilted != 0),
                       "ecc_soft_fwd_save");
}

int ecc_soft_bwd_saved(const float* grid, int ndim, const int64_t* dims, int64_t batch, const float* u, float alpha,
                       const float* tau, int T, float lambda, int tilted, const float* grad_chi, float* grad_X,
                       const void* state, size_t state_bytes, void* workspace, size_t workspace_bytes,
                       void* hip_stream) {
  ecc::Shape s;
  int rc = make_shape(ndim, dims, batch, &s);
  if (rc != ECC_OK) return rc;
  if ((rc = check_soft_common(grid, u, alpha, tau, T, lambda)) != ECC_OK) return rc;
  if (!grad_X) return fail(ECC_ERR_INVALID_ARG, "grad_X is NULL");
  if ((rc = check_f32_out(grad_chi, "grad_chi")) != ECC_OK || (rc = check_f32_out(grad_X, "grad_X")) != ECC_OK)
    return rc;
  if (!state || state_bytes < ecc::soft_state_bytes(s) || (reinterpret_cast<uintptr_t>(state) & 255))
    return fail(ECC_ERR_WORKSPACE, "state must be 256-byte aligned and hold ecc_soft_state_bytes() = %zu bytes",
                ecc::soft_state_bytes(s));
  if ((rc = check_workspace(workspace, workspace_bytes, ecc::soft_workspace_bytes(s, T))) != ECC_OK) return rc;
  return device_status(ecc::launch_soft_bwd_saved(grid, s, u, alpha, tau, T, lambda, grad_chi, grad_X, state, workspace,
                                                  static_cast<hipStream_t>(hip_stream), tilted != 0),
                       "ecc_soft_bwd_saved");
}

int ecc_soft_fwd(const float* grid, int ndim, const int64_t* dims, int64_t batch, const float* u,
                 float alpha, const float* tau, int T, float lambda, float* chi, void* workspace,
                 size_t workspace_bytes, void* hip_stream) {
  return soft_fwd_common("ecc_soft_fwd", false, grid, ndim, dims, batch, u, alpha, tau, T, lambda, chi,
                         workspace, workspace_bytes, hip_stream);
}

int ecc_soft_bwd(const float* grid, int ndim, const int64_t* dims, int64_t batch, const float* u,
                 float alpha, const float* tau, int T, float lambda, const float* grad_chi,
                 float* grad_X, float* dchi_dtau, float* dchi_du, void* workspace,
                 size_t workspace_bytes, void* hip_stream) {
  return soft_bwd_common("ecc_soft_bwd", false, grid, ndim, dims, batch, u, alpha, tau, T, lambda, grad_chi,
                         grad_X, dchi_dtau, dchi_du, workspace, workspace_bytes, hip_stream);
}

int ecc_soft_fwd_tilted(const float* grid, int ndim, const int64_t* dims, int64_t batch, const float* u,
                        float alpha, const float* tau, int T, float lambda, float* chi, void* workspace,
                        size_t workspace_bytes, void* hip_stream) {
  return soft_fwd_common("ecc_soft_fwd_tilted", true, grid, ndim, dims, batch, u, alpha, tau, T, lambda, chi,
                         workspace, workspace_bytes, hip_stream);
}

int ecc_soft_bwd_tilted(const float* grid, int ndim, const int64_t* dims, int64_t batch, const float* u,
                        float alpha, const float* tau, int T, float lambda, const float* grad_chi,
                        float* grad_X, float* dchi_dtau, float* dchi_du, void* workspace,
                        size_t workspace_bytes, void* hip_stream) {
  return soft_bwd_common("ecc_soft_bwd_tilted", true, grid, ndim, dims, batch, u, alpha, tau, T, lambda,
                         grad_chi, grad_X, dchi_dtau, dchi_du, workspace, workspace_bytes, hip_stream);
}

int ecc_count_nonfinite(const void* grid, int64_t n, ecc_dtype dtype, unsigned long long* count,
                        void* hip_stream) {
  if (!converted_dtype(dtype) && check_dtype(dtype) != ECC_OK) return ECC_ERR_INVALID_ARG;
  if (!grid) return fail(ECC_ERR_INVALID_ARG, "grid is NULL");
  if (!count) return fail(ECC_ERR_INVALID_ARG, "count is NULL");
  if (n < 1 || n > kMaxVertices) return fail(ECC_ERR_INVALID_ARG, "n must be in 1 .. 2^40, got %lld", (long long)n);
  if (reinterpret_cast<uintptr_t>(grid) % dtype_size(dtype))
    return fail(ECC_ERR_INVALID_ARG, "grid is not aligned to its element size");
  if (reinterpret_cast<uintptr_t>(count) % 8) return fail(ECC_ERR_INVALID_ARG, "count is not 8-byte aligned");
  return device_status(ecc::launch_count_nonfinite(grid, n, dtype, count, static_cast<hipStream_t>(hip_stream)),
                       "ecc_count_nonfinite");
}

int ecc_profile_begin(int max_launches) {
  if (max_launches < 1 || max_launches > 4096)
    return fail(ECC_ERR_INVALID_ARG, "max_launches must be in 1..4096");
  return device_status(ecc::profile_begin(max_launches), "ecc_profile_begin");
}

int ecc_profile_end(float* mean_ms, int* launches) {
  if (!mean_ms || !launches) return fail(ECC_ERR_INVALID_ARG, "output pointer is NULL");
  return device_status(ecc::profile_end(mean_ms, launches), "ecc_profile_end");
}

}  // extern "C"
