/*
 * libecc_hip -- Euler Characteristic Curves of dense 2D/3D grids on MI355X (gfx950).
 *
 * C ABI.  Every array argument is a DEVICE pointer owned by the caller unless
 * marked "host".  The library never allocates device memory, never
 * synchronises, and enqueues work only on the HIP stream it is given
 * (hip_stream is a hipStream_t passed as void*; NULL is the default stream).
 * Scratch space is passed in as `workspace` (device memory, 256-byte aligned,
 * at least ecc_workspace_bytes() long); two calls that may overlap in time
 * must not share one workspace.
 *
 * Every entry point validates its arguments on the host BEFORE the first HIP
 * call and returns an ecc_status; ecc_last_error() gives a message for the
 * last failure on the calling thread.
 *
 * Grid values must be finite.  This is NOT checked on the hot path (a test per
 * vertex would cost the 3D sweep, which is bound by instruction issue, about
 * 3 %): a NaN compares false with everything, so it ends up somewhere in the
 * order and the curve is unspecified -- no fault, every access stays in bounds.
 * A caller that cannot vouch for its data runs ecc_count_nonfinite() first (one
 * read pass) and looks at the count when convenient.
 *
 * Complex convention (the paper's Background section, Eq. 1-3, leaves it
 * open; this library fixes it): grid points are the vertices of a cubical
 * complex; an edge / square / cube (2 / 2x2 / 2x2x2 axis-adjacent points,
 * inside the grid, no wrap-around) is present at threshold tau once ALL its
 * vertices are <= tau; ECC(tau) = V - E + F - C.  In the per-vertex form
 * ECC(tau) = sum_p c(p) 1[X(p) <= tau] each cell is charged to its last
 * vertex under the order "smaller value first, equal values by C-order linear
 * index", so c(p) = 1 - #edges + #squares - #cubes charged to p.
 *
 * Grid layout: C-contiguous [batch][D][H][W] (3D) or [batch][H][W] (2D), W
 * fastest; `dims` lists one item's extents slowest-first.
 */
#ifndef ECC_H_
#define ECC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Element types.  ECC_U8, ECC_U16 and ECC_F32 are read as they are by every
 * entry point.  The others are taken by the hard curves only (ecc_hard,
 * ecc_hard_static, ecc_hard_top, ecc_hard_ex).  ECC_F16, ECC_BF16 and ECC_I16
 * widen to float32 without rounding and are loaded directly by the strip / tube
 * sweeps (two bytes per vertex of memory traffic).  ECC_I32 and ECC_F64 -- and
 * the two-byte types on the shapes the plain kernels take -- are first rounded
 * to float32 (to nearest even) into the workspace, and the curve is that of the
 * rounded grid: rounding is monotone, so every set {p : fl32(X(p)) <= t} is a
 * sublevel set of X and the curve is exact for the float32 thresholds it is
 * read at; values beyond the float32 range are not allowed.  All five need the
 * larger workspace of ecc_workspace_bytes_dtype.
 */
typedef enum {
  ECC_U8 = 0, ECC_U16 = 1, ECC_F32 = 2,
  ECC_F16 = 3, ECC_I32 = 4, ECC_F64 = 5, ECC_BF16 = 6, ECC_I16 = 7
} ecc_dtype;

typedef enum {
  ECC_OK = 0,
  ECC_ERR_INVALID_ARG = -1, /* NULL pointer, bad ndim/dims/batch/bins/T/lambda/dtype     */
  ECC_ERR_UNSUPPORTED = -2, /* valid request outside the built limits (see ECC_MAX_*)       */
  ECC_ERR_WORKSPACE = -3,   /* workspace NULL or smaller than ecc_workspace_bytes()         */
  ECC_ERR_RANGE = -4,       /* `range` argument: lo > hi, or lo / hi not finite             */
  ECC_ERR_DEVICE = -5       /* a HIP call failed; message holds hipGetErrorString           */
} ecc_status;

#define ECC_MAX_BINS 16384       /* per-block LDS histogram of int32 counters     */
#define ECC_MAX_THRESHOLDS 4096  /* soft thresholds held in LDS                   */

/* Message for the last non-OK status returned on this thread ("" if none). */
const char* ecc_last_error(void);

/* Library version string. */
const char* ecc_version(void);

/*
 * Bytes of device workspace sufficient for any entry point called with these
 * dims / batch and with bins (hard) or T (soft) = bins_or_T.  Host-only
 * arithmetic; returns 0 on invalid arguments.  For the hard curves this is
 * about one byte per vertex, except for batches of up to 2^27 vertices (2^25
 * in volumes), which get room for every vertex in a list (about 8.5 bytes per
 * vertex: their calls then need nothing cleared first and no second sweep in
 * reserve).
 */
size_t ecc_workspace_bytes(int ndim, const int64_t* dims /* host */, int64_t batch,
                           int bins_or_T);

/*
 * The same for the hard curves with element type `dtype` (any ecc_dtype): adds the
 * room for the float32 copy of the grid that ECC_F16 .. ECC_I16 need.
 */
size_t ecc_workspace_bytes_dtype(int ndim, const int64_t* dims /* host */, int64_t batch, ecc_dtype dtype,
                                 int bins);

/*
 * Hard ECC (Eq. 3 of the paper, Methods "full sweep"): per-vertex coefficient
 * c(p) from the 3x3 / 3x3x3 neighbourhood, histogram of c(p) over threshold
 * bins, inclusive prefix sum.
 *
 *   grid    device, [batch] items of dims, element type `dtype`
 *   ndim    2 or 3;  dims host array of ndim extents (slowest first, each >= 1)
 *   bins    number of thresholds B, 1..ECC_MAX_BINS
 *   range   host double[2] = {lo, hi} with lo <= hi, or NULL.
 *           Thresholds t_0 <= ... <= t_{B-1}:
 *             range given (any dtype): t_b = float32(lo + (b+1)(hi-lo)/B)
 *               evaluated in float64, and t_{B-1} = float32(hi);
 *             NULL, integer dtype:  t_b = b   (one bin per level);
 *             NULL, floating dtype: lo, hi = min, max over the WHOLE batch, then
 *               as above.  (No extra read pass: the one sweep tracks the range
 *               and lists the vertices with c != 0, which are binned afterwards;
 *               a field so rough that more than one vertex in eight has c != 0
 *               overflows the lists and is swept a second time.)
 *   curve   device out, int64 [batch][B]: curve[i][b] = ECC of item i at t_b.
 *           A point with X(p) > t_{B-1} is in no sublevel set and is dropped;
 *           a point with X(p) <= t_0 counts from bin 0.
 * The curve is exact (integer arithmetic end to end) and does not depend on
 * the tie-break.
 */
int ecc_hard(const void* grid, int ndim, const int64_t* dims, int64_t batch, ecc_dtype dtype,
             int bins, const double* range, int64_t* curve, void* workspace,
             size_t workspace_bytes, void* hip_stream);

/*
 * ecc_hard for callers that cannot allocate device memory and have no workspace
 * to pass: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, thresholds, output and errors as ecc_hard,
 * minus the workspace: the scratch space is a static device array inside the
 * library, ECC_STATIC_SCRATCH_BYTES long, one copy per GPU, held until the
 * process ends.  The call allocates and frees nothing (the array's address on
 * the current device is looked up once, on the first call on that device).
 * A request that would not fit returns ECC_ERR_UNSUPPORTED -- roughly one byte
 * of scratch per float32 vertex, so about 32 M vertices per call, e.g. two
 * 4096^2 images or 256^3 volumes (the larger workspace that ecc_workspace_bytes
 * asks for on behalf of mid-sized batches is used when it fits and done without
 * when it does not).
 * Every call on a GPU uses that GPU's one array: calls that may overlap in time
 * on one GPU (different streams, different threads) race and must not be made;
 * calls on one stream are ordered and safe.  Nothing needs to be cleared
 * between calls (each call resets what it uses).
 */
#define ECC_STATIC_SCRATCH_BYTES (32u << 20)
int ecc_hard_static(const void* grid, int ndim, const int64_t* dims, int64_t batch, ecc_dtype dtype,
                    int bins, const double* range, int64_t* curve, void* hip_stream);

/*
 * The coefficient map itself (Eq. 3): c_out[batch][N] int8, values in
 * [-3, 1] (2D) or [-5, 7] (3D).  Exposes the first step of ecc_hard and of
 * the soft path for inspection and tests: shapes that the strip / tube sweeps
 * of those paths take (rows of 8 elements or more) are computed by those very
 * sweeps -- the map is cleared and the sweep writes c(p) at the vertices with
 * c != 0 -- so the map shows, vertex by vertex, the stencil and the tie-break
 * (equal values: the smaller C-order index first; -0 equals +0) that every
 * other entry point runs.  Other shapes use a plain one-thread-per-vertex
 * kernel.  Every element of c_out is written.  Needs no workspace.
 */
int ecc_coeff(const void* grid, int ndim, const int64_t* dims, int64_t batch, ecc_dtype dtype,
              int8_t* c_out, void* hip_stream);

/*
 * Soft single-direction ECC forward (Eq. 6):
 *   chi[i][j] = sum_p c_i(p) sigma_lambda( tau_j - X_i(p) - alpha <u, p> ),
 *   sigma_lambda(z) = 1 / (1 + exp(-lambda z)).
 * c(p) is the integer coefficient of the raw grid X (as in ecc_coeff).
 * p = (x, y[, z]) are 0-based integer grid coordinates with x the FASTEST
 * axis (column), so for 2D <u,p> = u[0]*col + u[1]*row.  u is used as given
 * (the caller keeps it on the unit sphere).
 *
 *   grid  device float32 [batch] items;  u device float32 [ndim]
 *   tau   device float32 [T], 1 <= T <= ECC_MAX_THRESHOLDS, shared by the batch
 *   lambda > 0 and finite;  alpha finite
 *   chi   device out float32 [batch][T]
 * Sigmoids are evaluated in float32 on an argument formed in float64; partial
 * sums are combined in a fixed order, so results are run-to-run identical.
 */
int ecc_soft_fwd(const float* grid, int ndim, const int64_t* dims, int64_t batch,
                 const float* u, float alpha, const float* tau, int T, float lambda,
                 float* chi, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Soft ECC derivatives (Eq. 8, 9, 10 of the appendix; Eq. 7), with
 * sigma' = lambda sigma (1 - sigma) and z_pj = tau_j - X(p) - alpha <u,p>:
 *   grad_X[i][p]       = sum_j g[i][j] * ( -c_i(p) sigma'(z_pj) )       (Eq. 8, contracted)
 *   dchi_dtau[i][j]    =  sum_p c_i(p) sigma'(z_pj)                     (Eq. 9)
 *   dchi_du[i][j][k]   = -alpha sum_p c_i(p) sigma'(z_pj) p_k           (Eq. 10), k = x, y[, z]
 * c(p) is treated as a constant (the paper differentiates through the
 * sigmoid only); dchi_du is the unconstrained ambient derivative.
 *
 *   grad_chi  device float32 [batch][T] upstream g, or NULL for all ones
 *   grad_X    device out float32 [batch][N]        (every element written)
 *   dchi_dtau device out float32 [batch][T]
 *   dchi_du   device out float32 [batch][T][ndim]
 * Any of the three outputs may be NULL to skip it (not all three).
 */
int ecc_soft_bwd(const float* grid, int ndim, const int64_t* dims, int64_t batch,
                 const float* u, float alpha, const float* tau, int T, float lambda,
                 const float* grad_chi, float* grad_X, float* dchi_dtau, float* dchi_du,
                 void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Forward pass that saves state for the backward pass (a training step needs
 * both; Methods, "Learning Setup").  Every term of Eq. 6 and Eq. 8-10 carries
 * the factor c(p), so only the vertices with c != 0 matter, and the forward
 * sweep has to find them anyway: ecc_soft_fwd_save leaves them -- position,
 * c(p) and y = X(p) + alpha <u,p> -- in `state`, and ecc_soft_bwd_saved forms
 * grad_X (Eq. 8 contracted with grad_chi) from that list alone, without
 * sweeping the grid again.  The sums over p of Eq. 9 and Eq. 10 share their
 * sigmoids with Eq. 6, so the forward call returns them as well:
 *   ecc_soft_fwd_save   chi as ecc_soft_fwd (bit for bit); dchi_dtau, dchi_du as
 *                       ecc_soft_bwd (either may be NULL); fills `state`
 *   ecc_soft_bwd_saved  grad_X as ecc_soft_bwd (every element written)
 * tilted != 0: c(p) of the tilted field (as ecc_soft_fwd_tilted).
 *   state  device memory, 256-byte aligned, ecc_soft_state_bytes() long, owned by
 *          the caller.  It needs no initialisation.  What it holds depends on
 *          grid, dims, batch, u, alpha and `tilted` only -- tau, lambda and
 *          grad_chi may differ between the two calls -- and the caller must pass
 *          the same grid (unchanged), u and alpha to ecc_soft_bwd_saved.  A state
 *          written for another shape, and an item with so many vertices of c != 0
 *          (more than one in eight of some unit of rows / planes) that its list
 *          overflowed, are noticed on the device: those items are evaluated from
 *          the grid again, so the result is right either way.
 * Shapes outside the fused kernels (T > 256, grids narrower than 8, volumes of
 * 2^31 vertices or more) keep no state: the two calls then run ecc_soft_fwd +
 * ecc_soft_bwd's kernels.  workspace as ecc_soft_fwd.
 */
size_t ecc_soft_state_bytes(int ndim, const int64_t* dims /* host */, int64_t batch);
int ecc_soft_fwd_save(const float* grid, int ndim, const int64_t* dims, int64_t batch, const float* u,
                      float alpha, const float* tau, int T, float lambda, int tilted, float* chi,
                      float* dchi_dtau, float* dchi_du, void* state, size_t state_bytes, void* workspace,
                      size_t workspace_bytes, void* hip_stream);
int ecc_soft_bwd_saved(const float* grid, int ndim, const int64_t* dims, int64_t batch, const float* u,
                       float alpha, const float* tau, int T, float lambda, int tilted, const float* grad_chi,
                       float* grad_X, const void* state, size_t state_bytes, void* workspace,
                       size_t workspace_bytes, void* hip_stream);

/*
 * Soft ECC with the coefficient of the TILTED field: Eq. 6 and Eq. 8-10 exactly
 * as in ecc_soft_fwd / ecc_soft_bwd, except that c(p) is the coefficient (Eq. 3)
 * of Y(p) = X(p) + alpha <u,p> instead of the coefficient of X.  Y is formed in
 * float32 as ecc_hard_dir forms it (see there), so for lambda -> infinity
 * chi[i][j] tends to the directional hard curve of item i at tau_j -- with the
 * coefficient of X (the paper's Eq. 6 read literally) it tends to
 * sum_p c_X(p) 1[Y(p) <= tau_j], which is not an Euler characteristic.  The
 * sigmoid argument and the derivatives are unchanged (c is still a constant).
 * Arguments, outputs, workspace (ecc_workspace_bytes) and errors: as the two
 * entry points above.
 */
int ecc_soft_fwd_tilted(const float* grid, int ndim, const int64_t* dims, int64_t batch,
                        const float* u, float alpha, const float* tau, int T, float lambda,
                        float* chi, void* workspace, size_t workspace_bytes, void* hip_stream);
int ecc_soft_bwd_tilted(const float* grid, int ndim, const int64_t* dims, int64_t batch,
                        const float* u, float alpha, const float* tau, int T, float lambda,
                        const float* grad_chi, float* grad_X, float* dchi_dtau, float* dchi_du,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Hard ECC of the top-cell construction (the Background section leaves the
 * construction of the cubical complex open): the grid points are the
 * top-dimensional cells -- pixels are closed unit squares, voxels closed unit
 * cubes -- and a lower cell (edge, vertex, face) is present as soon as one of
 * the top cells around it is, so squares that touch in a corner are connected
 * (8- / 26-connectivity of the sublevel set, where ecc_hard has 4- / 6-).  Every
 * cell is charged to the first top cell around it; that coefficient is (-1)^d
 * times the vertex coefficient of Eq. 3 for the reversed order with everything
 * outside the grid coming first, which is how it is computed.  Arguments,
 * thresholds, bins, output, workspace and errors: exactly as ecc_hard.
 */
int ecc_hard_top(const void* grid, int ndim, const int64_t* dims, int64_t batch, ecc_dtype dtype, int bins,
                 const double* range, int64_t* curve, void* workspace, size_t workspace_bytes,
                 void* hip_stream);

/*
 * Hard ECC with the construction and the direction of the filtration chosen by
 * the caller (the Background section fixes neither beyond "cubical complex" and
 * sublevel sets; superlevel sets are the same definition, Eq. 1-2, on the
 * descending order):
 *   construction  ECC_VERTEX (as ecc_hard) or ECC_TOPCELL (as ecc_hard_top)
 *   filtration    ECC_SUBLEVEL: curve[i][b] = chi({p : X(p) <= t_b}), as those two;
 *                 ECC_SUPERLEVEL: curve[i][b] = chi({p : X(p) >= t'_b}), read at the
 *                 LOWER edges of the same bins: t'_0 = float32(lo), t'_b = t_{b-1}
 *                 (so curve[i][0] is the whole grid when lo is the minimum); integer
 *                 grids without a range: t'_b = b.  The comparison X >= t'_b is made
 *                 in float32 on that table, like X <= t_b for sublevel sets.
 * The superlevel curve is the sum of per-point coefficients over the points with
 * X(p) >= t'_b (Eq. 3 on the descending order), binned by max{b : t'_b <= X(p)}
 * and summed from the last bin down.  Everything else -- arguments, range, bins,
 * output, workspace, errors -- is as for ecc_hard.
 */
#define ECC_VERTEX 0
#define ECC_TOPCELL 1
#define ECC_SUBLEVEL 0
#define ECC_SUPERLEVEL 1
int ecc_hard_ex(const void* grid, int ndim, const int64_t* dims, int64_t batch, ecc_dtype dtype, int construction,
                int filtration, int bins, const double* range, int64_t* curve, void* workspace,
                size_t workspace_bytes, void* hip_stream);

/*
 * Directional hard curves (Background: the Euler characteristic transform looks at
 * a shape along directions; Eq. 6 tilts the filtration by alpha <u, p>).  For
 * every direction u_k the field
 *     Y_k(p) = X(p) + t_k(p),   p = (x, y[, z]) 0-based, x the fastest axis,
 *     t_k = fl(fl(fl(a_x x) + fl(a_y y)) + fl(a_z z))   (last term in 3D only),
 *     a_d = fl(alpha u_kd),
 * is formed in float32 -- every operation rounded to float32 in exactly this
 * order, the order on the vertices depends on it -- and its hard ECC taken
 * as in ecc_hard (Eq. 3): the coefficient c(p) is the one of the tilted field.
 *   grid   device float32 [batch][D][H][W]
 *   u      device float32 [ndir][ndim]   (used as given; the caller normalises)
 *   range  host [lo, hi] or NULL: the min / max over all directions and items
 *   curve  device int64 out [ndir][batch][bins]
 *   ndir * batch <= 65535; workspace of ecc_workspace_bytes_dir() bytes.
 * Other arguments, ownership, errors: as ecc_hard.
 */
size_t ecc_workspace_bytes_dir(int ndim, const int64_t* dims, int64_t batch, int ndir, int bins);
int ecc_hard_dir(const float* grid, int ndim, const int64_t* dims, int64_t batch, const float* u, int ndir,
                 float alpha, int bins, const double* range, int64_t* curve, void* workspace,
                 size_t workspace_bytes, void* hip_stream);

/*
 * Number of grid elements that are NaN or +-Inf (the entry points above need
 * finite values and do not check): *count (device, 8-byte aligned) receives
 * the count over all n elements; 0 for the integer types.  One read pass on
 * hip_stream; no workspace.  Any ecc_dtype.
 */
int ecc_count_nonfinite(const void* grid, int64_t n, ecc_dtype dtype, unsigned long long* count,
                        void* hip_stream);

/*
 * Test aid (not part of the method): forces the fall-back kernels on shapes
 * that would otherwise take the fast ones, so that tests can compare every
 * path with the oracle on the same inputs.  `mask` is an OR of
 *   ECC_FORCE_GENERIC     hard curves and ecc_coeff: the one-thread-per-vertex
 *                         kernels for every shape;
 *   ECC_FORCE_TWO_PASS    float grids without a range: a separate min / max
 *                         pass over the grid, then the histogram-mode sweep,
 *                         instead of the single pass that lists the critical
 *                         vertices;
 *   ECC_FORCE_SOFT_TILES  soft path: the tile kernels for every shape;
 *   ECC_FORCE_NO_SMALL    hard curves: small and mid-sized float inputs
 *                         without a range (up to 2^27 vertices, 2^25 in
 *                         volumes, up to 4096 bins) go through the five-launch
 *                         flow of the large ones instead of the two- /
 *                         three-launch flows made for them (any other bit
 *                         switches those flows off as well).
 * 0 restores normal operation.  Returns the previous mask.  The setting is
 * process-wide (one atomic word) and is read when a call is enqueued; results
 * are the same on every path, only the kernels differ.
 */
#define ECC_FORCE_GENERIC 1u
#define ECC_FORCE_TWO_PASS 2u
#define ECC_FORCE_SOFT_TILES 4u
#define ECC_FORCE_NO_SMALL 8u
unsigned ecc_debug_force(unsigned mask);

/*
 * Measurement aid (not part of the method; Experiments section reports
 * "kernel execution times"): between ecc_profile_begin() and
 * ecc_profile_end() every hard or soft call records a pair of HIP events around
 * its sweep kernel (the coefficient + histogram / sigmoid pass that dominates
 * the path; for ecc_soft_bwd_saved the list kernel) on the call's own stream.  ecc_profile_end() waits for the recorded
 * events, stores the mean kernel duration in milliseconds and the number of
 * launches measured, destroys the events and switches recording off.
 * max_launches in 1..4096; launches beyond it are not recorded.  One
 * recording at a time per process (a second ecc_profile_begin fails until
 * ecc_profile_end); the state is guarded by a mutex, so calls from several
 * threads are safe and all their sweeps land in the one recording.
 */
int ecc_profile_begin(int max_launches);
int ecc_profile_end(float* mean_ms /* host */, int* launches /* host */);

#ifdef __cplusplus
}
#endif
#endif /* ECC_H_ */
