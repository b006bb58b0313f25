"""Thin Python binding of the C ABI in include/ecc.h: argument marshalling only.

Tensors are torch CUDA(HIP) tensors; torch supplies device memory and the
current stream, every step of the computation runs inside libecc_hip.so.
"""
from __future__ import annotations

import ctypes

import torch

from . import _lib

ECC_U8, ECC_U16, ECC_F32, ECC_F16, ECC_I32, ECC_F64, ECC_BF16, ECC_I16 = 0, 1, 2, 3, 4, 5, 6, 7
# (the hard curves take all of these; ecc_coeff and the soft path uint8 / uint16 / float32 resp. float32)
_DTYPES = {torch.uint8: ECC_U8, torch.uint16: ECC_U16, torch.float32: ECC_F32, torch.float16: ECC_F16,
           torch.int32: ECC_I32, torch.float64: ECC_F64, torch.bfloat16: ECC_BF16, torch.int16: ECC_I16}


class EccError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"ecc status {status}: {message}")
        self.status = status


def ecc_last_error() -> str:
    return _lib.load().ecc_last_error().decode()


def _check(status: int):
    if status != 0:
        raise EccError(status, ecc_last_error())


def _dims(shape):
    arr = (ctypes.c_int64 * len(shape))(*shape)
    return arr


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _need_device(*tensors):
    for t in tensors:
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise ValueError("tensors must be contiguous device tensors")


def ecc_workspace_bytes(item_shape, batch: int, bins_or_T: int) -> int:
    return int(_lib.load().ecc_workspace_bytes(len(item_shape), _dims(item_shape), batch, bins_or_T))


def ecc_workspace_bytes_dtype(item_shape, batch: int, dtype: int, bins: int) -> int:
    return int(_lib.load().ecc_workspace_bytes_dtype(len(item_shape), _dims(item_shape), batch, dtype, bins))


# Workspaces handed out when the caller passes none: one per (device, stream), grown on demand
# and kept, so that repeated calls allocate nothing.  Calls on one stream run in order and may
# share it; calls on different streams get different ones.
_WS_CACHE = {}


def _cached_workspace(need: int, device) -> torch.Tensor:
    key = (torch.device(device).index, torch.cuda.current_stream().cuda_stream)
    ws = _WS_CACHE.get(key)
    if ws is None or ws.numel() < need:
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
        _WS_CACHE[key] = ws
    return ws


def _workspace(item_shape, batch, n, device, workspace, dtype=ECC_F32):
    if workspace is None:
        workspace = _cached_workspace(ecc_workspace_bytes_dtype(item_shape, batch, dtype, n), device)
    return workspace


def _need_f32(grid, u, tau, ndim):
    for name, t in (("grid", grid), ("u", u), ("tau", tau)):
        if t.dtype != torch.float32:
            raise ValueError(f"{name} must be float32, got {t.dtype}")
    if grid.dim() != ndim + 1:
        raise ValueError("grid must be [batch, *item_shape]")
    if u.numel() != ndim:
        raise ValueError(f"u must have {ndim} elements, got {u.numel()}")


ECC_VERTEX, ECC_TOPCELL = 0, 1
ECC_SUBLEVEL, ECC_SUPERLEVEL = 0, 1


def _hard_args(grid, ndim, bins, range, curve, workspace):
    """Marshalling shared by the hard entry points: (head, tail, curve) of the C call's arguments."""
    _need_device(grid, curve, workspace)
    if grid.dim() != ndim + 1:
        raise ValueError("grid must be [batch, *item_shape]")
    batch, item = grid.shape[0], tuple(grid.shape[1:])
    if curve is None:
        curve = torch.empty((batch, bins), dtype=torch.int64, device=grid.device)
    workspace = _workspace(item, batch, max(bins, 1), grid.device, workspace, _DTYPES[grid.dtype])
    rng = None
    if range is not None:
        rng = (ctypes.c_double * 2)(float(range[0]), float(range[1]))
    head = (_ptr(grid), ndim, _dims(item), batch, _DTYPES[grid.dtype])
    tail = (bins, rng, _ptr(curve), _ptr(workspace), workspace.numel(), _stream())
    return head, tail, curve


def ecc_hard(grid: torch.Tensor, ndim: int, bins: int, range=None, curve=None, workspace=None, top=False,
             superlevel=False):
    """grid: [batch, (D,) H, W] device tensor (uint8 / uint16 / float32; float16 / bfloat16 / int16 / int32 /
    float64 for the hard curves).  Returns the int64 curve [batch, bins].  top=True: top-cell construction
    (ecc_hard_top); superlevel=True: superlevel sets read at the lower bin edges (ecc_hard_ex)."""
    head, tail, curve = _hard_args(grid, ndim, bins, range, curve, workspace)
    if superlevel:
        _check(_lib.load().ecc_hard_ex(*head, ECC_TOPCELL if top else ECC_VERTEX, ECC_SUPERLEVEL, *tail))
    else:
        fn = _lib.load().ecc_hard_top if top else _lib.load().ecc_hard
        _check(fn(*head, *tail))
    return curve


def ecc_hard_static(grid: torch.Tensor, ndim: int, bins: int, range=None, curve=None):
    """ecc_hard on the library's static scratch (no workspace, no allocation inside the library);
    pass `curve` to keep this binding from allocating the output."""
    _need_device(grid, curve)
    if grid.dim() != ndim + 1:
        raise ValueError("grid must be [batch, *item_shape]")
    batch, item = grid.shape[0], tuple(grid.shape[1:])
    if curve is None:
        curve = torch.empty((batch, bins), dtype=torch.int64, device=grid.device)
    rng = None
    if range is not None:
        rng = (ctypes.c_double * 2)(float(range[0]), float(range[1]))
    _check(_lib.load().ecc_hard_static(_ptr(grid), ndim, _dims(item), batch, _DTYPES[grid.dtype], bins, rng,
                                       _ptr(curve), _stream()))
    return curve


def ecc_hard_ex(grid: torch.Tensor, ndim: int, construction: int, filtration: int, bins: int, range=None,
                curve=None, workspace=None):
    """The entry point with construction (ECC_VERTEX / ECC_TOPCELL) and filtration
    (ECC_SUBLEVEL / ECC_SUPERLEVEL) as arguments; every combination goes through ecc_hard_ex."""
    head, tail, curve = _hard_args(grid, ndim, bins, range, curve, workspace)
    _check(_lib.load().ecc_hard_ex(*head, int(construction), int(filtration), *tail))
    return curve


def ecc_hard_top(grid: torch.Tensor, ndim: int, bins: int, range=None, curve=None, workspace=None):
    """Hard ECC of the top-cell construction (grid points are squares / cubes)."""
    return ecc_hard(grid, ndim, bins, range=range, curve=curve, workspace=workspace, top=True)


def ecc_workspace_bytes_dir(item_shape, batch: int, ndir: int, bins: int) -> int:
    return int(_lib.load().ecc_workspace_bytes_dir(len(item_shape), _dims(item_shape), batch, ndir, bins))


def ecc_hard_dir(grid: torch.Tensor, ndim: int, u: torch.Tensor, alpha: float, bins: int, range=None,
                 curve=None, workspace=None):
    """Directional curves: grid [batch, (D,) H, W] float32, u [ndir, ndim] float32, both on the
    device.  Returns the int64 curves [ndir, batch, bins] of the tilted fields."""
    _need_device(grid, u, curve, workspace)
    if grid.dim() != ndim + 1 or u.dim() != 2 or u.shape[1] != ndim:
        raise ValueError("grid must be [batch, *item_shape] and u [ndir, ndim]")
    if grid.dtype != torch.float32 or u.dtype != torch.float32:
        raise ValueError("grid and u must be float32")
    batch, item = grid.shape[0], tuple(grid.shape[1:])
    ndir = u.shape[0]
    if curve is None:
        curve = torch.empty((ndir, batch, bins), dtype=torch.int64, device=grid.device)
    if workspace is None:
        workspace = _cached_workspace(ecc_workspace_bytes_dir(item, batch, ndir, bins), grid.device)
    rng = None
    if range is not None:
        rng = (ctypes.c_double * 2)(float(range[0]), float(range[1]))
    _check(_lib.load().ecc_hard_dir(_ptr(grid), ndim, _dims(item), batch, _ptr(u.contiguous()), ndir,
                                    float(alpha), bins, rng, _ptr(curve), _ptr(workspace), workspace.numel(),
                                    _stream()))
    return curve


def ecc_coeff(grid: torch.Tensor, ndim: int, c_out=None):
    _need_device(grid, c_out)
    batch, item = grid.shape[0], tuple(grid.shape[1:])
    if c_out is None:
        c_out = torch.empty(grid.shape, dtype=torch.int8, device=grid.device)
    _check(_lib.load().ecc_coeff(_ptr(grid), ndim, _dims(item), batch, _DTYPES[grid.dtype],
                                 _ptr(c_out), _stream()))
    return c_out


def ecc_soft_fwd(grid, ndim, u, alpha, tau, lam, chi=None, workspace=None, tilted_c=False):
    """tilted_c=True: c(p) of the tilted field X + alpha <u,p> (ecc_soft_fwd_tilted)."""
    _need_device(grid, u, tau, chi, workspace)
    _need_f32(grid, u, tau, ndim)
    batch, item = grid.shape[0], tuple(grid.shape[1:])
    T = tau.numel()
    if chi is None:
        chi = torch.empty((batch, T), dtype=torch.float32, device=grid.device)
    workspace = _workspace(item, batch, max(T, 1), grid.device, workspace)
    fn = _lib.load().ecc_soft_fwd_tilted if tilted_c else _lib.load().ecc_soft_fwd
    _check(fn(_ptr(grid), ndim, _dims(item), batch, _ptr(u), float(alpha), _ptr(tau), T, float(lam), _ptr(chi),
              _ptr(workspace), workspace.numel(), _stream()))
    return chi


def ecc_soft_bwd(grid, ndim, u, alpha, tau, lam, grad_chi=None, grad_X=None, dchi_dtau=None,
                 dchi_du=None, workspace=None, tilted_c=False, skip=()):
    """Returns (grad_X [batch,*item], dchi_dtau [batch,T], dchi_du [batch,T,ndim]).
    skip: names among "grad_X", "dchi_dtau", "dchi_du" of outputs that are not wanted (the
    library is handed NULL for them and None is returned in their place); not all three."""
    _need_device(grid, u, tau, grad_chi, grad_X, dchi_dtau, dchi_du, workspace)
    _need_f32(grid, u, tau, ndim)
    if grad_chi is not None and grad_chi.dtype != torch.float32:
        raise ValueError("grad_chi must be float32")
    batch, item = grid.shape[0], tuple(grid.shape[1:])
    T = tau.numel()
    dev = grid.device
    if grad_X is None and "grad_X" not in skip:
        grad_X = torch.empty(grid.shape, dtype=torch.float32, device=dev)
    if dchi_dtau is None and "dchi_dtau" not in skip:
        dchi_dtau = torch.empty((batch, T), dtype=torch.float32, device=dev)
    if dchi_du is None and "dchi_du" not in skip:
        dchi_du = torch.empty((batch, T, ndim), dtype=torch.float32, device=dev)
    workspace = _workspace(item, batch, max(T, 1), dev, workspace)
    fn = _lib.load().ecc_soft_bwd_tilted if tilted_c else _lib.load().ecc_soft_bwd
    _check(fn(_ptr(grid), ndim, _dims(item), batch, _ptr(u), float(alpha), _ptr(tau), T, float(lam),
              _ptr(grad_chi), _ptr(grad_X), _ptr(dchi_dtau), _ptr(dchi_du), _ptr(workspace),
              workspace.numel(), _stream()))
    return grad_X, dchi_dtau, dchi_du


def ecc_soft_state_bytes(item_shape, batch: int) -> int:
    return int(_lib.load().ecc_soft_state_bytes(len(item_shape), _dims(item_shape), batch))


def ecc_soft_fwd_save(grid, ndim, u, alpha, tau, lam, chi=None, dchi_dtau=None, dchi_du=None, state=None,
                      workspace=None, tilted_c=False, want=("dchi_dtau", "dchi_du")):
    """Forward pass that also returns the threshold / direction derivatives named in `want` and
    leaves the critical vertices in `state` for ecc_soft_bwd_saved.
    Returns (chi, dchi_dtau or None, dchi_du or None, state)."""
    _need_device(grid, u, tau, chi, dchi_dtau, dchi_du, state, workspace)
    _need_f32(grid, u, tau, ndim)
    batch, item = grid.shape[0], tuple(grid.shape[1:])
    T = tau.numel()
    dev = grid.device
    if chi is None:
        chi = torch.empty((batch, T), dtype=torch.float32, device=dev)
    if dchi_dtau is None and "dchi_dtau" in want:
        dchi_dtau = torch.empty((batch, T), dtype=torch.float32, device=dev)
    if dchi_du is None and "dchi_du" in want:
        dchi_du = torch.empty((batch, T, ndim), dtype=torch.float32, device=dev)
    if state is None:
        state = torch.empty(max(ecc_soft_state_bytes(item, batch), 256), dtype=torch.uint8, device=dev)
    workspace = _workspace(item, batch, max(T, 1), dev, workspace)
    _check(_lib.load().ecc_soft_fwd_save(_ptr(grid), ndim, _dims(item), batch, _ptr(u), float(alpha), _ptr(tau), T,
                                         float(lam), int(bool(tilted_c)), _ptr(chi), _ptr(dchi_dtau), _ptr(dchi_du),
                                         _ptr(state), state.numel(), _ptr(workspace), workspace.numel(), _stream()))
    return chi, dchi_dtau, dchi_du, state


def ecc_soft_bwd_saved(grid, ndim, u, alpha, tau, lam, state, grad_chi=None, grad_X=None, workspace=None,
                       tilted_c=False):
    """grad_X [batch, *item] from the state an ecc_soft_fwd_save call on the same grid, u, alpha left."""
    _need_device(grid, u, tau, grad_chi, grad_X, state, workspace)
    _need_f32(grid, u, tau, ndim)
    if grad_chi is not None and grad_chi.dtype != torch.float32:
        raise ValueError("grad_chi must be float32")
    batch, item = grid.shape[0], tuple(grid.shape[1:])
    T = tau.numel()
    if grad_X is None:
        grad_X = torch.empty(grid.shape, dtype=torch.float32, device=grid.device)
    workspace = _workspace(item, batch, max(T, 1), grid.device, workspace)
    _check(_lib.load().ecc_soft_bwd_saved(_ptr(grid), ndim, _dims(item), batch, _ptr(u), float(alpha), _ptr(tau), T,
                                          float(lam), int(bool(tilted_c)), _ptr(grad_chi), _ptr(grad_X), _ptr(state),
                                          state.numel(), _ptr(workspace), workspace.numel(), _stream()))
    return grad_X


def ecc_count_nonfinite(grid: torch.Tensor, count=None):
    """Number of NaN / Inf elements of a device tensor, as a device int64 scalar tensor (no sync)."""
    _need_device(grid, count)
    if count is None:
        count = torch.empty((), dtype=torch.int64, device=grid.device)
    _check(_lib.load().ecc_count_nonfinite(_ptr(grid), grid.numel(), _DTYPES[grid.dtype], _ptr(count), _stream()))
    return count


ECC_FORCE_GENERIC, ECC_FORCE_TWO_PASS, ECC_FORCE_SOFT_TILES, ECC_FORCE_NO_SMALL = 1, 2, 4, 8


def ecc_debug_force(mask: int) -> int:
    """Test aid: force the fall-back kernels (OR of ECC_FORCE_*; 0 = normal).  Returns the previous mask."""
    return int(_lib.load().ecc_debug_force(int(mask)))


def ecc_profile_begin(max_launches: int = 256):
    _check(_lib.load().ecc_profile_begin(int(max_launches)))


def ecc_profile_end():
    """Returns (mean sweep-kernel milliseconds, launches measured)."""
    ms, n = ctypes.c_float(0), ctypes.c_int(0)
    _check(_lib.load().ecc_profile_end(ctypes.byref(ms), ctypes.byref(n)))
    return float(ms.value), int(n.value)
