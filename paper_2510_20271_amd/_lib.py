"""ctypes loader for libecc_hip.so.  Fails loudly when the library is missing:
there is no CPU fallback."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
SO_PATH = os.path.join(_HERE, "libecc_hip.so")
_lib = None

c_i64 = ctypes.c_int64
c_vp = ctypes.c_void_p

# name -> (restype, argtypes); mirrors include/ecc.h
SIGNATURES = {
    "ecc_last_error": (ctypes.c_char_p, []),
    "ecc_version": (ctypes.c_char_p, []),
    "ecc_workspace_bytes": (ctypes.c_size_t, [ctypes.c_int, ctypes.POINTER(c_i64), c_i64, ctypes.c_int]),
    "ecc_workspace_bytes_dtype": (ctypes.c_size_t, [ctypes.c_int, ctypes.POINTER(c_i64), c_i64, ctypes.c_int,
                                                    ctypes.c_int]),
    "ecc_hard": (ctypes.c_int, [c_vp, ctypes.c_int, ctypes.POINTER(c_i64), c_i64, ctypes.c_int,
                                ctypes.c_int, ctypes.POINTER(ctypes.c_double), c_vp, c_vp,
                                ctypes.c_size_t, c_vp]),
    "ecc_hard_static": (ctypes.c_int, [c_vp, ctypes.c_int, ctypes.POINTER(c_i64), c_i64, ctypes.c_int,
                                       ctypes.c_int, ctypes.POINTER(ctypes.c_double), c_vp, c_vp]),
    "ecc_hard_top": (ctypes.c_int, [c_vp, ctypes.c_int, ctypes.POINTER(c_i64), c_i64, ctypes.c_int,
                                    ctypes.c_int, ctypes.POINTER(ctypes.c_double), c_vp, c_vp,
                                    ctypes.c_size_t, c_vp]),
    "ecc_hard_ex": (ctypes.c_int, [c_vp, ctypes.c_int, ctypes.POINTER(c_i64), c_i64, ctypes.c_int,
                                   ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double),
                                   c_vp, c_vp, ctypes.c_size_t, c_vp]),
    "ecc_coeff": (ctypes.c_int, [c_vp, ctypes.c_int, ctypes.POINTER(c_i64), c_i64, ctypes.c_int,
                                 c_vp, c_vp]),
    "ecc_soft_fwd": (ctypes.c_int, [c_vp, ctypes.c_int, ctypes.POINTER(c_i64), c_i64, c_vp,
                                    ctypes.c_float, c_vp, ctypes.c_int, ctypes.c_float, c_vp, c_vp,
                                    ctypes.c_size_t, c_vp]),
    "ecc_soft_bwd": (ctypes.c_int, [c_vp, ctypes.c_int, ctypes.POINTER(c_i64), c_i64, c_vp,
                                    ctypes.c_float, c_vp, ctypes.c_int, ctypes.c_float, c_vp, c_vp,
                                    c_vp, c_vp, c_vp, ctypes.c_size_t, c_vp]),
    "ecc_soft_state_bytes": (ctypes.c_size_t, [ctypes.c_int, ctypes.POINTER(c_i64), c_i64]),
    "ecc_soft_fwd_save": (ctypes.c_int, [c_vp, ctypes.c_int, ctypes.POINTER(c_i64), c_i64, c_vp, ctypes.c_float,
                                         c_vp, ctypes.c_int, ctypes.c_float, ctypes.c_int, c_vp, c_vp, c_vp, c_vp,
                                         ctypes.c_size_t, c_vp, ctypes.c_size_t, c_vp]),
    "ecc_soft_bwd_saved": (ctypes.c_int, [c_vp, ctypes.c_int, ctypes.POINTER(c_i64), c_i64, c_vp, ctypes.c_float,
                                          c_vp, ctypes.c_int, ctypes.c_float, ctypes.c_int, c_vp, c_vp, c_vp,
                                          ctypes.c_size_t, c_vp, ctypes.c_size_t, c_vp]),
    "ecc_soft_fwd_tilted": (ctypes.c_int, [c_vp, ctypes.c_int, ctypes.POINTER(c_i64), c_i64, c_vp,
                                           ctypes.c_float, c_vp, ctypes.c_int, ctypes.c_float, c_vp, c_vp,
                                           ctypes.c_size_t, c_vp]),
    "ecc_soft_bwd_tilted": (ctypes.c_int, [c_vp, ctypes.c_int, ctypes.POINTER(c_i64), c_i64, c_vp,
                                           ctypes.c_float, c_vp, ctypes.c_int, ctypes.c_float, c_vp, c_vp,
                                           c_vp, c_vp, c_vp, ctypes.c_size_t, c_vp]),
    "ecc_workspace_bytes_dir": (ctypes.c_size_t, [ctypes.c_int, ctypes.POINTER(c_i64), c_i64, ctypes.c_int,
                                                  ctypes.c_int]),
    "ecc_hard_dir": (ctypes.c_int, [c_vp, ctypes.c_int, ctypes.POINTER(c_i64), c_i64, c_vp, ctypes.c_int,
                                    ctypes.c_float, ctypes.c_int, ctypes.POINTER(ctypes.c_double), c_vp, c_vp,
                                    ctypes.c_size_t, c_vp]),
    "ecc_count_nonfinite": (ctypes.c_int, [c_vp, c_i64, ctypes.c_int, c_vp, c_vp]),
    "ecc_debug_force": (ctypes.c_uint, [ctypes.c_uint]),
    "ecc_profile_begin": (ctypes.c_int, [ctypes.c_int]),
    "ecc_profile_end": (ctypes.c_int, [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int)]),
}


def load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(SO_PATH):
            raise RuntimeError(
                f"{SO_PATH} is missing: build it with `python -m paper_2510_20271_amd.build` "
                "(hipcc, gfx950). There is no CPU fallback.")
        lib = ctypes.CDLL(SO_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib
