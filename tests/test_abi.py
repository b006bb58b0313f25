"""The C-ABI library loads, exports every symbol include/ecc.h declares, and
rejects bad arguments on the host before any HIP call (so this runs without a
GPU; no compute call is made here)."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2510_20271_amd import _lib

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(0x1000)  # non-NULL, 256-aligned, never dereferenced: validation fails first


def _declared():
    text = open(os.path.join(ROOT, "include", "ecc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ecc_[a-z_]+)\s*\(", text)))


def test_exports_match_header():
    lib = _lib.load()
    names = _declared()
    assert set(names) == set(_lib.SIGNATURES), names
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_error_string():
    lib = _lib.load()
    assert b"gfx950" in lib.ecc_version()
    assert isinstance(lib.ecc_last_error(), bytes)


def _dims(*d):
    return (ctypes.c_int64 * len(d))(*d)


def test_workspace_bytes_host_only():
    lib = _lib.load()
    assert lib.ecc_workspace_bytes(2, _dims(256, 256), 1, 256) >= 256 + 4 * 256
    assert lib.ecc_workspace_bytes(4, _dims(2, 2, 2, 2), 1, 8) == 0
    assert lib.ecc_workspace_bytes(2, _dims(0, 5), 1, 8) == 0
    assert lib.ecc_workspace_bytes(2, _dims(5, 5), 0, 8) == 0
    assert lib.ecc_workspace_bytes(2, _dims(5, 5), 1, 0) == 0
    # soft partials dominate for many tiles
    big = lib.ecc_workspace_bytes(2, _dims(512, 512), 32, 128)
    assert big >= 32 * 128 * 128 * 16


def test_workspace_bytes_of_the_hard_flows():
    # small inputs: a list slot per vertex (8 bytes) and a head per stage block
    lib = _lib.load()
    n = 256 * 256
    # (a 256-wide image is two strips of 248 columns to the sweep: its blocks own up to twice its vertices)
    assert 8 * n <= lib.ecc_workspace_bytes(2, _dims(256, 256), 1, 64) <= 16 * n + (1 << 16)
    # mid-sized batches (up to 2^27 vertices in images, 2^25 in volumes): room for every vertex of every
    # sweep block, rounded up to whole blocks
    for nd, dims, batch in ((2, (1024, 1024), 1), (2, (512, 512), 32), (2, (4096, 4096), 8), (3, (256, 256, 256), 2)):
        n = int(np.prod(dims)) * batch
        w = lib.ecc_workspace_bytes(nd, _dims(*dims), batch, 1024)
        assert 8 * n <= w <= 12 * n, (dims, batch, w / n)
    # beyond: one byte per vertex for the shared lists (the soft partial sums of a call with T = 1024 aside)
    for nd, dims, batch in ((2, (4096, 4096), 16), (3, (512, 512, 512), 1), (2, (224, 224), 5000)):
        n = int(np.prod(dims)) * batch
        w = lib.ecc_workspace_bytes(nd, _dims(*dims), batch, 8)
        assert n <= w <= 2 * n, (dims, batch, w / n)


INVALID, UNSUPPORTED, WORKSPACE, RANGE = -1, -2, -3, -4


@pytest.mark.parametrize("kw,status,word", [
    (dict(ndim=4), INVALID, "ndim"),
    (dict(dims=(0, 4)), INVALID, "dims"),
    (dict(batch=0), INVALID, "batch"),
    (dict(batch=70000), UNSUPPORTED, "batch"),
    (dict(dtype=9), INVALID, "dtype"),
    (dict(grid=None), INVALID, "grid"),
    (dict(curve=None), INVALID, "curve"),
    (dict(bins=0), INVALID, "bins"),
    (dict(bins=1 << 20), UNSUPPORTED, "bins"),
    (dict(range=(2.0, 1.0)), RANGE, "range"),
    (dict(range=(float("nan"), 1.0)), RANGE, "range"),
    (dict(range=(0.0, float("inf"))), RANGE, "range"),
    (dict(ws=None), WORKSPACE, "workspace"),
    (dict(ws_bytes=8), WORKSPACE, "workspace"),
    (dict(ws=ctypes.c_void_p(0x1004)), WORKSPACE, "aligned"),
    (dict(grid=ctypes.c_void_p(0x1001), dtype=2), INVALID, "aligned"),
])
def test_hard_rejects_bad_arguments(kw, status, word):
    lib = _lib.load()
    a = dict(grid=FAKE, ndim=2, dims=(4, 4), batch=1, dtype=0, bins=8, range=None, curve=FAKE, ws=FAKE,
             ws_bytes=1 << 20)
    a.update(kw)
    rng = None if a["range"] is None else (ctypes.c_double * 2)(*a["range"])
    rc = lib.ecc_hard(a["grid"], a["ndim"], _dims(*a["dims"]), a["batch"], a["dtype"], a["bins"], rng,
                      a["curve"], a["ws"], a["ws_bytes"], None)
    assert rc == status
    assert word in lib.ecc_last_error().decode()


@pytest.mark.parametrize("kw,status,word", [
    (dict(construction=2), INVALID, "construction"),
    (dict(filtration=-1), INVALID, "filtration"),
    (dict(bins=0), INVALID, "bins"),
    (dict(dtype=9), INVALID, "dtype"),
    (dict(ws_bytes=8), WORKSPACE, "workspace"),
])
def test_hard_ex_rejects_bad_arguments(kw, status, word):
    lib = _lib.load()
    a = dict(construction=1, filtration=1, bins=8, dtype=0, ws_bytes=1 << 20)
    a.update(kw)
    rc = lib.ecc_hard_ex(FAKE, 2, _dims(4, 4), 1, a["dtype"], a["construction"], a["filtration"], a["bins"], None,
                         FAKE, FAKE, a["ws_bytes"], None)
    assert rc == status
    assert word in lib.ecc_last_error().decode()


def test_workspace_bytes_dtype_host_only():
    lib = _lib.load()
    base = lib.ecc_workspace_bytes(2, _dims(100, 200), 3, 64)
    for dt in (0, 1, 2):
        assert lib.ecc_workspace_bytes_dtype(2, _dims(100, 200), 3, dt, 64) == base
    for dt in (3, 4, 5, 6, 7):  # room for the float32 copy of the grid
        assert lib.ecc_workspace_bytes_dtype(2, _dims(100, 200), 3, dt, 64) >= base + 3 * 100 * 200 * 4
    assert lib.ecc_workspace_bytes_dtype(2, _dims(100, 200), 3, 8, 64) == 0
    # a converted type with only the plain workspace is refused; ecc_coeff does not take it at all
    rc = lib.ecc_hard(FAKE, 2, _dims(100, 200), 3, 5, 64, None, FAKE, FAKE, base, None)
    assert rc == WORKSPACE and "workspace" in lib.ecc_last_error().decode()
    rc = lib.ecc_coeff(FAKE, 2, _dims(4, 4), 1, 5, FAKE, None)
    assert rc == INVALID and "dtype" in lib.ecc_last_error().decode()
    rc = lib.ecc_hard(ctypes.c_void_p(0x1004), 2, _dims(4, 4), 1, 5, 8, None, FAKE, FAKE, 1 << 20, None)
    assert rc == INVALID and "aligned" in lib.ecc_last_error().decode()


def test_hard_rejects_null_dims():
    lib = _lib.load()
    rc = lib.ecc_hard(FAKE, 2, None, 1, 0, 8, None, FAKE, FAKE, 1 << 20, None)
    assert rc == INVALID and "dims" in lib.ecc_last_error().decode()


@pytest.mark.parametrize("kw,status,word", [
    (dict(ndim=1), INVALID, "ndim"),
    (dict(u=None), INVALID, "u is"),
    (dict(tau=None), INVALID, "tau"),
    (dict(T=0), INVALID, "T must"),
    (dict(T=1 << 20), UNSUPPORTED, "T "),
    (dict(lam=0.0), INVALID, "lambda"),
    (dict(lam=float("inf")), INVALID, "lambda"),
    (dict(alpha=float("nan")), INVALID, "alpha"),
    (dict(out=None), INVALID, "NULL"),
    (dict(ws_bytes=16), WORKSPACE, "workspace"),
    (dict(grid=ctypes.c_void_p(0x1002)), INVALID, "aligned"),
    (dict(tau=ctypes.c_void_p(0x1001)), INVALID, "aligned"),
    (dict(out=ctypes.c_void_p(0x1002)), INVALID, "aligned"),
])
def test_soft_rejects_bad_arguments(kw, status, word):
    lib = _lib.load()
    a = dict(grid=FAKE, ndim=2, dims=(4, 4), batch=1, u=FAKE, alpha=0.1, tau=FAKE, T=4, lam=2.0, out=FAKE,
             ws=FAKE, ws_bytes=1 << 20)
    a.update(kw)
    rc = lib.ecc_soft_fwd(a["grid"], a["ndim"], _dims(*a["dims"]), a["batch"], a["u"], a["alpha"], a["tau"],
                          a["T"], a["lam"], a["out"], a["ws"], a["ws_bytes"], None)
    assert rc == status, lib.ecc_last_error()
    assert word in lib.ecc_last_error().decode()
    rc = lib.ecc_soft_bwd(a["grid"], a["ndim"], _dims(*a["dims"]), a["batch"], a["u"], a["alpha"], a["tau"],
                          a["T"], a["lam"], None, a["out"], None, None, a["ws"], a["ws_bytes"], None)
    assert rc == status, lib.ecc_last_error()


@pytest.mark.parametrize("kw,status,word", [
    (dict(ndim=1), INVALID, "ndim"),
    (dict(grid=None), INVALID, "grid"),
    (dict(u=None), INVALID, "u is"),
    (dict(curve=None), INVALID, "curve"),
    (dict(ndir=0), INVALID, "ndir"),
    (dict(ndir=300, batch=300), UNSUPPORTED, "ndir * batch"),
    (dict(alpha=float("inf")), INVALID, "alpha"),
    (dict(bins=0), INVALID, "bins"),
    (dict(bins=1 << 20), UNSUPPORTED, "bins"),
    (dict(range=(3.0, 1.0)), RANGE, "range"),
    (dict(ws_bytes=8), WORKSPACE, "workspace"),
    (dict(u=ctypes.c_void_p(0x1002)), INVALID, "aligned"),
])
def test_hard_dir_rejects_bad_arguments(kw, status, word):
    lib = _lib.load()
    a = dict(grid=FAKE, ndim=2, dims=(4, 4), batch=1, u=FAKE, ndir=2, alpha=0.5, bins=8, range=None, curve=FAKE,
             ws=FAKE, ws_bytes=1 << 20)
    a.update(kw)
    rng = None if a["range"] is None else (ctypes.c_double * 2)(*a["range"])
    rc = lib.ecc_hard_dir(a["grid"], a["ndim"], _dims(*a["dims"]), a["batch"], a["u"], a["ndir"], a["alpha"],
                          a["bins"], rng, a["curve"], a["ws"], a["ws_bytes"], None)
    assert rc == status, lib.ecc_last_error()
    assert word in lib.ecc_last_error().decode()


def test_hard_dir_workspace_bytes_host_only():
    lib = _lib.load()
    one = lib.ecc_workspace_bytes_dir(2, _dims(300, 1000), 2, 1, 64)
    four = lib.ecc_workspace_bytes_dir(2, _dims(300, 1000), 2, 4, 64)
    assert 0 < one < four
    assert lib.ecc_workspace_bytes_dir(2, _dims(300, 1000), 2, 0, 64) == 0
    assert lib.ecc_workspace_bytes_dir(2, _dims(300, 1000), 300, 300, 64) == 0
    # shapes the strip sweep does not take also need room for the tilted fields
    tiny = lib.ecc_workspace_bytes_dir(2, _dims(50, 5), 1, 3, 64)
    assert tiny >= 3 * 50 * 5 * 4


def test_coeff_rejects_bad_arguments():
    lib = _lib.load()
    assert lib.ecc_coeff(None, 2, _dims(4, 4), 1, 0, FAKE, None) == INVALID
    assert lib.ecc_coeff(FAKE, 2, _dims(4, 4), 1, 0, None, None) == INVALID
    assert lib.ecc_coeff(FAKE, 5, _dims(4, 4), 1, 0, FAKE, None) == INVALID


def test_hard_static_rejects_on_the_host():
    lib = _lib.load()
    assert lib.ecc_hard_static(None, 2, _dims(4, 4), 1, 0, 8, None, FAKE, None) == INVALID
    assert lib.ecc_hard_static(FAKE, 2, _dims(4, 4), 1, 0, 0, None, FAKE, None) == INVALID
    assert lib.ecc_hard_static(FAKE, 2, _dims(4, 4), 1, 0, 8, (ctypes.c_double * 2)(2.0, 1.0), FAKE, None) == RANGE
    # more scratch than the static buffer holds: refused before any HIP call
    assert lib.ecc_workspace_bytes(2, _dims(8192, 8192), 1, 8) > 32 << 20
    assert lib.ecc_hard_static(FAKE, 2, _dims(8192, 8192), 1, 2, 8, None, FAKE, None) == UNSUPPORTED
    assert "scratch" in lib.ecc_last_error().decode()


def test_count_nonfinite_and_debug_force_host_side():
    lib = _lib.load()
    assert lib.ecc_count_nonfinite(None, 16, 2, FAKE, None) == INVALID
    assert lib.ecc_count_nonfinite(FAKE, 16, 2, None, None) == INVALID
    assert lib.ecc_count_nonfinite(FAKE, 0, 2, FAKE, None) == INVALID
    assert lib.ecc_count_nonfinite(FAKE, 16, 9, FAKE, None) == INVALID
    assert lib.ecc_count_nonfinite(ctypes.c_void_p(0x1002), 16, 2, FAKE, None) == INVALID
    assert lib.ecc_count_nonfinite(FAKE, 16, 2, ctypes.c_void_p(0x1004), None) == INVALID
    # the switch of the fall-back paths: returns the previous mask, ignores unknown bits
    assert lib.ecc_debug_force(3) == 0
    assert lib.ecc_debug_force(0xff) == 3
    assert lib.ecc_debug_force(0) == 15
    assert lib.ecc_debug_force(0) == 0


def test_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2510_20271_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.replace("CPU oracle", ""), f
