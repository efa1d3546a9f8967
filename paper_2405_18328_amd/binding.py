"""ctypes binding of libgpws.so: argument marshalling only.

Every function has the name and argument order of its C entry point in
include/gpws.h; torch tensors are accepted wherever the C side takes a device
pointer (their data_ptr() is passed, nothing is copied or computed here).
There is no fallback: if the HIP library is missing or fails to load, importing
this module raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

GP_SE_ARD = 0
GP_MATERN32_ARD = 1
GP_OK = 0
GP_NOT_CONVERGED = 1
GP_ERR_ARG = -1
GP_ERR_HIP = -2
GP_ERR_WORKSPACE = -3
GP_ERR_BREAKDOWN = -4
GP_MAX_D = 126
GP_MAX_T = 1024

# GPWS_LIB names another build of the library (developer aid for side-by-side timing of two builds)
LIB_PATH = os.environ.get("GPWS_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libgpws.so")

GP_AP_MAX_BLOCK = 2048

EXPORTS = ["gp_create", "gp_destroy", "gp_set_theta", "gp_kmv", "gp_kmv_static", "gp_workspace_bytes", "gp_cg_solve",
           "gp_ap_workspace_bytes", "gp_ap_solve", "gp_sgd_workspace_bytes", "gp_sgd_solve", "gp_mll_grad", "gp_predict", "gp_profile", "gp_profile_read", "gp_profile_read_kind", "gp_product_path", "gp_last_error"]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = C.CDLL(LIB_PATH)
    p, i64, i32, dbl, sz = C.c_void_p, C.c_int64, C.c_int, C.c_double, C.c_size_t
    lib.gp_create.argtypes = [C.POINTER(p), i32, i64, i32, p, p]
    lib.gp_destroy.argtypes = [p]
    lib.gp_set_theta.argtypes = [p, C.POINTER(dbl), dbl, dbl]
    lib.gp_kmv.argtypes = [p, p, i64, i32, p, i64, i32]
    lib.gp_kmv_static.argtypes = [p, p, i64, i32, p, i64, i32]
    lib.gp_workspace_bytes.argtypes = [p, i32]
    lib.gp_workspace_bytes.restype = sz
    lib.gp_cg_solve.argtypes = [p, p, i64, p, p, i64, i32, C.POINTER(C.c_float), i32, p, sz,
                                C.POINTER(i32), C.POINTER(i32), C.POINTER(C.c_float)]
    lib.gp_ap_workspace_bytes.argtypes = [p, i32, i32]
    lib.gp_ap_workspace_bytes.restype = sz
    lib.gp_ap_solve.argtypes = [p, p, i64, p, p, i64, i32, C.POINTER(C.c_float), i32, i32, p, sz,
                                C.POINTER(i32), C.POINTER(i32), C.POINTER(C.c_float), C.POINTER(i32)]
    lib.gp_sgd_workspace_bytes.argtypes = [p, i32, i32]
    lib.gp_sgd_workspace_bytes.restype = sz
    lib.gp_sgd_solve.argtypes = [p, p, i64, p, p, i64, i32, C.POINTER(C.c_float), p, i32, i32, dbl, dbl, p, sz,
                                 C.POINTER(i32), C.POINTER(i32), C.POINTER(C.c_float)]
    lib.gp_mll_grad.argtypes = [p, p, i64, p, i64, i32, C.POINTER(dbl)]
    lib.gp_predict.argtypes = [p, p, i64, p, i64, i32, p, i64]
    lib.gp_profile.argtypes = [p, i32]
    lib.gp_profile_read.argtypes = [p, C.POINTER(i32), C.POINTER(dbl)]
    lib.gp_profile_read_kind.argtypes = [p, i32, C.POINTER(i32), C.POINTER(dbl)]
    lib.gp_product_path.argtypes = [p]
    lib.gp_last_error.argtypes = [p]
    lib.gp_last_error.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("gp_workspace_bytes", "gp_ap_workspace_bytes", "gp_sgd_workspace_bytes", "gp_last_error"):
            getattr(lib, name).restype = i32
    return lib


_lib = _load()


def _ptr(x):
    """Device (or NULL) pointer of a torch tensor / int / None."""
    if x is None:
        return None
    if isinstance(x, torch.Tensor):
        return x.data_ptr()
    return int(x)


class GpError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libgpws error {code}: {msg}")
        self.code = code


def gp_last_error(ctx):
    return _lib.gp_last_error(ctx).decode()


def _check(ctx, rc):
    if rc < 0:
        raise GpError(rc, gp_last_error(ctx) if ctx else "invalid arguments")
    return rc


def gp_create(kernel, n, d, dX, hip_stream=None):
    """Returns the opaque context handle (an int)."""
    ctx = C.c_void_p()
    rc = _lib.gp_create(C.byref(ctx), int(kernel), int(n), int(d), _ptr(dX), _ptr(hip_stream))
    if rc < 0:
        msg = gp_last_error(ctx) if ctx.value else "invalid arguments"
        if ctx.value:
            _lib.gp_destroy(ctx)
        raise GpError(rc, msg)
    return ctx


def gp_destroy(ctx):
    return _lib.gp_destroy(ctx)


def gp_set_theta(ctx, lengthscale, signal_scale, noise_scale):
    ell = np.ascontiguousarray(lengthscale, dtype=np.float64)
    return _check(ctx, _lib.gp_set_theta(ctx, ell.ctypes.data_as(C.POINTER(C.c_double)),
                                         float(signal_scale), float(noise_scale)))


def gp_kmv(ctx, dV, ldv, t, dOut, ldo, add_noise):
    return _check(ctx, _lib.gp_kmv(ctx, _ptr(dV), int(ldv), int(t), _ptr(dOut), int(ldo), int(add_noise)))


GP_KMV_STATIC_SCRATCH_BYTES = 64 << 20


def gp_kmv_static(ctx, dV, ldv, t, dOut, ldo, add_noise):
    return _check(ctx, _lib.gp_kmv_static(ctx, _ptr(dV), int(ldv), int(t), _ptr(dOut), int(ldo), int(add_noise)))


def gp_workspace_bytes(ctx, t):
    return int(_lib.gp_workspace_bytes(ctx, int(t)))


def gp_cg_solve(ctx, dB, ldb, dX0, dV, ldv, t, tol, max_iters, dWork, work_bytes):
    """Returns (rc, iters, kmv_count, relres[t]); raises GpError on rc < 0."""
    tol_arr = np.ascontiguousarray(np.broadcast_to(np.asarray(tol, dtype=np.float32), (t,)))
    iters, kmv = C.c_int(0), C.c_int(0)
    relres = np.zeros(t, dtype=np.float32)
    rc = _lib.gp_cg_solve(ctx, _ptr(dB), int(ldb), _ptr(dX0), _ptr(dV), int(ldv), int(t),
                          tol_arr.ctypes.data_as(C.POINTER(C.c_float)), int(max_iters), _ptr(dWork),
                          int(work_bytes), C.byref(iters), C.byref(kmv),
                          relres.ctypes.data_as(C.POINTER(C.c_float)))
    _check(ctx, rc)
    return rc, iters.value, kmv.value, relres


def gp_ap_workspace_bytes(ctx, t, block):
    return int(_lib.gp_ap_workspace_bytes(ctx, int(t), int(block)))


def gp_ap_solve(ctx, dB, ldb, dX0, dV, ldv, t, tol, block, max_iters, dWork, work_bytes, want_picks=False):
    """Returns (rc, iters, kmv_count, relres[t], picks or None); raises GpError on rc < 0."""
    tol_arr = np.ascontiguousarray(np.broadcast_to(np.asarray(tol, dtype=np.float32), (t,)))
    iters, kmv = C.c_int(0), C.c_int(0)
    relres = np.zeros(t, dtype=np.float32)
    picks = np.full(max(int(max_iters), 1), -1, dtype=np.int32) if want_picks else None
    rc = _lib.gp_ap_solve(ctx, _ptr(dB), int(ldb), _ptr(dX0), _ptr(dV), int(ldv), int(t),
                          tol_arr.ctypes.data_as(C.POINTER(C.c_float)), int(block), int(max_iters), _ptr(dWork),
                          int(work_bytes), C.byref(iters), C.byref(kmv),
                          relres.ctypes.data_as(C.POINTER(C.c_float)),
                          picks.ctypes.data_as(C.POINTER(C.c_int)) if want_picks else None)
    _check(ctx, rc)
    return rc, iters.value, kmv.value, relres, (picks[:iters.value] if want_picks else None)


def gp_sgd_workspace_bytes(ctx, t, batch):
    return int(_lib.gp_sgd_workspace_bytes(ctx, int(t), int(batch)))


def gp_sgd_solve(ctx, dB, ldb, dX0, dV, ldv, t, tol, dBatches, batch, max_iters, lr, momentum, dWork, work_bytes):
    """dBatches: device int32 [max_iters, batch].  Returns (rc, iters, kmv_count, relres_est[t]); raises GpError on rc < 0."""
    tol_arr = np.ascontiguousarray(np.broadcast_to(np.asarray(tol, dtype=np.float32), (t,)))
    iters, kmv = C.c_int(0), C.c_int(0)
    relres = np.zeros(t, dtype=np.float32)
    rc = _lib.gp_sgd_solve(ctx, _ptr(dB), int(ldb), _ptr(dX0), _ptr(dV), int(ldv), int(t),
                           tol_arr.ctypes.data_as(C.POINTER(C.c_float)), _ptr(dBatches), int(batch), int(max_iters),
                           float(lr), float(momentum), _ptr(dWork), int(work_bytes), C.byref(iters), C.byref(kmv),
                           relres.ctypes.data_as(C.POINTER(C.c_float)))
    _check(ctx, rc)
    return rc, iters.value, kmv.value, relres


def gp_mll_grad(ctx, dV, ldv, dB, ldb, t, d):
    """Returns the d + 2 gradient entries as a float64 numpy array."""
    g = np.zeros(d + 2, dtype=np.float64)
    _check(ctx, _lib.gp_mll_grad(ctx, _ptr(dV), int(ldv), _ptr(dB), int(ldb), int(t),
                                 g.ctypes.data_as(C.POINTER(C.c_double))))
    return g


def gp_predict(ctx, dXstar, m, dV, ldv, t, dOut, ldo):
    return _check(ctx, _lib.gp_predict(ctx, _ptr(dXstar), int(m), _ptr(dV), int(ldv), int(t), _ptr(dOut), int(ldo)))


def gp_profile(ctx, enable):
    return _check(ctx, _lib.gp_profile(ctx, int(enable)))


def gp_product_path(ctx):
    rc = _lib.gp_product_path(ctx)
    if rc < 0:
        raise GpError(rc, "gp_product_path: no theta set")
    return rc


GP_PROF_TILE, GP_PROF_CG_DOT, GP_PROF_CG_XR, GP_PROF_CG_P, GP_PROF_GRAD_TILE = range(5)
GP_PROF_KINDS = 5


def gp_profile_read_kind(ctx, kind):
    """Returns (launches, total_ms) of the bracketed launches of one kind (GP_PROF_*)."""
    n, ms = C.c_int(0), C.c_double(0.0)
    _check(ctx, _lib.gp_profile_read_kind(ctx, int(kind), C.byref(n), C.byref(ms)))
    return n.value, ms.value


def gp_profile_read(ctx):
    """Returns (launches, total_ms) of the bracketed tile-pass launches."""
    n, ms = C.c_int(0), C.c_double(0.0)
    _check(ctx, _lib.gp_profile_read(ctx, C.byref(n), C.byref(ms)))
    return n.value, ms.value
