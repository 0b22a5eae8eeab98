"""ctypes loader for the fp64 CPU oracle (oracle/ziplm_oracle.c).

TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's CPU-baseline
leg may import this module.  The product package never does.

All arrays are numpy float64, C-contiguous, host memory.  Inputs are copied, so
callers keep their arrays.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libziplm_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (seconds)."""
    src = os.path.join(_HERE, "ziplm_oracle.c")
    if (not force and os.path.exists(_LIB_PATH)
            and os.path.getmtime(_LIB_PATH) >= os.path.getmtime(src)):
        return _LIB_PATH
    subprocess.check_call(["sh", os.path.join(_HERE, "build.sh")])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB_PATH)
    dp = ctypes.POINTER(ctypes.c_double)
    ip = ctypes.POINTER(ctypes.c_int32)
    bp = ctypes.POINTER(ctypes.c_uint8)
    lib.ziplm_oracle_hessian.restype = ctypes.c_int
    lib.ziplm_oracle_hessian.argtypes = [dp, dp, ctypes.c_int, ctypes.c_int64, ctypes.c_double]
    lib.ziplm_oracle_hinv.restype = ctypes.c_int
    lib.ziplm_oracle_hinv.argtypes = [dp, dp, ctypes.c_int, ctypes.c_double, dp,
                                      ctypes.POINTER(ctypes.c_int)]
    lib.ziplm_oracle_prune.restype = ctypes.c_int
    lib.ziplm_oracle_prune.argtypes = [dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                       ctypes.c_int, bp, ip, ip, dp, dp, dp,
                                       ctypes.c_int, ip, dp]
    lib.ziplm_oracle_threads.restype = ctypes.c_int
    lib.ziplm_oracle_threads.argtypes = []
    lib.ziplm_oracle_module_error.restype = ctypes.c_int
    lib.ziplm_oracle_module_error.argtypes = [dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_double, dp]
    lib.ziplm_oracle_prior.restype = ctypes.c_int
    lib.ziplm_oracle_prior.argtypes = [dp, ctypes.c_int, ctypes.c_double, dp]
    _lib = lib
    return lib


def threads():
    """OpenMP threads the oracle's loops use."""
    return int(_load().ziplm_oracle_threads())


class OracleError(RuntimeError):
    def __init__(self, code, info=None):
        super().__init__("oracle status %d (info=%s)" % (code, info))
        self.code = code
        self.info = info


def _f64(a):
    return np.ascontiguousarray(np.array(a, dtype=np.float64, copy=True))


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def hessian(X, scale=2.0, H=None):
    """H (+)= scale * X X^T for X of shape (d_col, n_tok)."""
    lib = _load()
    X = _f64(X)
    d, n = X.shape
    H = np.zeros((d, d), dtype=np.float64) if H is None else _f64(H)
    rc = lib.ziplm_oracle_hessian(_ptr(H, ctypes.c_double), _ptr(X, ctypes.c_double), d, n,
                                  float(scale))
    if rc:
        raise OracleError(rc)
    return H


def hinv(H, damp_rel=0.01):
    """Returns (Hinv, lambda) with Hinv = (H + lambda I)^-1, lambda = damp_rel*mean(diag H)."""
    lib = _load()
    H = _f64(H)
    d = H.shape[0]
    assert H.shape == (d, d)
    out = np.empty((d, d), dtype=np.float64)
    lam = ctypes.c_double(0.0)
    info = ctypes.c_int(0)
    rc = lib.ziplm_oracle_hinv(_ptr(H, ctypes.c_double), _ptr(out, ctypes.c_double), d,
                               float(damp_rel), ctypes.byref(lam), ctypes.byref(info))
    if rc:
        raise OracleError(rc, info.value)
    return out, lam.value


def prune(W, Hinv, group_size, n_remove, alive=None, forced=None, snap_steps=None):
    """Algorithm 1.  Returns a dict with W, Hinv (updated copies), order, err, best, gap,
    and W_snap (len(snap_steps) x d_row x d_col) when snapshots were asked for."""
    lib = _load()
    W = _f64(W)
    Hinv = _f64(Hinv)
    m, d = W.shape
    assert Hinv.shape == (d, d)
    order = np.full(n_remove, -1, dtype=np.int32)
    err = np.zeros(n_remove, dtype=np.float64)
    best = np.zeros(n_remove, dtype=np.float64)
    gap = np.zeros(n_remove, dtype=np.float64)
    alive_a = None if alive is None else np.ascontiguousarray(alive, dtype=np.uint8)
    forced_a = None if forced is None else np.ascontiguousarray(forced, dtype=np.int32)
    if forced_a is not None:
        assert forced_a.shape[0] >= n_remove
    snaps = np.ascontiguousarray([] if snap_steps is None else snap_steps, dtype=np.int32)
    W_snap = np.zeros((len(snaps), m, d), dtype=np.float64)
    rc = lib.ziplm_oracle_prune(
        _ptr(W, ctypes.c_double), _ptr(Hinv, ctypes.c_double), m, d, int(group_size),
        int(n_remove),
        None if alive_a is None else _ptr(alive_a, ctypes.c_uint8),
        None if forced_a is None else _ptr(forced_a, ctypes.c_int32),
        _ptr(order, ctypes.c_int32), _ptr(err, ctypes.c_double), _ptr(best, ctypes.c_double),
        _ptr(gap, ctypes.c_double), len(snaps),
        _ptr(snaps, ctypes.c_int32) if len(snaps) else None,
        _ptr(W_snap, ctypes.c_double) if len(snaps) else None)
    if rc:
        raise OracleError(rc)
    return dict(W=W, Hinv=Hinv, order=order, err=err, best=best, gap=gap, W_snap=W_snap)


def module_error(W, H, lam=0.0):
    """tr(W (H + lam I) W^T): the layer-wise error of dropping the whole module."""
    lib = _load()
    W = _f64(W)
    H = _f64(H)
    m, d = W.shape
    assert H.shape == (d, d)
    out = ctypes.c_double(0.0)
    rc = lib.ziplm_oracle_module_error(_ptr(W, ctypes.c_double), _ptr(H, ctypes.c_double), m, d, float(lam),
                                       ctypes.byref(out))
    if rc:
        raise OracleError(rc)
    return out.value


def prior(err, total):
    """p_s after each removal: sqrt(cumulative error / whole-module error)."""
    lib = _load()
    err = _f64(err).reshape(-1)
    out = np.empty_like(err)
    rc = lib.ziplm_oracle_prior(_ptr(err, ctypes.c_double), int(err.size), float(total), _ptr(out, ctypes.c_double))
    if rc:
        raise OracleError(rc)
    return out
