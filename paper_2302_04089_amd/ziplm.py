"""Thin ctypes binding of libziplm.so (argument marshalling only).

Same names as the C ABI in include/ziplm.h.  Tensors are torch CUDA tensors (PyTorch provides
device memory and the stream, nothing else); every computation runs inside the library's HIP
kernels.  There is no CPU fallback: if the library is missing, loading raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# ZIPLM_LIBRARY selects another build of the same ABI (for instance an instrumented one)
LIB_PATH = os.environ.get("ZIPLM_LIBRARY") or os.path.join(_HERE, "libziplm.so")

OK = 0
ERR_INVALID_ARG = -1
ERR_NOT_PD = -2
ERR_WORKSPACE = -3
ERR_DEVICE = -4
ERR_UNSUPPORTED = -5
X_FEATURE_MAJOR = 0
X_TOKEN_MAJOR = 1

EXPORTS = (
    "ziplm_version", "ziplm_status_string",
    "ziplm_hessian_accumulate", "ziplm_hessian_workspace_bytes",
    "ziplm_hinv", "ziplm_hinv_workspace_bytes",
    "ziplm_structured_obs_prune", "ziplm_prune_workspace_bytes",
    "ziplm_module_error", "ziplm_module_error_workspace_bytes", "ziplm_prior",
    "ziplm_structured_obs_prune_batch", "ziplm_prune_batch_workspace_bytes",
    "ziplm_prune_exchange_bytes", "ziplm_exchange_alloc",
    "ziplm_structured_obs_prune_eager", "ziplm_prune_eager_workspace_bytes",
    "ziplm_selftest_bounded_wait", "ziplm_selftest_handoff_latency",
    "ziplm_module_error_static", "ziplm_module_error_static_max_tiles",
    "ziplm_search_select", "ziplm_search_mutate",
)

_lib = None
SCORE_CALLBACK = ctypes.CFUNCTYPE(ctypes.c_double, ctypes.POINTER(ctypes.c_int32), ctypes.c_void_p)


class ZiplmError(RuntimeError):
    def __init__(self, status, info=None):
        msg = lib().ziplm_status_string(int(status)).decode()
        super().__init__("libziplm: %s (status %d, info %s)" % (msg, status, info))
        self.status = int(status)
        self.info = info


def lib():
    """Loads libziplm.so (built in-tree by paper_2302_04089_amd/build.py).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libziplm.so is not built: run `python paper_2302_04089_amd/build.py`")
    L = ctypes.CDLL(LIB_PATH)
    vp, sz, i32, i64, f32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int64, ctypes.c_float
    L.ziplm_version.restype = i32
    L.ziplm_version.argtypes = []
    L.ziplm_status_string.restype = ctypes.c_char_p
    L.ziplm_status_string.argtypes = [i32]
    L.ziplm_hessian_accumulate.restype = i32
    L.ziplm_hessian_accumulate.argtypes = [vp, vp, i32, i64, i64, i32, f32, vp, sz, vp]
    L.ziplm_hessian_workspace_bytes.restype = sz
    L.ziplm_hessian_workspace_bytes.argtypes = [i32, i64]
    L.ziplm_hinv.restype = i32
    L.ziplm_hinv.argtypes = [vp, vp, i32, f32, ctypes.POINTER(f32), ctypes.POINTER(i32), vp, sz, vp]
    L.ziplm_hinv_workspace_bytes.restype = sz
    L.ziplm_hinv_workspace_bytes.argtypes = [i32]
    L.ziplm_structured_obs_prune.restype = i32
    L.ziplm_structured_obs_prune.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp, i32,
                                             ctypes.POINTER(ctypes.c_int32), vp, ctypes.POINTER(i32),
                                             vp, sz, vp, sz, vp]
    L.ziplm_prune_exchange_bytes.restype = sz
    L.ziplm_prune_exchange_bytes.argtypes = [i32, i32, i32, i32]
    L.ziplm_exchange_alloc.restype = i32
    L.ziplm_exchange_alloc.argtypes = [sz, ctypes.POINTER(vp)]
    L.ziplm_structured_obs_prune_eager.restype = i32
    L.ziplm_structured_obs_prune_eager.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp, i32,
                                                   ctypes.POINTER(ctypes.c_int32), vp, ctypes.POINTER(i32),
                                                   vp, sz, vp]
    L.ziplm_prune_eager_workspace_bytes.restype = sz
    L.ziplm_prune_eager_workspace_bytes.argtypes = [i32, i32, i32]
    L.ziplm_selftest_bounded_wait.restype = i32
    L.ziplm_selftest_bounded_wait.argtypes = [vp, vp, i32, i32, vp, vp, ctypes.POINTER(i32), vp, sz, vp]
    L.ziplm_selftest_handoff_latency.restype = i32
    L.ziplm_selftest_handoff_latency.argtypes = [i32, i32, ctypes.POINTER(ctypes.c_double), vp, sz, vp]
    L.ziplm_prune_workspace_bytes.restype = sz
    L.ziplm_prune_workspace_bytes.argtypes = [i32, i32, i32, i32]
    L.ziplm_structured_obs_prune_batch.restype = i32
    L.ziplm_structured_obs_prune_batch.argtypes = [vp, vp, i32, i64, i64, i32, i32, i32, i32, vp, vp, i32,
                                                   ctypes.POINTER(ctypes.c_int32), vp, ctypes.POINTER(i32),
                                                   vp, sz, vp, sz, vp]
    L.ziplm_prune_batch_workspace_bytes.restype = sz
    L.ziplm_prune_batch_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
    L.ziplm_module_error.restype = i32
    L.ziplm_module_error.argtypes = [vp, vp, i32, i32, f32, vp, vp, sz, vp]
    L.ziplm_module_error_workspace_bytes.restype = sz
    L.ziplm_module_error_workspace_bytes.argtypes = [i32, i32]
    L.ziplm_module_error_static.restype = i32
    L.ziplm_module_error_static.argtypes = [vp, vp, i32, i32, f32, vp, vp]
    L.ziplm_module_error_static_max_tiles.restype = i32
    L.ziplm_module_error_static_max_tiles.argtypes = []
    L.ziplm_prior.restype = i32
    L.ziplm_prior.argtypes = [vp, i32, vp, vp, vp]
    dp_, ip_ = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)
    L.ziplm_search_select.restype = i32
    L.ziplm_search_select.argtypes = [i32, ip_, dp_, dp_, ctypes.c_double, i32, ip_, dp_, dp_]
    L.ziplm_search_mutate.restype = i32
    L.ziplm_search_mutate.argtypes = [i32, ip_, dp_, dp_, ctypes.c_double, i32, i32, ctypes.c_double, dp_,
                                      SCORE_CALLBACK, vp, ip_, dp_, dp_]
    _lib = L
    return L


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check(t, dtype, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("%s must be a contiguous CUDA tensor of dtype %s" % (name, dtype))


def _workspace(nbytes, device):
    # torch's caching allocator returns 512-byte aligned blocks
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def ziplm_hessian_workspace_bytes(d_col, n_tok):
    return int(lib().ziplm_hessian_workspace_bytes(int(d_col), int(n_tok)))


def ziplm_hinv_workspace_bytes(d_col):
    return int(lib().ziplm_hinv_workspace_bytes(int(d_col)))


def ziplm_prune_workspace_bytes(d_row, d_col, group_size, n_snap=0):
    return int(lib().ziplm_prune_workspace_bytes(int(d_row), int(d_col), int(group_size), int(n_snap)))


def ziplm_hessian_accumulate(H, X, scale=2.0, layout=X_FEATURE_MAJOR, workspace=None, stream=None):
    """H += scale * X X^T.  X: (d_col, n_tok) feature-major or (n_tok, d_col) token-major."""
    _check(H, torch.float32, "H")
    _check(X, torch.float32, "X")
    d = H.shape[0]
    if layout == X_FEATURE_MAJOR:
        n_tok, ldx = X.shape[1], X.stride(0)
        assert X.shape[0] == d
    else:
        n_tok, ldx = X.shape[0], X.stride(0)
        assert X.shape[1] == d
    need = ziplm_hessian_workspace_bytes(d, n_tok)
    ws = workspace if workspace is not None else _workspace(need, H.device)
    rc = lib().ziplm_hessian_accumulate(H.data_ptr(), X.data_ptr(), d, n_tok, ldx, int(layout), float(scale),
                                        ws.data_ptr(), ws.numel(), _stream(stream))
    if rc != OK:
        raise ZiplmError(rc)
    return H


def ziplm_hinv(H, damp_rel=0.01, out=None, workspace=None, stream=None, check=True):
    """Returns (Hinv, lambda).  With check=False nothing is copied back and lambda is None."""
    _check(H, torch.float32, "H")
    d = H.shape[0]
    out = torch.empty_like(H) if out is None else out
    _check(out, torch.float32, "out")
    need = ziplm_hinv_workspace_bytes(d)
    ws = workspace if workspace is not None else _workspace(need, H.device)
    lam = ctypes.c_float(0.0)
    info = ctypes.c_int(0)
    rc = lib().ziplm_hinv(H.data_ptr(), out.data_ptr(), d, float(damp_rel),
                          ctypes.byref(lam) if check else None, ctypes.byref(info) if check else None,
                          ws.data_ptr(), ws.numel(), _stream(stream))
    if rc != OK:
        raise ZiplmError(rc, info.value)
    return out, (lam.value if check else None)


class ExchangeArea:
    """An exchange area from ziplm_exchange_alloc: uncached device memory the caller keeps for the life of the
    process (the library has no call that frees it) and passes to the single-column loops."""

    def __init__(self, ptr, nbytes):
        self.ptr = int(ptr)
        self.nbytes = int(nbytes)


def ziplm_prune_exchange_bytes(n_layers, d_row, d_col, group_size=1):
    return int(lib().ziplm_prune_exchange_bytes(int(n_layers), int(d_row), int(d_col), int(group_size)))


def ziplm_exchange_alloc(nbytes):
    out = ctypes.c_void_p()
    rc = lib().ziplm_exchange_alloc(int(nbytes), ctypes.byref(out))
    if rc != OK:
        raise ZiplmError(rc)
    return ExchangeArea(out.value, nbytes)


def _exchange_args(exchange):
    if exchange is None:
        return None, 0
    return ctypes.c_void_p(exchange.ptr), exchange.nbytes


def ziplm_structured_obs_prune(W, Hinv, group_size, n_remove, alive=None, snapshot_steps=None,
                               workspace=None, stream=None, check=True, exchange=None):
    """Algorithm 1 in place on W and Hinv.  Returns (order int32[n_remove], err float64[n_remove],
    W_snap or None), all on the device.  exchange: an ExchangeArea or None."""
    _check(W, torch.float32, "W")
    _check(Hinv, torch.float32, "Hinv")
    m, d = W.shape
    dev = W.device
    order = torch.empty(max(n_remove, 1), dtype=torch.int32, device=dev)
    err = torch.empty(max(n_remove, 1), dtype=torch.float64, device=dev)
    steps = [] if snapshot_steps is None else [int(s) for s in snapshot_steps]
    n_snap = len(steps)
    W_snap = torch.empty((n_snap, m, d), dtype=torch.float32, device=dev) if n_snap else None
    steps_c = (ctypes.c_int32 * n_snap)(*steps) if n_snap else None
    if alive is not None:
        _check(alive, torch.uint8, "alive")
    need = ziplm_prune_workspace_bytes(m, d, group_size, n_snap)
    ws = workspace if workspace is not None else _workspace(need, dev)
    info = ctypes.c_int(0)
    rc = lib().ziplm_structured_obs_prune(
        W.data_ptr(), Hinv.data_ptr(), m, d, int(group_size), int(n_remove), order.data_ptr(), err.data_ptr(),
        alive.data_ptr() if alive is not None else None, n_snap, steps_c,
        W_snap.data_ptr() if n_snap else None, ctypes.byref(info) if check else None,
        *_exchange_args(exchange), ws.data_ptr(), ws.numel(), _stream(stream))
    if rc != OK:
        raise ZiplmError(rc, info.value)
    return order[:n_remove], err[:n_remove], W_snap


def ziplm_prune_eager_workspace_bytes(d_row, d_col, n_snap=0):
    return int(lib().ziplm_prune_eager_workspace_bytes(int(d_row), int(d_col), int(n_snap)))


def ziplm_structured_obs_prune_eager(W, Hinv, n_remove, alive=None, snapshot_steps=None, workspace=None,
                                     stream=None, check=True):
    """Algorithm 1 over single columns on the eager kernel (whole state read and written every step)."""
    _check(W, torch.float32, "W")
    _check(Hinv, torch.float32, "Hinv")
    m, d = W.shape
    dev = W.device
    order = torch.empty(max(n_remove, 1), dtype=torch.int32, device=dev)
    err = torch.empty(max(n_remove, 1), dtype=torch.float64, device=dev)
    steps = [] if snapshot_steps is None else [int(s) for s in snapshot_steps]
    n_snap = len(steps)
    W_snap = torch.empty((n_snap, m, d), dtype=torch.float32, device=dev) if n_snap else None
    steps_c = (ctypes.c_int32 * n_snap)(*steps) if n_snap else None
    if alive is not None:
        _check(alive, torch.uint8, "alive")
    ws = workspace if workspace is not None else _workspace(ziplm_prune_eager_workspace_bytes(m, d, n_snap), dev)
    info = ctypes.c_int(0)
    rc = lib().ziplm_structured_obs_prune_eager(
        W.data_ptr(), Hinv.data_ptr(), m, d, int(n_remove), order.data_ptr(), err.data_ptr(),
        alive.data_ptr() if alive is not None else None, n_snap, steps_c,
        W_snap.data_ptr() if n_snap else None, ctypes.byref(info) if check else None,
        ws.data_ptr(), ws.numel(), _stream(stream))
    if rc != OK:
        raise ZiplmError(rc, info.value)
    return order[:n_remove], err[:n_remove], W_snap


def ziplm_selftest_bounded_wait(W, Hinv, workspace=None, stream=None):
    """Runs the single-column loop with one workgroup held back; returns (status, info): expected
    (ERR_DEVICE, -1) after a little over 4 s, with W and Hinv unchanged."""
    _check(W, torch.float32, "W")
    _check(Hinv, torch.float32, "Hinv")
    m, d = W.shape
    order = torch.empty(d, dtype=torch.int32, device=W.device)
    err = torch.empty(d, dtype=torch.float64, device=W.device)
    ws = workspace if workspace is not None else _workspace(ziplm_prune_workspace_bytes(m, d, 1, 0), W.device)
    info = ctypes.c_int(0)
    rc = lib().ziplm_selftest_bounded_wait(W.data_ptr(), Hinv.data_ptr(), m, d, order.data_ptr(), err.data_ptr(),
                                           ctypes.byref(info), ws.data_ptr(), ws.numel(), _stream(stream))
    return rc, info.value


def ziplm_selftest_handoff_latency(rounds=2000, partner=1, exchange=None, stream=None):
    """Mean one-way hand-off time (us) between workgroup 0 and workgroup `partner`; the words live in `exchange`
    (an ExchangeArea) or in ordinary device memory."""
    us = ctypes.c_double(0.0)
    if exchange is None:
        ws = _workspace(1024, torch.device("cuda", torch.cuda.current_device()))
        ptr, nbytes = ws.data_ptr(), ws.numel()
    else:
        ptr, nbytes = ctypes.c_void_p(exchange.ptr), exchange.nbytes
    rc = lib().ziplm_selftest_handoff_latency(int(rounds), int(partner), ctypes.byref(us), ptr, nbytes, _stream(stream))
    if rc != OK:
        raise ZiplmError(rc)
    return us.value


def ziplm_prune_batch_workspace_bytes(n_layers, d_row, d_col, group_size, n_snap=0):
    return int(lib().ziplm_prune_batch_workspace_bytes(int(n_layers), int(d_row), int(d_col), int(group_size), int(n_snap)))


def ziplm_structured_obs_prune_batch(W, Hinv, group_size, n_remove, snapshot_steps=None, workspace=None,
                                     stream=None, check=True, exchange=None):
    """Algorithm 1 for a stack of layers of one shape: W (n_layers, d_row, d_col), Hinv (n_layers, d_col,
    d_col), both in place.  Returns (order int32[n_layers, n_remove], err float64[n_layers, n_remove],
    W_snap (n_layers, n_snap, d_row, d_col) or None), all on the device."""
    _check(W, torch.float32, "W")
    _check(Hinv, torch.float32, "Hinv")
    n_layers, m, d = W.shape
    assert Hinv.shape == (n_layers, d, d)
    dev = W.device
    order = torch.empty((n_layers, max(n_remove, 1)), dtype=torch.int32, device=dev)
    err = torch.empty((n_layers, max(n_remove, 1)), dtype=torch.float64, device=dev)
    steps = [] if snapshot_steps is None else [int(s) for s in snapshot_steps]
    n_snap = len(steps)
    W_snap = torch.empty((n_layers, n_snap, m, d), dtype=torch.float32, device=dev) if n_snap else None
    steps_c = (ctypes.c_int32 * n_snap)(*steps) if n_snap else None
    need = ziplm_prune_batch_workspace_bytes(n_layers, m, d, group_size, n_snap)
    ws = workspace if workspace is not None else _workspace(need, dev)
    info = (ctypes.c_int * n_layers)()
    rc = lib().ziplm_structured_obs_prune_batch(
        W.data_ptr(), Hinv.data_ptr(), n_layers, m * d, d * d, m, d, int(group_size), int(n_remove),
        order.data_ptr(), err.data_ptr(), n_snap, steps_c, W_snap.data_ptr() if n_snap else None,
        info if check else None, *_exchange_args(exchange), ws.data_ptr(), ws.numel(), _stream(stream))
    if rc != OK:
        raise ZiplmError(rc, list(info))
    if n_remove == 0:
        return order[:, :0], err[:, :0], W_snap
    return order, err, W_snap


def database_steps(n_structures, kind):
    """Removal counts at which to snapshot W so that one greedy run yields the per-layer database of
    Section 3.2 on the grid of its "Runtime awareness" paragraph (host-side list arithmetic only).

    kind "columns": intermediate sizes n * 0.9**i, i = 0..42 (truncated to integers, duplicates
    dropped) -> snapshot after n - size removals.  kind "heads": 0, 1, ..., n heads removed.
    Returns a sorted list of distinct step counts, usable as `snapshot_steps`."""
    n = int(n_structures)
    if kind == "heads":
        return list(range(n + 1))
    if kind == "columns":
        return sorted({n - int(n * 0.9 ** i) for i in range(43)})
    raise ValueError("kind must be 'columns' or 'heads'")


def ziplm_module_error_workspace_bytes(d_row, d_col):
    return int(lib().ziplm_module_error_workspace_bytes(int(d_row), int(d_col)))


def ziplm_module_error(W, H, lam=0.0, out=None, workspace=None, stream=None):
    """tr(W (H + lam I) W^T) as a one-element float64 device tensor."""
    _check(W, torch.float32, "W")
    _check(H, torch.float32, "H")
    m, d = W.shape
    assert H.shape == (d, d)
    out = torch.empty(1, dtype=torch.float64, device=W.device) if out is None else out
    _check(out, torch.float64, "out")
    need = ziplm_module_error_workspace_bytes(m, d)
    ws = workspace if workspace is not None else _workspace(need, W.device)
    rc = lib().ziplm_module_error(W.data_ptr(), H.data_ptr(), m, d, float(lam), out.data_ptr(), ws.data_ptr(),
                                  ws.numel(), _stream(stream))
    if rc != OK:
        raise ZiplmError(rc)
    return out


def ziplm_module_error_static(W, H, lam=0.0, out=None, stream=None):
    """ziplm_module_error without a workspace: the partial sums go to the library's built-in scratch array."""
    _check(W, torch.float32, "W")
    _check(H, torch.float32, "H")
    m, d = W.shape
    assert H.shape == (d, d)
    out = torch.empty(1, dtype=torch.float64, device=W.device) if out is None else out
    _check(out, torch.float64, "out")
    rc = lib().ziplm_module_error_static(W.data_ptr(), H.data_ptr(), m, d, float(lam), out.data_ptr(), _stream(stream))
    if rc != OK:
        raise ZiplmError(rc)
    return out


def ziplm_prior(err, total, out=None, stream=None):
    """p_s after each removal: sqrt(cumsum(err) / total); err float64[n] and total float64[1] on the device."""
    _check(err, torch.float64, "err")
    _check(total, torch.float64, "total")
    out = torch.empty_like(err) if out is None else out
    _check(out, torch.float64, "out")
    assert out.numel() >= err.numel()
    rc = lib().ziplm_prior(err.data_ptr(), int(err.numel()), total.data_ptr(), out.data_ptr(), _stream(stream))
    if rc != OK:
        raise ZiplmError(rc)
    return out


def _flat_levels(per_layer):
    n_levels = (ctypes.c_int32 * len(per_layer))(*[len(v) for v in per_layer])
    flat = [float(x) for v in per_layer for x in v]
    return n_levels, (ctypes.c_double * len(flat))(*flat)


def ziplm_search_select(levels_time, levels_cost, budget, buckets=10000):
    """Host-side: one level per layer of least total cost within the time budget.  levels_time / levels_cost: a list
    per layer.  Returns (choice list, total cost, total time)."""
    n = len(levels_time)
    n_levels, t = _flat_levels(levels_time)
    _, c = _flat_levels(levels_cost)
    choice = (ctypes.c_int32 * n)()
    cost, time_ = ctypes.c_double(0.0), ctypes.c_double(0.0)
    rc = lib().ziplm_search_select(n, n_levels, t, c, float(budget), int(buckets), choice, ctypes.byref(cost), ctypes.byref(time_))
    if rc != OK:
        raise ZiplmError(rc)
    return list(choice), cost.value, time_.value


def ziplm_search_mutate(levels_time, levels_prior, budget, score, uniforms, buckets=10000, mutate_prob=0.1):
    """Host-side: the outer loop of the structured SPDY search.  score(choice list) -> float, lower is better;
    uniforms: array-like [n_steps][n_layers][2] of numbers in [0, 1).  Returns (choice, coefficients, best score)."""
    n = len(levels_time)
    n_levels, t = _flat_levels(levels_time)
    _, p = _flat_levels(levels_prior)
    flat_u = [float(x) for step in uniforms for pair in step for x in pair]
    n_steps = len(uniforms)
    u = (ctypes.c_double * max(len(flat_u), 1))(*flat_u)
    cb = SCORE_CALLBACK(lambda ch, _user: float(score([ch[i] for i in range(n)])))
    choice = (ctypes.c_int32 * n)()
    coef = (ctypes.c_double * n)()
    best = ctypes.c_double(0.0)
    rc = lib().ziplm_search_mutate(n, n_levels, t, p, float(budget), int(buckets), n_steps, float(mutate_prob), u, cb, None,
                                   choice, coef, ctypes.byref(best))
    if rc != OK:
        raise ZiplmError(rc)
    return list(choice), list(coef), best.value
