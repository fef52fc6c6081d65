"""ctypes binding of librmm.so: same names as the C entry points, argument
marshalling only.  There is no fallback: if the library is not built, or a tensor
is not on the GPU, the call raises."""
import ctypes
import os

import torch

GAUSSIAN = 0
RADEMACHER = 1
SORS = 2
OP_FORWARD, OP_BACKWARD, OP_SKETCH, OP_VARIANCE = 0, 1, 2, 3
_DTYPES = {torch.float32: 0, torch.bfloat16: 1}

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class RmmError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s: %s (status %d)" % (what, rmm_status_string(status), status))


class _State(ctypes.Structure):
    _fields_ = [("seed", ctypes.c_uint64), ("offset", ctypes.c_uint64)]


class _Desc(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64), ("d_in", ctypes.c_int64), ("d_out", ctypes.c_int64), ("k", ctypes.c_int64),
                ("dtype", ctypes.c_int32), ("kind", ctypes.c_int32)]


def lib_path():
    return os.path.join(_HERE, "librmm.so")


def load_library():
    """Loads librmm.so (built by `python -m paper_2201_13195_amd.build`)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise RuntimeError("librmm.so is not built: run `python -m paper_2201_13195_amd.build` "
                           "(there is no CPU or PyTorch fallback)")
    L = ctypes.CDLL(path)
    vp, i64, u32, sz, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint32, ctypes.c_size_t, ctypes.c_int
    L.rmm_version.restype = ci
    L.rmm_version.argtypes = []
    L.rmm_status_string.restype = ctypes.c_char_p
    L.rmm_status_string.argtypes = [ci]
    L.rmm_workspace_bytes.restype = sz
    L.rmm_workspace_bytes.argtypes = [ctypes.POINTER(_Desc), ci]
    L.rmm_sketch.restype = ci
    L.rmm_sketch.argtypes = [i64, i64, i64, ci, ci, _State, vp, vp, vp, sz, vp]
    L.rmm_sketch_profiled.restype = ci
    L.rmm_sketch_profiled.argtypes = L.rmm_sketch.argtypes + [vp, vp]
    L.rmm_sketch_static.restype = ci
    L.rmm_sketch_static.argtypes = [i64, i64, i64, ci, ci, _State, vp, vp, vp]
    L.rmm_forward.restype = ci
    L.rmm_forward.argtypes = [ctypes.POINTER(_Desc), _State, vp, vp, vp, vp, vp, vp, sz, vp]
    L.rmm_backward.restype = ci
    L.rmm_backward.argtypes = [ctypes.POINTER(_Desc), _State, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.rmm_forward_profiled.restype = ci
    L.rmm_forward_profiled.argtypes = L.rmm_forward.argtypes + [ci, vp, vp]
    L.rmm_variance_stats.restype = ci
    L.rmm_variance_stats.argtypes = [ctypes.POINTER(_Desc), vp, vp, vp, vp, sz, vp]
    L.rmm_backward_accumulate.restype = ci
    L.rmm_backward_accumulate.argtypes = L.rmm_backward.argtypes
    L.rmm_backward_profiled.restype = ci
    L.rmm_backward_profiled.argtypes = L.rmm_backward.argtypes + [ci, vp, vp]
    L.rmm_uses_paired_launch.restype = ci
    L.rmm_uses_paired_launch.argtypes = [ctypes.POINTER(_Desc), ci]
    L.rmm_probe_mfma.restype = ci
    L.rmm_probe_mfma.argtypes = [ci, ci, vp, vp]
    L.rmm_probe_read.restype = ci
    L.rmm_probe_read.argtypes = [vp, sz, ci, vp, vp]
    L.rmm_debug_philox.restype = ci
    L.rmm_debug_philox.argtypes = [_State, u32, u32, i64, vp, vp]
    L.rmm_debug_sketch_tile.restype = ci
    L.rmm_debug_sketch_tile.argtypes = [ci, _State, i64, i64, i64, i64, vp, vp]
    _LIB = L
    return L


def rmm_version():
    return load_library().rmm_version()


def rmm_status_string(status):
    return load_library().rmm_status_string(int(status)).decode()


def _desc(n, d_in, d_out, k, dtype, kind):
    if dtype not in _DTYPES:
        raise TypeError("dtype must be torch.float32 or torch.bfloat16")
    return _Desc(int(n), int(d_in), int(d_out), int(k), _DTYPES[dtype], int(kind))


def rmm_workspace_bytes(n, d_in, d_out, k, dtype, kind, op):
    return int(load_library().rmm_workspace_bytes(ctypes.byref(_desc(n, d_in, d_out, k, dtype, kind)), int(op)))


_PLANS = {}


def _plan(n, d_in, d_out, k, dtype, kind, op):
    """(descriptor by reference, workspace bytes) of a layer call; kept per shape, so that a
    training loop builds the descriptor and asks the library for the workspace size once."""
    key = (n, d_in, d_out, k, dtype, kind, op)
    hit = _PLANS.get(key)
    if hit is None:
        if len(_PLANS) > 4096:
            _PLANS.clear()
        desc = _desc(n, d_in, d_out, k, dtype, kind)
        hit = _PLANS[key] = (ctypes.byref(desc), int(load_library().rmm_workspace_bytes(ctypes.byref(desc), int(op))), desc)
    return hit[0], hit[1]


def _ptr(t, name, dtype=None, shape=None, optional=False):
    if t is None:
        if optional:
            return None
        raise ValueError("%s is required" % name)
    if not t.is_cuda:
        raise ValueError("%s must be a GPU tensor (the library has no CPU path)" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must be %s" % (name, dtype))
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, has %s" % (name, tuple(shape), tuple(t.shape)))
    return t.data_ptr()  # (an int where a void* is declared)


def _stream(t):
    return torch.cuda.current_stream(t.device).cuda_stream


def _workspace(ws, need, device):
    if ws is None:
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=device)
    return ws, ws.data_ptr(), ws.numel() * ws.element_size()


def rmm_sketch(A, k, kind, seed, offset, out=None, ws=None, events=None):
    """A (n x d) -> S^T A (k x d).  Returns `out`.  `events` = (begin, end), torch.cuda.Event
    objects recorded once before, are re-recorded around the product kernel alone."""
    n, d = A.shape
    if out is None:
        out = torch.empty((k, d), dtype=A.dtype, device=A.device)
    need = rmm_workspace_bytes(n, d, d, k, A.dtype, kind, OP_SKETCH)
    ws, wsp, wsb = _workspace(ws, need, A.device)
    evb = eve = None
    if events is not None:
        evb, eve = ctypes.c_void_p(events[0].cuda_event), ctypes.c_void_p(events[1].cuda_event)
    rc = load_library().rmm_sketch_profiled(n, d, k, _DTYPES[A.dtype], kind, _State(seed, offset), _ptr(A, "A"),
                                            _ptr(out, "out", A.dtype, (k, d)), wsp, wsb, _stream(A), evb, eve)
    if rc != 0:
        raise RmmError(rc, "rmm_sketch")
    return out


STATIC_SCRATCH_BYTES = 32 << 20


def rmm_sketch_static(A, k, kind, seed, offset, out):
    """rmm_sketch on the library's own static scratch: no workspace, no allocation (the caller
    passes `out`).  Raises RmmError(-5) when the shape needs more than STATIC_SCRATCH_BYTES."""
    n, d = A.shape
    rc = load_library().rmm_sketch_static(n, d, k, _DTYPES[A.dtype], kind, _State(seed, offset), _ptr(A, "A"),
                                          _ptr(out, "out", A.dtype, (k, d)), _stream(A))
    if rc != 0:
        raise RmmError(rc, "rmm_sketch_static")
    return out


VARIANCE_FIELDS = ("x_fro2", "y_fro2", "rows", "xty_fro2", "d2_sgd", "d2_rmm", "alpha", "d2_rmm_printed")


def rmm_variance_stats(X, dY, k, kind, out=None, ws=None):
    """Variance monitors of Section 2.3.  Returns a device tensor of 8 doubles (VARIANCE_FIELDS)."""
    n, d_in = X.shape
    d_out = dY.shape[1]
    if out is None:
        out = torch.empty((8,), dtype=torch.float64, device=X.device)
    desc = _desc(n, d_in, d_out, k, X.dtype, kind)
    need = rmm_workspace_bytes(n, d_in, d_out, k, X.dtype, kind, OP_VARIANCE)
    ws, wsp, wsb = _workspace(ws, need, X.device)
    rc = load_library().rmm_variance_stats(ctypes.byref(desc), _ptr(X, "X"), _ptr(dY, "dY", X.dtype, (n, d_out)),
                                           _ptr(out, "out", torch.float64, (8,)), wsp, wsb, _stream(X))
    if rc != 0:
        raise RmmError(rc, "rmm_variance_stats")
    return out


STAGE_FWD_Y, STAGE_FWD_XPROJ, STAGE_BWD_DX, STAGE_BWD_G, STAGE_BWD_DW, STAGE_BWD_DBIAS = range(6)
STAGE_FWD_XPROJ_PRODUCT, STAGE_BWD_G_PRODUCT = 6, 7
STAGE_FWD_PAIR, STAGE_BWD_PAIR = 8, 9     # the one-launch kernel for Y with X_proj / dX with G, where the library has one


def _event_args(profile):
    """profile = (stage, begin, end) with torch.cuda.Event objects that have been
    recorded once (so that their handles exist), or None."""
    if profile is None:
        return -1, None, None
    stage, begin, end = profile
    return int(stage), ctypes.c_void_p(begin.cuda_event), ctypes.c_void_p(end.cuda_event)


def rmm_forward(X, W, bias, k, kind, seed, offset, Y=None, X_proj=None, ws=None, profile=None, need_xproj=True):
    """Algorithm 1 forward.  Returns (Y, X_proj); with need_xproj=False (no backward pass will
    follow) the sketch is skipped and X_proj is None."""
    n, d_in = X.shape
    d_out = W.shape[0]
    if Y is None:
        Y = torch.empty((n, d_out), dtype=X.dtype, device=X.device)
    if X_proj is None and need_xproj:
        X_proj = torch.empty((k, d_in), dtype=X.dtype, device=X.device)
    desc, need = _plan(n, d_in, d_out, k, X.dtype, kind, OP_FORWARD)
    ws, wsp, wsb = _workspace(ws, need if need_xproj else 0, X.device)
    rc = load_library().rmm_forward_profiled(desc, _State(seed, offset), _ptr(X, "X"),
                                             _ptr(W, "W", X.dtype, (d_out, d_in)),
                                             _ptr(bias, "bias", X.dtype, (d_out,), optional=True),
                                             _ptr(Y, "Y", X.dtype, (n, d_out)),
                                             _ptr(X_proj, "X_proj", X.dtype, (k, d_in), optional=not need_xproj),
                                             wsp, wsb, _stream(X), *_event_args(profile))
    if rc != 0:
        raise RmmError(rc, "rmm_forward")
    return Y, X_proj


def rmm_backward(dY, W, X_proj, kind, seed, offset, need_dX=True, need_dbias=False, dX=None, dW=None, dbias=None,
                 ws=None, profile=None, accumulate=False):
    """Algorithm 1 backward with the forward call's state.  Returns (dX, dW, dbias).  With
    `accumulate` the given dW (and dbias) are added to instead of overwritten."""
    if accumulate and (dW is None or (need_dbias and dbias is None) or profile is not None):
        raise ValueError("accumulate needs existing dW / dbias tensors and no profile")
    n, d_out = dY.shape
    k, d_in = X_proj.shape
    if need_dX and dX is None:
        dX = torch.empty((n, d_in), dtype=dY.dtype, device=dY.device)
    if dW is None:
        dW = torch.empty((d_out, d_in), dtype=dY.dtype, device=dY.device)
    if need_dbias and dbias is None:
        dbias = torch.empty((d_out,), dtype=dY.dtype, device=dY.device)
    desc, need = _plan(n, d_in, d_out, k, dY.dtype, kind, OP_BACKWARD)
    ws, wsp, wsb = _workspace(ws, need, dY.device)
    args = (desc, _State(seed, offset), _ptr(dY, "dY"), _ptr(W, "W", dY.dtype, (d_out, d_in)),
            _ptr(X_proj, "X_proj", dY.dtype, (k, d_in)), _ptr(dX, "dX", dY.dtype, (n, d_in), optional=True),
            _ptr(dW, "dW", dY.dtype, (d_out, d_in)), _ptr(dbias, "dbias", dY.dtype, (d_out,), optional=True),
            wsp, wsb, _stream(dY))
    if accumulate:
        rc = load_library().rmm_backward_accumulate(*args)
    else:
        rc = load_library().rmm_backward_profiled(*args, *_event_args(profile))
    if rc != 0:
        raise RmmError(rc, "rmm_backward")
    return dX, dW, dbias


def rmm_uses_paired_launch(n, d_in, d_out, k, dtype, kind, op):
    return bool(load_library().rmm_uses_paired_launch(ctypes.byref(_desc(n, d_in, d_out, k, dtype, kind)), int(op)))


def rmm_probe_mfma(work_groups, iters, sink):
    """Pure MFMA loop (work_groups x 4 waves x 16 x iters MFMAs of 32768 flop); returns the flop count."""
    rc = load_library().rmm_probe_mfma(int(work_groups), int(iters), _ptr(sink, "sink"), _stream(sink))
    if rc != 0:
        raise RmmError(rc, "rmm_probe_mfma")
    return work_groups * 4 * 16 * iters * 32768


def rmm_probe_read(src, work_groups, sink):
    """One streaming read of `src` (a contiguous GPU tensor); returns the byte count."""
    nbytes = src.numel() * src.element_size() // 16 * 16
    rc = load_library().rmm_probe_read(_ptr(src, "src"), nbytes, int(work_groups), _ptr(sink, "sink"), _stream(src))
    if rc != 0:
        raise RmmError(rc, "rmm_probe_read")
    return nbytes


def rmm_debug_philox(seed, offset, c0, c1, ncalls, device="cuda"):
    """uint32 words (ncalls x 4) of Philox calls with counters (c0 + t, c1, offset lo, offset hi)."""
    out = torch.empty((ncalls, 4), dtype=torch.int32, device=device)
    rc = load_library().rmm_debug_philox(_State(seed, offset), c0, c1, ncalls, _ptr(out, "out"), _stream(out))
    if rc != 0:
        raise RmmError(rc, "rmm_debug_philox")
    return out


def rmm_debug_sketch_tile(kind, seed, offset, i0, j0, rows, cols, device="cuda"):
    """fp32 (rows x cols) tile of the unscaled sketch P starting at (i0, j0)."""
    out = torch.empty((rows, cols), dtype=torch.float32, device=device)
    rc = load_library().rmm_debug_sketch_tile(kind, _State(seed, offset), i0, j0, rows, cols, _ptr(out, "out"),
                                              _stream(out))
    if rc != 0:
        raise RmmError(rc, "rmm_debug_sketch_tile")
    return out
