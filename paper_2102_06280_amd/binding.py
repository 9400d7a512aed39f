"""Thin ctypes binding over libdbw.so: the same entry points as include/dbw.h, with
argument marshalling only.  Device arrays are torch tensors (used for memory and streams,
nothing else); every computation happens inside the library's kernels.

There is no fallback: if the library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch  # noqa: F401  (first: the library must bind to the HIP runtime that torch has already loaded)

_HERE = os.path.dirname(os.path.abspath(__file__))
# DBW_LIB: another build of the same sources (e.g. host code under sanitizers); default: the in-tree library
LIB_PATH = os.environ.get("DBW_LIB") or os.path.join(_HERE, "libdbw.so")

OK, ERR_NULL, ERR_INVALID, ERR_GRAPH, ERR_ALIAS, ERR_STATE, ERR_ALLOC, ERR_HIP, ERR_UNSUPPORTED = (
    0, -1, -2, -3, -4, -5, -6, -7, -8)
ORDER_CTA, ORDER_ATC = 0, 1
MIX_AUTO, MIX_CSR, MIX_DENSE = 0, 1, 2
MODEL_NONE, MODEL_SOFTMAX, MODEL_MLP, MODEL_CNN = 0, 1, 2, 3
WARN_THETA_INF = 1
LOSS_XENT, LOSS_MSE = 0, 1
GRAD_AUTO, GRAD_LAYERS, GRAD_CHAIN = 0, 1, 2
CAL_HBM_TRIAD, CAL_MFMA_FP32 = 0, 1
LAYOUT_ROWS, LAYOUT_TILES = 0, 1
TILE_COLUMNS = 64

EXPORTS = ["dbw_create", "dbw_select", "dbw_dtur_b", "dbw_dtur_select", "dbw_dtur_reset", "dbw_dtur_get_state", "dbw_dtur_set_state",
           "dbw_get_selection",
           "dbw_get_weights", "dbw_round_time", "dbw_round", "dbw_round_eta", "dbw_consensus_rounds",
           "dbw_consensus_rounds_static",
           "dbw_convert_layout", "dbw_grad", "dbw_check", "dbw_get_links", "dbw_mix_path",
           "dbw_destroy", "dbw_strerror", "dbw_set_timing", "dbw_get_timing", "dbw_calibrate"]


class dbw_model(C.Structure):
    _fields_ = [("kind", C.c_int32), ("batch", C.c_int32), ("n_layers", C.c_int32), ("loss", C.c_int32),
                ("dims", C.c_int32 * 9), ("grad_path", C.c_int32)]


class dbw_opts(C.Structure):
    _fields_ = [("ld", C.c_int64), ("order", C.c_int32), ("mix_path", C.c_int32), ("layout", C.c_int32),
                ("model", dbw_model)]


class dbw_kernel_time(C.Structure):
    _fields_ = [("name", C.c_char_p), ("ms_total", C.c_double), ("launches", C.c_int64)]


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2102_06280_amd.build` "
                      "(there is no CPU fallback)")
_lib = C.CDLL(LIB_PATH)
_lib.dbw_strerror.restype = C.c_char_p
_lib.dbw_strerror.argtypes = [C.c_int]
_vp, _i32, _i64, _f = C.c_void_p, C.c_int32, C.c_int64, C.c_float
_lib.dbw_create.argtypes = [C.POINTER(_vp), _i32, _i64, _vp, _vp, C.POINTER(dbw_opts)]
_lib.dbw_select.argtypes = [_vp, _vp, _vp, _vp]
_lib.dbw_dtur_b.argtypes = [_vp, _vp, _vp, _vp, _vp]
_lib.dbw_dtur_select.argtypes = [_vp, _vp, _vp, _vp, _vp]
_lib.dbw_dtur_reset.argtypes = [_vp, _vp]
_lib.dbw_dtur_get_state.argtypes = [_vp, _vp, _vp, _vp]
_lib.dbw_dtur_set_state.argtypes = [_vp, _vp, _i32, _vp]
_lib.dbw_get_selection.argtypes = [_vp, _vp, _vp, _vp, _vp]
_lib.dbw_get_weights.argtypes = [_vp, _vp, _vp]
_lib.dbw_round_time.argtypes = [_vp, _vp, _vp]
_lib.dbw_round.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _f, _vp]
_lib.dbw_round_eta.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.dbw_consensus_rounds.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _vp]
_lib.dbw_consensus_rounds_static.argtypes = [_i32, _i64, _i64, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp]
_lib.dbw_convert_layout.argtypes = [_vp, _vp, _vp, _i32, _vp]
_lib.dbw_grad.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.dbw_check.argtypes = [_vp, _vp]
_lib.dbw_get_links.argtypes = [_vp, _vp]
_lib.dbw_mix_path.argtypes = [_vp]
_lib.dbw_destroy.argtypes = [_vp]
_lib.dbw_set_timing.argtypes = [_vp, _i32]
_lib.dbw_get_timing.argtypes = [_vp, C.POINTER(dbw_kernel_time), _i32]
_lib.dbw_calibrate.argtypes = [_i32, _i64, _i32, C.POINTER(C.c_double), _vp]


class DbwError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {dbw_strerror(code)} ({code})")


def dbw_strerror(code: int) -> str:
    return _lib.dbw_strerror(int(code)).decode()


def _chk(code: int, where: str) -> int:
    if code < 0:
        raise DbwError(code, where)
    return code


def _ptr(t):
    """Device pointer of a torch tensor (or None)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("device arrays must be contiguous tensors on the GPU")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def make_model(kind: int = MODEL_NONE, batch: int = 0, dims=(), loss: int = LOSS_XENT,
               grad_path: int = GRAD_AUTO) -> dbw_model:
    m = dbw_model()
    m.kind, m.batch, m.loss, m.grad_path = kind, batch, loss, grad_path
    dims = list(dims)
    m.n_layers = len(dims) - 1 if kind in (MODEL_MLP, MODEL_SOFTMAX) else 0
    for k, v in enumerate(dims):
        m.dims[k] = int(v)
    return m


def dbw_create(rowptr, colidx, N: int, d: int, ld: int = 0, order: int = ORDER_CTA,
               mix_path: int = MIX_AUTO, model: dbw_model | None = None, layout: int = LAYOUT_ROWS):
    """rowptr / colidx: host int32 arrays (NumPy).  Returns an opaque handle."""
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    opts = dbw_opts()
    opts.ld, opts.order, opts.mix_path, opts.layout = ld, order, mix_path, layout
    opts.model = model if model is not None else make_model()
    h = _vp()
    _chk(_lib.dbw_create(C.byref(h), N, d, rowptr.ctypes.data, colidx.ctypes.data if colidx.size else None,
                         C.byref(opts)), "dbw_create")
    return h


def dbw_select(h, resp_times, b):
    return _chk(_lib.dbw_select(h, _ptr(resp_times), _ptr(b), _stream()), "dbw_select")


def dbw_dtur_b(h, resp_times, b_out, theta_out=None):
    return _chk(_lib.dbw_dtur_b(h, _ptr(resp_times), _ptr(b_out), _ptr(theta_out), _stream()), "dbw_dtur_b")


def dbw_dtur_select(h, resp_times, b_out, theta_out=None):
    return _chk(_lib.dbw_dtur_select(h, _ptr(resp_times), _ptr(b_out), _ptr(theta_out), _stream()), "dbw_dtur_select")


def dbw_dtur_reset(h):
    return _chk(_lib.dbw_dtur_reset(h, _stream()), "dbw_dtur_reset")


def dbw_dtur_get_state(h, N: int):
    """-> (visited [N-1] uint8, n_visited) on the host."""
    visited = np.zeros(max(N - 1, 1), dtype=np.uint8)
    n = C.c_int32(0)
    _chk(_lib.dbw_dtur_get_state(h, visited.ctypes.data, C.addressof(n), _stream()), "dbw_dtur_get_state")
    return visited[:N - 1], int(n.value)


def dbw_dtur_set_state(h, visited, n_visited: int):
    visited = np.ascontiguousarray(visited, dtype=np.uint8)
    keep = visited if visited.size else np.zeros(1, np.uint8)
    return _chk(_lib.dbw_dtur_set_state(h, keep.ctypes.data, int(n_visited), _stream()), "dbw_dtur_set_state")


def dbw_get_selection(h, p=None, mask=None, wait_time=None):
    return _chk(_lib.dbw_get_selection(h, _ptr(p), _ptr(mask), _ptr(wait_time), _stream()), "dbw_get_selection")


def dbw_round_time(h, T_out):
    return _chk(_lib.dbw_round_time(h, _ptr(T_out), _stream()), "dbw_round_time")


def dbw_get_weights(h, P):
    return _chk(_lib.dbw_get_weights(h, _ptr(P), _stream()), "dbw_get_weights")


def dbw_round(h, params_in, params_out, lr: float, batch_x=None, batch_y=None, ext_grads=None, loss_out=None):
    return _chk(_lib.dbw_round(h, _ptr(params_in), _ptr(params_out), _ptr(batch_x), _ptr(batch_y),
                               _ptr(ext_grads), _ptr(loss_out), float(lr), _stream()), "dbw_round")


def dbw_round_eta(h, params_in, params_out, eta, batch_x=None, batch_y=None, ext_grads=None, loss_out=None):
    return _chk(_lib.dbw_round_eta(h, _ptr(params_in), _ptr(params_out), _ptr(batch_x), _ptr(batch_y),
                                   _ptr(ext_grads), _ptr(loss_out), _ptr(eta), _stream()), "dbw_round_eta")


def dbw_consensus_rounds(h, params_in, params_out, resp_times, b, r: int):
    """resp_times [r, N] float32, b [r, N] int32 on the device."""
    return _chk(_lib.dbw_consensus_rounds(h, _ptr(params_in), _ptr(params_out), _ptr(resp_times), _ptr(b), int(r),
                                          _stream()), "dbw_consensus_rounds")


def dbw_consensus_rounds_static(N: int, d: int, ld: int, rowptr, colidx, params_in, params_out, resp_times, b,
                                r: int, status_out=None):
    """rowptr [N+1] / colidx [nnz] int32 on the device; nothing is allocated by the call."""
    return _chk(_lib.dbw_consensus_rounds_static(int(N), int(d), int(ld), int(colidx.numel()), _ptr(rowptr),
                                                 _ptr(colidx) if colidx.numel() else None, _ptr(params_in),
                                                 _ptr(params_out), _ptr(resp_times), _ptr(b), int(r),
                                                 _ptr(status_out), _stream()), "dbw_consensus_rounds_static")


def dbw_convert_layout(h, src, dst, to_tiles: bool):
    return _chk(_lib.dbw_convert_layout(h, _ptr(src), _ptr(dst), 1 if to_tiles else 0, _stream()),
                "dbw_convert_layout")


def dbw_grad(h, params, batch_x, batch_y, grads, loss_out=None):
    return _chk(_lib.dbw_grad(h, _ptr(params), _ptr(batch_x), _ptr(batch_y), _ptr(grads), _ptr(loss_out),
                              _stream()), "dbw_grad")


def dbw_check(h):
    return _chk(_lib.dbw_check(h, _stream()), "dbw_check")


def dbw_get_links(h, N: int):
    edges = np.zeros((max(N - 1, 1), 2), dtype=np.int32)
    n = _chk(_lib.dbw_get_links(h, edges.ctypes.data), "dbw_get_links")
    return edges[:n]


def dbw_mix_path(h) -> int:
    return _chk(_lib.dbw_mix_path(h), "dbw_mix_path")


def dbw_destroy(h):
    return _chk(_lib.dbw_destroy(h), "dbw_destroy")


def dbw_set_timing(h, on: bool):
    return _chk(_lib.dbw_set_timing(h, 1 if on else 0), "dbw_set_timing")


def dbw_get_timing(h):
    """{kernel name: (total ms, launches)} since timing was switched on."""
    buf = (dbw_kernel_time * 32)()
    n = _chk(_lib.dbw_get_timing(h, buf, 32), "dbw_get_timing")
    return {buf[k].name.decode(): (buf[k].ms_total, buf[k].launches) for k in range(n)}


def dbw_calibrate(what: int, size: int, repeats: int = 10) -> float:
    """Measured ceiling: GB/s (CAL_HBM_TRIAD, size = bytes per array) or TFLOP/s (CAL_MFMA_FP32,
    size = loop iterations)."""
    res = C.c_double(0.0)
    _chk(_lib.dbw_calibrate(what, size, repeats, C.byref(res), _stream()), "dbw_calibrate")
    return res.value
