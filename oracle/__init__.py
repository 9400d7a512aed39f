"""ctypes access to the CPU oracle (oracle/dbw_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg; never by the product package.  This wrapper marshals NumPy arrays and
holds no arithmetic of its own.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "dbw_oracle.c")
_LIB = os.path.join(_DIR, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP over workers)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def build_sanitized(path: str) -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (host code only),
    for the test that runs the pins over it."""
    subprocess.check_call(["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", path,
                           _SRC, "-lm"])
    return path


_lib = None


def lib():
    global _lib
    if _lib is None:
        os.environ.setdefault("OMP_WAIT_POLICY", "passive")   # idle workers sleep instead of spinning
        override = os.environ.get("DBW_ORACLE_LIB")           # a build of the same source, e.g. with sanitizers
        if not override:
            build()
        _lib = C.CDLL(override or _LIB)
        _lib.orc_select.restype = C.c_int
        _lib.orc_spanning_tree.restype = C.c_int
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def select(rowptr, colidx, t, b):
    """-> (mask[nnz] uint8, p[N] int32, wait[N] fp32); raises ValueError on b out of range."""
    rowptr, colidx, t, b = _i32(rowptr), _i32(colidx), _f32(t), _i32(b)
    n = rowptr.size - 1
    mask = np.zeros(colidx.size, dtype=np.uint8)
    p = np.zeros(n, dtype=np.int32)
    wait = np.zeros(n, dtype=np.float32)
    rc = lib().orc_select(n, _p(rowptr, C.c_int32), _p(colidx, C.c_int32), _p(t, C.c_float),
                          _p(b, C.c_int32), _p(mask, C.c_uint8), _p(p, C.c_int32), _p(wait, C.c_float))
    if rc != 0:
        raise ValueError(f"orc_select: {rc}")
    return mask, p, wait


def round_time(rowptr, colidx, mask, wait):
    """-> (max wait over all workers, max wait over workers somebody waits for)."""
    rowptr, colidx, wait = _i32(rowptr), _i32(colidx), _f32(wait)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    out = np.zeros(2, dtype=np.float32)
    lib().orc_round_time(rowptr.size - 1, _p(rowptr, C.c_int32), _p(colidx, C.c_int32), _p(mask, C.c_uint8),
                         _p(wait, C.c_float), _p(out, C.c_float))
    return float(out[0]), float(out[1])


def weights(rowptr, colidx, mask, p):
    rowptr, colidx, p = _i32(rowptr), _i32(colidx), _i32(p)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    n = rowptr.size - 1
    we = np.zeros(max(colidx.size, 1), dtype=np.float64)
    ws = np.zeros(n, dtype=np.float64)
    lib().orc_weights(n, _p(rowptr, C.c_int32), _p(colidx, C.c_int32), _p(mask, C.c_uint8),
                      _p(p, C.c_int32), _p(we, C.c_double), _p(ws, C.c_double))
    return we[:colidx.size], ws


def dense_P(rowptr, colidx, mask, p):
    rowptr, colidx, p = _i32(rowptr), _i32(colidx), _i32(p)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    n = rowptr.size - 1
    P = np.zeros((n, n), dtype=np.float64)
    lib().orc_dense_P(n, _p(rowptr, C.c_int32), _p(colidx, C.c_int32), _p(mask, C.c_uint8),
                      _p(p, C.c_int32), _p(P, C.c_double))
    return P


def round_(rowptr, colidx, mask, p, x, g, lr, order=0, d=None):
    """x, g: [N, ld] fp32 (g may be None) -> out [N, ld] fp32 (columns >= d left zero)."""
    rowptr, colidx, p = _i32(rowptr), _i32(colidx), _i32(p)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    x = _f32(x)
    n, ld = x.shape
    d = ld if d is None else d
    gp = None
    if g is not None:
        g = _f32(g)
        assert g.shape == x.shape
        gp = _p(g, C.c_float)
    out = np.zeros_like(x)
    lib().orc_round(n, C.c_int64(d), C.c_int64(ld), _p(rowptr, C.c_int32), _p(colidx, C.c_int32),
                    _p(mask, C.c_uint8), _p(p, C.c_int32), _p(x, C.c_float), gp,
                    C.c_float(lr), int(order), _p(out, C.c_float))
    return out


def round_eta(rowptr, colidx, mask, p, x, g, eta, order=0, d=None):
    """round_ with a learning rate per worker: eta [N] fp32."""
    rowptr, colidx, p = _i32(rowptr), _i32(colidx), _i32(p)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    x, g, eta = _f32(x), _f32(g), _f32(eta)
    n, ld = x.shape
    assert g.shape == x.shape and eta.shape == (n,)
    d = ld if d is None else d
    out = np.zeros_like(x)
    lib().orc_round_eta(n, C.c_int64(d), C.c_int64(ld), _p(rowptr, C.c_int32), _p(colidx, C.c_int32),
                        _p(mask, C.c_uint8), _p(p, C.c_int32), _p(x, C.c_float), _p(g, C.c_float),
                        _p(eta, C.c_float), int(order), _p(out, C.c_float))
    return out


def spanning_tree(rowptr, colidx):
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    n = rowptr.size - 1
    edges = np.zeros((max(n - 1, 1), 2), dtype=np.int32)
    rc = lib().orc_spanning_tree(n, _p(rowptr, C.c_int32), _p(colidx, C.c_int32), _p(edges, C.c_int32))
    if rc < 0:
        raise ValueError("graph not connected")
    return edges[:rc]


class Dtur:
    """State of the d-iteration procedure: the link set, the visited set P', its size."""

    def __init__(self, rowptr, colidx):
        self.rowptr, self.colidx = _i32(rowptr), _i32(colidx)
        self.n = self.rowptr.size - 1
        self.edges = np.ascontiguousarray(spanning_tree(rowptr, colidx))
        self.visited = np.zeros(max(len(self.edges), 1), dtype=np.uint8)
        self.n_visited = C.c_int32(0)

    def step(self, t):
        t = _f32(t)
        b = np.zeros(self.n, dtype=np.int32)
        theta = C.c_float(0)
        lib().orc_dtur(self.n, _p(self.rowptr, C.c_int32), _p(self.colidx, C.c_int32), len(self.edges),
                       _p(self.edges, C.c_int32), _p(self.visited, C.c_uint8), C.byref(self.n_visited),
                       _p(t, C.c_float), _p(b, C.c_int32), C.byref(theta))
        return b, float(theta.value)


class Decision(C.Structure):
    """One branch decision of a gradient evaluation (orc_decision in the C source): stage 0 / 1 =
    ReLU + pooling window of a convolutional stage, 16 + l = ReLU after fully connected layer l;
    alt = the outcome on the other side; gap = distance from turning in rounding units."""
    _fields_ = [("stage", C.c_int32), ("sample", C.c_int32), ("unit", C.c_int32), ("alt", C.c_int32),
                ("gap", C.c_double)]

    def key(self):
        return (self.stage, self.sample, self.unit, self.alt)

    def __repr__(self):
        return f"Decision(stage={self.stage}, sample={self.sample}, unit={self.unit}, alt={self.alt}, gap={self.gap:.3g})"


class _Branch(C.Structure):
    _fields_ = [("flips", C.POINTER(Decision)), ("n_flips", C.c_int32), ("near", C.POINTER(Decision)),
                ("near_cap", C.c_int32), ("n_near", C.c_int32), ("near_scale", C.c_double)]


NEAR_CAP = 4096


def _branch(flips, near_scale):
    """-> (orc_branch or None, keep-alive objects)."""
    if not flips and near_scale is None:
        return None, None
    br = _Branch()
    fl = (Decision * max(len(flips or ()), 1))()
    for k, f in enumerate(flips or ()):
        fl[k].stage, fl[k].sample, fl[k].unit, fl[k].alt = f.stage, f.sample, f.unit, f.alt
    br.flips, br.n_flips = fl, len(flips or ())
    near = (Decision * NEAR_CAP)() if near_scale is not None else None
    if near is not None:
        br.near, br.near_cap, br.near_scale = near, NEAR_CAP, float(near_scale)
    return br, (fl, near)


def _near_list(br, keep):
    if br is None or keep[1] is None:
        return None
    if br.n_near > NEAR_CAP:
        raise ValueError(f"{br.n_near} near decisions exceed the list capacity {NEAR_CAP}")
    out = []
    for k in range(br.n_near):
        e = keep[1][k]
        out.append(Decision(e.stage, e.sample, e.unit, e.alt, e.gap))
    return out


def grad_mlp(dims, params, x, y, loss_kind="xent", flips=None, near_scale=None):
    """One worker: params [d], x [B, dims[0]], y [B] -> (grad [d] fp32, loss float).
    loss_kind: "xent" (softmax cross-entropy) or "mse" (squared error of the softmax outputs).
    flips: decisions to take the other way; near_scale: also return, as a third result, the
    decisions closer than that many rounding units to turning."""
    dims = _i32(dims)
    params, x, y = _f32(params), _f32(x), _i32(y)
    grad = np.zeros_like(params)
    loss = C.c_double(0)
    br, keep = _branch(flips, near_scale)
    lib().orc_grad_mlp_loss(len(dims) - 1, _p(dims, C.c_int32), x.shape[0], _p(params, C.c_float),
                            _p(x, C.c_float), _p(y, C.c_int32), 1 if loss_kind == "mse" else 0,
                            _p(grad, C.c_float), C.byref(loss), C.byref(br) if br is not None else None)
    if near_scale is not None:
        return grad, loss.value, _near_list(br, keep)
    return grad, loss.value


def grad_cnn(shape, params, x, y, flips=None, near_scale=None):
    """One worker: shape = (C0, H, W, C1, C2, K, F, classes); flips / near_scale as grad_mlp."""
    shape = _i32(shape)
    params, x, y = _f32(params), _f32(x), _i32(y)
    grad = np.zeros_like(params)
    loss = C.c_double(0)
    br, keep = _branch(flips, near_scale)
    lib().orc_grad_cnn(_p(shape, C.c_int32), x.shape[0], _p(params, C.c_float), _p(x, C.c_float),
                       _p(y, C.c_int32), _p(grad, C.c_float), C.byref(loss), C.byref(br) if br is not None else None)
    if near_scale is not None:
        return grad, loss.value, _near_list(br, keep)
    return grad, loss.value


def grad_one(kind, desc, d, params_row, x, y, flips=None):
    """Worker-level entry with grad_all's (kind, descriptor): gradient [d] of one worker, with
    `flips` taken the other way."""
    desc = _i32(desc)
    if kind == 1:
        return grad_cnn(desc, params_row[:d], x.reshape(x.shape[0], -1), y, flips=flips)[0]
    return grad_mlp(desc[1:], params_row[:d], x.reshape(x.shape[0], -1), y,
                    loss_kind="mse" if kind == 2 else "xent", flips=flips)[0]


def grad_all(kind, desc, d, params, x, y, near_scale=None):
    """All workers: params [N, ld], x [N, B, in], y [N, B] -> (grad [N, ld], loss [N]).
    near_scale adds a third result: per worker, the list of decisions (ReLU signs, pooling
    maxima) closer than that many rounding units to turning (the gradient is discontinuous
    there, see grad_one's `flips`)."""
    desc = _i32(desc)
    params, x, y = _f32(params), _f32(x), _i32(y)
    n, ld = params.shape
    B = x.shape[1]
    in_dim = int(np.prod(x.shape[2:]))
    grad = np.zeros_like(params)
    loss = np.zeros(n, dtype=np.float64)
    near = n_near = None
    if near_scale is not None:
        near = (Decision * (n * NEAR_CAP))()
        n_near = np.zeros(n, dtype=np.int32)
    lib().orc_grad_all(int(kind), _p(desc, C.c_int32), n, C.c_int64(d), C.c_int64(ld), B,
                       C.c_int64(in_dim), _p(params, C.c_float), _p(x, C.c_float), _p(y, C.c_int32),
                       _p(grad, C.c_float), _p(loss, C.c_double), near, NEAR_CAP,
                       _p(n_near, C.c_int32) if n_near is not None else None,
                       C.c_double(near_scale if near_scale is not None else 0.0))
    if near_scale is None:
        return grad, loss
    if n_near.max(initial=0) > NEAR_CAP:
        raise ValueError(f"{n_near.max()} near decisions exceed the list capacity {NEAR_CAP}")
    lists = []
    for i in range(n):
        lists.append([Decision(e.stage, e.sample, e.unit, e.alt, e.gap)
                      for e in (near[i * NEAR_CAP + k] for k in range(n_near[i]))])
    return grad, loss, lists


def model_desc(desc):
    """(kind, int32 descriptor) for grad_all from a model description dict."""
    if desc["kind"] == "mlp":
        dims = desc["dims"]
        return (2 if desc.get("loss") == "mse" else 0), np.array([len(dims) - 1] + list(dims), dtype=np.int32)
    c, h, w = desc["in"]
    return 1, np.array([c, h, w, desc["c1"], desc["c2"], desc["k"], desc["fc"], desc["classes"]], dtype=np.int32)


def set_threads(n: int) -> int:
    """Threads for the loops over workers (default 1); returns the value in force."""
    lib().orc_set_threads(int(n))
    return int(lib().orc_get_threads())
