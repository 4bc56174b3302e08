"""ctypes front end of ``lobra_oracle.c`` (test infrastructure, never the product path).

The arithmetic lives in the C file; this module only compiles it with gcc,
marshals numpy arrays and returns fp64 results.  Notation follows the C
header: ``A`` [R_tot, d_in] stacks the down projections, ``B`` [R_tot, d_out]
the up projections, ``rank_off`` [n_tasks+1] delimits each task's rows, ``s``
[n_tasks] is the per-task scale (paper section 2.1 has s = 1).

Arrays may be float32, or uint16 holding bf16 bit patterns; both are widened
exactly to double inside the C code.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lobra_oracle.c")
_SRC_ADAM = os.path.join(_HERE, "lobra_adam_oracle.c")
_LIB = os.path.join(_HERE, "liblobra_oracle.so")
_lock = threading.Lock()
_handle = None

F32, BF16 = 0, 1


def build_oracle(force: bool = False, src: str = _SRC, out: str = _LIB) -> str:
    """Compile the C oracle with gcc (-O2 -fopenmp, no fast-math). Returns the .so path."""
    srcs = [src, _SRC_ADAM]
    if (not force and os.path.exists(out)
            and os.path.getmtime(out) >= max(os.path.getmtime(f) for f in srcs)):
        return out
    tmp = out + ".tmp%d" % os.getpid()
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
           "-Wall", "-Wextra", "-o", tmp] + srcs + ["-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, out)
    return out


def _lib():
    global _handle
    with _lock:
        if _handle is None:
            _handle = _bind(ctypes.CDLL(build_oracle()))
    return _handle


def _bind(lib):
    i32p = ctypes.POINTER(ctypes.c_int32)
    i64p = ctypes.POINTER(ctypes.c_int64)
    f32p = ctypes.POINTER(ctypes.c_float)
    f64p = ctypes.POINTER(ctypes.c_double)
    vp = ctypes.c_void_p
    lib.lobra_oracle_token_task.restype = ctypes.c_int
    lib.lobra_oracle_token_task.argtypes = [
        ctypes.c_int64, ctypes.c_int32, i32p, i32p, ctypes.c_int32, i32p]
    lib.lobra_oracle_fwd.restype = ctypes.c_int
    lib.lobra_oracle_fwd.argtypes = [
        ctypes.c_int, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
        ctypes.c_int32, i32p, i32p, vp, vp, vp, vp, f32p,
        ctypes.c_int64, i64p, f64p, f64p]
    lib.lobra_oracle_bwd_dx.restype = ctypes.c_int
    lib.lobra_oracle_bwd_dx.argtypes = [
        ctypes.c_int, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
        ctypes.c_int32, i32p, i32p, vp, vp, vp, f32p, vp,
        ctypes.c_int64, i64p, f64p, f64p]
    lib.lobra_oracle_adam.restype = ctypes.c_int
    lib.lobra_oracle_adam.argtypes = [
        ctypes.c_int32, i32p, ctypes.c_int32, f64p, i32p, f64p,
        ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_double,
        f64p, f64p, f64p, f64p]
    lib.lobra_oracle_bwd_grads.restype = ctypes.c_int
    lib.lobra_oracle_bwd_grads.argtypes = [
        ctypes.c_int, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
        ctypes.c_int32, i32p, i32p, vp, vp, vp, f32p, vp, f64p, f64p]
    return lib


def _dtype_code(*arrays) -> int:
    kinds = {a.dtype for a in arrays if a is not None}
    if kinds == {np.dtype(np.float32)}:
        return F32
    if kinds == {np.dtype(np.uint16)}:
        return BF16
    raise TypeError("oracle inputs must all be float32, or all uint16 (bf16 bits); got %s" % kinds)


def _c(a, dtype=None):
    a = np.ascontiguousarray(a if dtype is None else np.asarray(a, dtype=dtype))
    return a


def _p(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _vp(a):
    return ctypes.c_void_p(a.ctypes.data)


def token_task(T, seg_off, seg_task, n_tasks):
    """Token -> task map [T] int32 of a segment table (-1 = no adapter)."""
    seg_off = _c(seg_off, np.int32)
    seg_task = _c(seg_task, np.int32)
    S = int(seg_task.shape[0])
    if seg_off.shape[0] != S + 1:
        raise ValueError("seg_off must have S+1 entries")
    out = np.empty(max(int(T), 0), dtype=np.int32)
    rc = _lib().lobra_oracle_token_task(
        int(T), S, _p(seg_off, ctypes.c_int32), _p(seg_task, ctypes.c_int32),
        int(n_tasks), _p(out, ctypes.c_int32))
    if rc != 0:
        raise ValueError("malformed segment table")
    return out


def _common(rank_off, task_of, s):
    rank_off = _c(rank_off, np.int32)
    task_of = _c(task_of, np.int32)
    s = _c(s, np.float32)
    n_tasks = int(rank_off.shape[0]) - 1
    if s.shape[0] < n_tasks:
        raise ValueError("s needs one entry per task")
    if s.shape[0] == 0:
        s = np.zeros(1, np.float32)
    r = np.diff(rank_off)
    r_max = int(r.max()) if n_tasks > 0 else 0
    return rank_off, task_of, s, n_tasks, r_max


def _empty_like_param(ref):
    # A / B of a problem without tasks: a valid non-null pointer of the same dtype.
    return np.zeros(1, dtype=ref.dtype)


def forward(x, W, A, B, s, rank_off, task_of, rows=None, want_h=False):
    """y rows (fp64) of  y_i = x_i W + s_t (A_t x_i) B_t ; rows=None means all tokens."""
    rank_off, task_of, s, n_tasks, r_max = _common(rank_off, task_of, s)
    x, W = _c(x), _c(W)
    A = _c(A) if n_tasks > 0 and A.size else _empty_like_param(x)
    B = _c(B) if n_tasks > 0 and B.size else _empty_like_param(x)
    dt = _dtype_code(x, W, A, B)
    T, d_in = x.shape
    d_out = W.shape[1]
    assert W.shape[0] == d_in and task_of.shape[0] == T
    if rows is None:
        nrows, rows_p = T, None
    else:
        rows = _c(rows, np.int64)
        assert rows.size == 0 or (rows.min() >= 0 and rows.max() < T)
        nrows, rows_p = int(rows.shape[0]), _p(rows, ctypes.c_int64)
    y = np.empty((nrows, d_out), dtype=np.float64)
    h = np.empty((nrows, r_max), dtype=np.float64) if want_h else None
    rc = _lib().lobra_oracle_fwd(
        dt, T, d_in, d_out, n_tasks, _p(rank_off, ctypes.c_int32),
        _p(task_of, ctypes.c_int32), _vp(x), _vp(W), _vp(A), _vp(B),
        _p(s, ctypes.c_float), nrows, rows_p, _p(y, ctypes.c_double),
        _p(h, ctypes.c_double) if want_h else None)
    if rc != 0:
        raise RuntimeError("lobra_oracle_fwd failed: %d" % rc)
    return (y, h) if want_h else y


def backward_dx(W, A, B, s, dy, rank_off, task_of, rows=None, want_g=False):
    """dx rows (fp64) of  dx_i = dy_i W^T + s_t (B_t dy_i) A_t."""
    rank_off, task_of, s, n_tasks, r_max = _common(rank_off, task_of, s)
    W, dy = _c(W), _c(dy)
    A = _c(A) if n_tasks > 0 and A.size else _empty_like_param(W)
    B = _c(B) if n_tasks > 0 and B.size else _empty_like_param(W)
    dt = _dtype_code(W, A, B, dy)
    d_in, d_out = W.shape
    T = dy.shape[0]
    assert dy.shape[1] == d_out and task_of.shape[0] == T
    if rows is None:
        nrows, rows_p = T, None
    else:
        rows = _c(rows, np.int64)
        assert rows.size == 0 or (rows.min() >= 0 and rows.max() < T)
        nrows, rows_p = int(rows.shape[0]), _p(rows, ctypes.c_int64)
    dx = np.empty((nrows, d_in), dtype=np.float64)
    g = np.empty((nrows, r_max), dtype=np.float64) if want_g else None
    rc = _lib().lobra_oracle_bwd_dx(
        dt, T, d_in, d_out, n_tasks, _p(rank_off, ctypes.c_int32),
        _p(task_of, ctypes.c_int32), _vp(W), _vp(A), _vp(B),
        _p(s, ctypes.c_float), _vp(dy), nrows, rows_p,
        _p(dx, ctypes.c_double), _p(g, ctypes.c_double) if want_g else None)
    if rc != 0:
        raise RuntimeError("lobra_oracle_bwd_dx failed: %d" % rc)
    return (dx, g) if want_g else dx


def backward_grads(x, A, B, s, dy, rank_off, task_of):
    """(dA [R_tot,d_in], dB [R_tot,d_out]) in fp64, summed over each task's tokens."""
    rank_off, task_of, s, n_tasks, _ = _common(rank_off, task_of, s)
    x, dy = _c(x), _c(dy)
    T, d_in = x.shape
    d_out = dy.shape[1]
    R_tot = int(rank_off[-1]) if n_tasks > 0 else 0
    dA = np.zeros((R_tot, d_in), dtype=np.float64)
    dB = np.zeros((R_tot, d_out), dtype=np.float64)
    if R_tot == 0:
        return dA, dB
    A, B = _c(A), _c(B)
    dt = _dtype_code(x, A, B, dy)
    assert A.shape == (R_tot, d_in) and B.shape == (R_tot, d_out)
    assert dy.shape[0] == T and task_of.shape[0] == T
    rc = _lib().lobra_oracle_bwd_grads(
        dt, T, d_in, d_out, n_tasks, _p(rank_off, ctypes.c_int32),
        _p(task_of, ctypes.c_int32), _vp(x), _vp(A), _vp(B),
        _p(s, ctypes.c_float), _vp(dy), _p(dA, ctypes.c_double),
        _p(dB, ctypes.c_double))
    if rc != 0:
        raise RuntimeError("lobra_oracle_bwd_grads failed: %d" % rc)
    return dA, dB


def adam_step(rank_off, lr, step, scale, beta1, beta2, eps, wd, grad, theta, m, v):
    """One Adam / AdamW step on a stacked [R_tot, d] parameter; returns new (theta, m, v) in fp64."""
    rank_off = _c(rank_off, np.int32)
    n_tasks = int(rank_off.shape[0]) - 1
    grad = _c(grad, np.float64)
    theta, m, v = (np.array(a, dtype=np.float64, order="C", copy=True) for a in (theta, m, v))
    assert grad.shape == theta.shape == m.shape == v.shape and grad.shape[0] == rank_off[-1]
    lr, scale = _c(lr, np.float64), _c(scale, np.float64)
    step = _c(step, np.int32)
    rc = _lib().lobra_oracle_adam(
        n_tasks, _p(rank_off, ctypes.c_int32), int(grad.shape[1]), _p(lr, ctypes.c_double),
        _p(step, ctypes.c_int32), _p(scale, ctypes.c_double), float(beta1), float(beta2),
        float(eps), float(wd), _p(grad, ctypes.c_double), _p(theta, ctypes.c_double),
        _p(m, ctypes.c_double), _p(v, ctypes.c_double))
    if rc != 0:
        raise ValueError("lobra_oracle_adam failed: %d" % rc)
    return theta, m, v


class Oracle:
    """All of the path for one problem: segment table in, fp64 y / dx / dA / dB out."""

    def __init__(self, x, W, A, B, s, dy, rank_off, seg_off, seg_task):
        self.x, self.W, self.A, self.B, self.dy = x, W, A, B, dy
        self.s = np.asarray(s, np.float32)
        self.rank_off = np.asarray(rank_off, np.int32)
        self.n_tasks = self.rank_off.shape[0] - 1
        self.task_of = token_task(x.shape[0], seg_off, seg_task, self.n_tasks)

    def y(self, rows=None):
        return forward(self.x, self.W, self.A, self.B, self.s, self.rank_off,
                       self.task_of, rows)

    def dx(self, rows=None):
        return backward_dx(self.W, self.A, self.B, self.s, self.dy,
                           self.rank_off, self.task_of, rows)

    def grads(self):
        return backward_grads(self.x, self.A, self.B, self.s, self.dy,
                              self.rank_off, self.task_of)


class FusedProjections:
    """Several layers that read the same x (the q/k/v projections of an attention block, gate/up of
    an MLP: the LoRA linears of one transformer layer that section 2.1 adapts), each computed by the oracle above
    on its own slice - nothing is fused here, the definition is "P separate layers":

        y[:, j]  = layer_j(x)                 dx = sum_j dx_j
        dA rows (t, j, :) = dA_t of layer j   dB rows (t, j, :) = dB_t of layer j

    Layouts as the library takes them: W [d_in, P dg], y/dy [T, P dg], every task's rank rows stacked
    P times in A [R_tot, d_in] (rows j r_t .. (j+1) r_t - 1 of task t belong to layer j), B [R_tot, dg].
    """

    def __init__(self, n_proj, x, W, A, B, s, dy, rank_off, seg_off, seg_task):
        P = int(n_proj)
        rank_off = np.asarray(rank_off, np.int64)
        ranks = np.diff(rank_off)
        if (ranks % P).any() or W.shape[1] % P or dy.shape[1] != W.shape[1]:
            raise ValueError("ranks and d_out must be multiples of the number of projections")
        self.P, self.dg = P, W.shape[1] // P
        self.sub_ranks = ranks // P
        sub_off = np.concatenate([[0], np.cumsum(self.sub_ranks)]).astype(np.int32)
        # rows of the stacked factors that belong to layer j, in task order
        self.rows = []
        for j in range(P):
            idx = [np.arange(rank_off[t] + j * r, rank_off[t] + (j + 1) * r) for t, r in enumerate(self.sub_ranks)]
            self.rows.append(np.concatenate(idx).astype(np.int64) if idx else np.zeros(0, np.int64))
        self.R_tot = int(rank_off[-1])
        self.layers = []
        for j in range(P):
            cols = slice(j * self.dg, (j + 1) * self.dg)
            self.layers.append(Oracle(x, np.ascontiguousarray(W[:, cols]), np.ascontiguousarray(A[self.rows[j]]),
                                      np.ascontiguousarray(B[self.rows[j]]), s, np.ascontiguousarray(dy[:, cols]),
                                      sub_off, seg_off, seg_task))

    def y(self, rows=None):
        return np.concatenate([L.y(rows) for L in self.layers], axis=1)

    def dx(self, rows=None):
        out = self.layers[0].dx(rows)
        for L in self.layers[1:]:
            out = out + L.dx(rows)
        return out

    def grads(self):
        d_in = self.layers[0].x.shape[1]
        dA = np.zeros((self.R_tot, d_in), np.float64)
        dB = np.zeros((self.R_tot, self.dg), np.float64)
        for j, L in enumerate(self.layers):
            a, b = L.grads()
            dA[self.rows[j]] = a
            dB[self.rows[j]] = b
        return dA, dB
