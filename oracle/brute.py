"""ctypes loader for the brute-force C loops in `brute.c`.

TEST INFRASTRUCTURE ONLY (see `oracle/__init__.py`).  `build()` compiles
`brute.c` with gcc into `libbrute.so` next to it; the functions below marshal
numpy arrays and return float64 / int64 results.  No arithmetic happens here.
"""

from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "brute.c")
_LIB = os.path.join(_HERE, "libbrute.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile brute.c (portable x86-64 code: the library travels to another host)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-Wall",
                        "-Wextra", "-o", _LIB, _SRC], check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(_LIB)
    return _lib


def num_threads() -> int:
    """Threads the OpenMP loops use on this host."""
    return int(os.environ.get("OMP_NUM_THREADS", 0)) or len(os.sched_getaffinity(0))


def _kind(*arrays):
    if all(np.issubdtype(np.asarray(a).dtype, np.integer) for a in arrays):
        return "i64", np.int64, ctypes.c_int64
    return "f64", np.float64, ctypes.c_double


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _i64(*xs):
    return [ctypes.c_int64(int(x)) for x in xs]


def conv2d(A, W, stride, pad=(0, 0)):
    """(N,C,H,W) x (O,C,Kh,Kw) -> (N,O,H',W') by the 2D-convolution equation of Sec. 5.1."""
    suffix, dt, _ = _kind(A, W)
    A = np.ascontiguousarray(A, dtype=dt)
    W = np.ascontiguousarray(W, dtype=dt)
    n, c, h, w = A.shape
    o, c2, kh, kw = W.shape
    if c != c2:
        raise ValueError("channel mismatch")
    ho = (h + 2 * pad[0] - kh) // stride[0] + 1
    wo = (w + 2 * pad[1] - kw) // stride[1] + 1
    out = np.empty((n, o, ho, wo), dtype=dt)
    fn = getattr(_load(), "brute_conv2d_" + suffix)
    rc = fn(_ptr(A), _ptr(W), _ptr(out), *_i64(n, c, h, w, o, kh, kw, stride[0], stride[1],
                                               pad[0], pad[1]))
    if rc:
        raise ValueError("brute_conv2d rejected the shapes")
    return out


def max_pool2d(A, window, stride, pad=(0, 0), fill=None):
    """(N,C,H,W) -> (N,C,H',W') by the max-pooling equation of Sec. 5.1."""
    suffix, dt, ct = _kind(A)
    A = np.ascontiguousarray(A, dtype=dt)
    n, c, h, w = A.shape
    ho = (h + 2 * pad[0] - window[0]) // stride[0] + 1
    wo = (w + 2 * pad[1] - window[1]) // stride[1] + 1
    if fill is None:
        if any(pad):
            raise ValueError("padded max-pool needs a fill value")
        fill = 0
    out = np.empty((n, c, ho, wo), dtype=dt)
    fn = getattr(_load(), "brute_maxpool_" + suffix)
    rc = fn(_ptr(A), _ptr(out), *_i64(n, c, h, w, window[0], window[1], stride[0], stride[1],
                                      pad[0], pad[1]), ct(fill))
    if rc:
        raise ValueError("brute_maxpool rejected the shapes")
    return out


def matmul(P, Q):
    """R[i,j] = sum_k P[i,k] Q[k,j]  (Sec. 3.1)."""
    suffix, dt, _ = _kind(P, Q)
    P = np.ascontiguousarray(P, dtype=dt)
    Q = np.ascontiguousarray(Q, dtype=dt)
    i, k = P.shape
    k2, j = Q.shape
    if k != k2:
        raise ValueError("inner dimension mismatch")
    R = np.empty((i, j), dtype=dt)
    getattr(_load(), "brute_matmul_" + suffix)(_ptr(P), _ptr(Q), _ptr(R), *_i64(i, k, j))
    return R


def row_reduce(X, is_max: bool):
    """Sum or max over the last axis of a 2D array."""
    suffix, dt, _ = _kind(X)
    X = np.ascontiguousarray(X, dtype=dt)
    rows, cols = X.shape
    out = np.empty((rows,), dtype=dt)
    rc = getattr(_load(), "brute_rowreduce_" + suffix)(_ptr(X), _ptr(out), *_i64(rows, cols),
                                                       ctypes.c_int(1 if is_max else 0))
    if rc:
        raise ValueError("brute_rowreduce rejected the shapes")
    return out
