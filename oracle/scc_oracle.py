"""ctypes front end of the fp64 CPU oracle in ``scc_oracle.c``.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  The GPU library and its Python
binding never import this module, and this module never imports them.

Arrays go in as NumPy arrays of any float dtype and are widened to float64
before the C routines see them; results come back as float64.  Tensors are
``x[N, Cin, H, W]``, ``y/dy[N, Cout, H, W]``, ``w/dw[Cout, L]`` (Section 3.1 of the
paper: each filter takes 1/cg of the input channels; Section 4.2 for the
forward and backward definitions), depthwise filters ``kdw[C, 3, 3]`` (Eq. 2).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "scc_oracle.c")
_LIB = os.path.join(_HERE, "libscc_oracle.so")
_lib = None


def build(force=False):
    """Compile scc_oracle.c with gcc (-O2, a bare OpenMP parallel-for, nothing else)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        lib.scc_oracle_threads.restype = ctypes.c_int
        lib.scc_oracle_window.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_double, ip, ip]
        lib.scc_oracle_starts.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double, ip]
        for name in ("scc_oracle_forward", "scc_oracle_backward_input", "scc_oracle_backward_weight"):
            getattr(lib, name).argtypes = [dp, dp, dp] + [ctypes.c_int] * 5 + [ctypes.c_double]
            getattr(lib, name).restype = ctypes.c_int
        lib.scc_oracle_depthwise_out.argtypes = [ctypes.c_int, ctypes.c_int]
        lib.scc_oracle_depthwise_out.restype = ctypes.c_int
        lib.scc_oracle_depthwise3x3.argtypes = [dp, dp, dp] + [ctypes.c_int] * 5
        lib.scc_oracle_depthwise3x3.restype = ctypes.c_int
        lib.scc_oracle_depthwise3x3_backward.argtypes = [dp] * 5 + [ctypes.c_int] * 5
        lib.scc_oracle_depthwise3x3_backward.restype = ctypes.c_int
        _lib = lib
    return _lib


def _d(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def threads():
    """Host threads the oracle's parallel loops use."""
    return int(_load().scc_oracle_threads())


def window(Cin, cg, co):
    """(L, ov): window length Cin//cg and overlap int(co*L) of Algorithm 1."""
    L, ov = ctypes.c_int(), ctypes.c_int()
    if _load().scc_oracle_window(Cin, cg, float(co), ctypes.byref(L), ctypes.byref(ov)) != 0:
        raise ValueError("not an SCC layer: Cin=%r cg=%r co=%r" % (Cin, cg, co))
    return L.value, ov.value


def starts(Cin, Cout, cg, co):
    """Window start of each of the Cout filters (Algorithm 1 walked filter by filter)."""
    s = np.zeros(Cout, dtype=np.int32)
    rc = _load().scc_oracle_starts(Cin, Cout, cg, float(co), s.ctypes.data_as(ctypes.POINTER(ctypes.c_int)))
    if rc != 0:
        raise ValueError("not an SCC layer: Cin=%r Cout=%r cg=%r co=%r" % (Cin, Cout, cg, co))
    return s


def _check(rc):
    if rc != 0:
        raise ValueError("scc oracle rejected its arguments (rc=%d)" % rc)


def forward(x, w, cg, co):
    """y[n,k,h,w] = sum_j w[k,j] * x[n,(s_k+j) mod Cin,h,w]   (output-centric forward)."""
    x, w = _d(x), _d(w)
    N, Cin, H, W = x.shape
    Cout, L = w.shape
    assert L == window(Cin, cg, co)[0], "w must be [Cout, Cin//cg]"
    y = np.empty((N, Cout, H, W), dtype=np.float64)
    _check(_load().scc_oracle_forward(_ptr(x), _ptr(w), _ptr(y), N, Cin, Cout, H * W, cg, float(co)))
    return y


def backward_input(dy, w, Cin, cg, co):
    """dx[n,c,h,w] = sum over filters covering c of w[k,(c-s_k) mod Cin] * dy[n,k,h,w]."""
    dy, w = _d(dy), _d(w)
    N, Cout, H, W = dy.shape
    assert w.shape == (Cout, window(Cin, cg, co)[0])
    dx = np.empty((N, Cin, H, W), dtype=np.float64)
    _check(_load().scc_oracle_backward_input(_ptr(dy), _ptr(w), _ptr(dx), N, Cin, Cout, H * W, cg, float(co)))
    return dx


def backward_weight(x, dy, cg, co):
    """dw[k,j] = sum_{n,h,w} dy[n,k,h,w] * x[n,(s_k+j) mod Cin,h,w]."""
    x, dy = _d(x), _d(dy)
    N, Cin, H, W = x.shape
    Cout = dy.shape[1]
    assert dy.shape == (N, Cout, H, W)
    L = window(Cin, cg, co)[0]
    dw = np.empty((Cout, L), dtype=np.float64)
    _check(_load().scc_oracle_backward_weight(_ptr(x), _ptr(dy), _ptr(dw), N, Cin, Cout, H * W, cg, float(co)))
    return dw


def depthwise_out(size, stride):
    """Rows (or columns) the depthwise stage produces from `size` rows at spatial stride `stride`."""
    r = _load().scc_oracle_depthwise_out(int(size), int(stride))
    if r < 0:
        raise ValueError("not a depthwise stage: size=%r stride=%r" % (size, stride))
    return r


def depthwise3x3(x, kdw, stride=1):
    """z[n,a,m,q] = sum_{i,j<3} kdw[a,i,j] * x[n,a,stride*m+i-1,stride*q+j-1], zero outside the map (Eq. 2)."""
    x, kdw = _d(x), _d(kdw)
    N, C, H, W = x.shape
    assert kdw.shape == (C, 3, 3), "kdw must be [C, 3, 3]"
    z = np.empty((N, C, depthwise_out(H, stride), depthwise_out(W, stride)), dtype=np.float64)
    _check(_load().scc_oracle_depthwise3x3(_ptr(x), _ptr(kdw), _ptr(z), N, C, H, W, int(stride)))
    return z


def depthwise_scc_forward(x, kdw, w, cg, co, stride=1):
    """The DW + SCC block's forward: the SCC forward of the depthwise stage's output (Section 3.1 on Eq. 2)."""
    return forward(depthwise3x3(x, kdw, stride), w, cg, co)


def depthwise3x3_backward(x, kdw, dz, stride=1):
    """(dx, dkdw): the gradients of depthwise3x3 with respect to its input and its filters, given dz = dL/dz."""
    x, kdw, dz = _d(x), _d(kdw), _d(dz)
    N, C, H, W = x.shape
    assert kdw.shape == (C, 3, 3), "kdw must be [C, 3, 3]"
    assert dz.shape == (N, C, depthwise_out(H, stride), depthwise_out(W, stride)), "dz must have the shape of the stage's output"
    dx = np.empty_like(x)
    dk = np.empty((C, 3, 3), dtype=np.float64)
    _check(_load().scc_oracle_depthwise3x3_backward(_ptr(x), _ptr(kdw), _ptr(dz), _ptr(dx), _ptr(dk), N, C, H, W, int(stride)))
    return dx, dk
