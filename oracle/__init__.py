"""ctypes front end of the CPU oracle (oracle/wgrad_oracle.c).

Test infrastructure only: the test-suite, the smoke check and the benchmark's
cpu_baseline leg import this; the product package never does.  It contains no
arithmetic of its own: every function marshals numpy arrays into the C oracle.

Arrays: X [N,C,H,W], dY [N,K,Ho,Wo], dW [K,C,R,S] (float64 results).  Inputs may
be float32, float64, or uint16 holding bfloat16 bit patterns (upcast exactly in C).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "wgrad_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force=False):
    """Compile the C oracle with gcc (OpenMP over output elements only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "C", "H", "W", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w")]


def shape(N, C, H, W, K, R=3, S=3, stride=1, pad=1, stride_w=None, pad_w=None):
    return Shape(N, C, H, W, K, R, S, stride, stride if stride_w is None else stride_w,
                 pad, pad if pad_w is None else pad_w)


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        P = ctypes.POINTER
        L.oracle_out_h.argtypes = [P(Shape)]
        L.oracle_out_w.argtypes = [P(Shape)]
        L.oracle_wgrad_exact.argtypes = [P(Shape), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                         ctypes.c_void_p]
        L.oracle_wgrad_exact_at.argtypes = [P(Shape), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                            ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
        L.oracle_select.argtypes = [P(Shape), ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p,
                                    ctypes.c_void_p]
        L.oracle_wgrad_approx.argtypes = [P(Shape), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                          ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_void_p]
        L.oracle_select_topk.argtypes = [P(Shape), ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                         ctypes.c_void_p]
        L.oracle_wgrad_approx_topk.argtypes = [P(Shape), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int,
                                               ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.oracle_wgrad_exact_nhwc.argtypes = [P(Shape), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int,
                                              ctypes.c_void_p]
        L.oracle_wgrad_approx_nhwc.argtypes = [P(Shape), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int,
                                               ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.oracle_philox4x32_10.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.oracle_philox4x32_10.restype = None
        L.oracle_random_normal.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int64,
                                           ctypes.c_double, ctypes.c_void_p]
        L.oracle_random_normal.restype = None
        L.oracle_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


_DT = {np.dtype(np.float32): 0, np.dtype(np.uint16): 1, np.dtype(np.float64): 2}


def _prep(a):
    a = np.ascontiguousarray(a)
    if a.dtype not in _DT:
        raise TypeError(f"oracle input dtype {a.dtype}: use float32, float64 or uint16 (bf16 bits)")
    return a, _DT[a.dtype]


def _pair(X, dY):
    X, dx = _prep(X)
    dY, dy = _prep(dY)
    if dx != dy:
        raise TypeError("X and dY must share a dtype")
    return X, dY, dx


def out_hw(g):
    return lib().oracle_out_h(ctypes.byref(g)), lib().oracle_out_w(ctypes.byref(g))


def _check(g, X, dY):
    Ho, Wo = out_hw(g)
    assert X.shape == (g.N, g.C, g.H, g.W), (X.shape, (g.N, g.C, g.H, g.W))
    assert dY.shape == (g.N, g.K, Ho, Wo), (dY.shape, (g.N, g.K, Ho, Wo))


def wgrad_exact(g, X, dY):
    X, dY, dt = _pair(X, dY)
    _check(g, X, dY)
    dW = np.empty((g.K, g.C, g.R, g.S), np.float64)
    rc = lib().oracle_wgrad_exact(ctypes.byref(g), X.ctypes.data, dY.ctypes.data, dt, dW.ctypes.data)
    assert rc == 0
    return dW


def wgrad_exact_at(g, X, dY, flat_indices):
    X, dY, dt = _pair(X, dY)
    _check(g, X, dY)
    flat = np.ascontiguousarray(flat_indices, np.int64)
    assert flat.min(initial=0) >= 0 and flat.max(initial=0) < g.K * g.C * g.R * g.S
    out = np.empty(flat.shape, np.float64)
    rc = lib().oracle_wgrad_exact_at(ctypes.byref(g), X.ctypes.data, dY.ctypes.data, dt,
                                     flat.ctypes.data, flat.size, out.ctypes.data)
    assert rc == 0
    return out


def select(g, dY):
    dY, dt = _prep(dY)
    Ho, Wo = out_hw(g)
    assert dY.shape == (g.N, g.K, Ho, Wo)
    idx = np.empty((g.N, g.K), np.int32)
    S = np.empty((g.N, g.K), np.float64)
    rc = lib().oracle_select(ctypes.byref(g), dY.ctypes.data, dt, idx.ctypes.data, S.ctypes.data)
    assert rc == 0
    return idx, S


def wgrad_approx(g, X, dY, scale=1.0):
    """Returns (dW, idx, S)."""
    X, dY, dt = _pair(X, dY)
    _check(g, X, dY)
    dW = np.empty((g.K, g.C, g.R, g.S), np.float64)
    idx = np.empty((g.N, g.K), np.int32)
    S = np.empty((g.N, g.K), np.float64)
    rc = lib().oracle_wgrad_approx(ctypes.byref(g), X.ctypes.data, dY.ctypes.data, dt, float(scale),
                                   dW.ctypes.data, idx.ctypes.data, S.ctypes.data)
    assert rc == 0
    return dW, idx, S


def select_topk(g, dY, k):
    """Returns (idx [N,K,k], S [N,K]): the k largest-magnitude positions of every map, in order."""
    dY, dt = _prep(dY)
    Ho, Wo = out_hw(g)
    assert dY.shape == (g.N, g.K, Ho, Wo)
    idx = np.empty((g.N, g.K, k), np.int32)
    S = np.empty((g.N, g.K), np.float64)
    rc = lib().oracle_select_topk(ctypes.byref(g), dY.ctypes.data, dt, int(k), idx.ctypes.data, S.ctypes.data)
    assert rc == 0, rc
    return idx, S


def wgrad_approx_topk(g, X, dY, k, scale=1.0):
    """Returns (dW, idx [N,K,k], S)."""
    X, dY, dt = _pair(X, dY)
    _check(g, X, dY)
    dW = np.empty((g.K, g.C, g.R, g.S), np.float64)
    idx = np.empty((g.N, g.K, k), np.int32)
    S = np.empty((g.N, g.K), np.float64)
    rc = lib().oracle_wgrad_approx_topk(ctypes.byref(g), X.ctypes.data, dY.ctypes.data, dt, int(k), float(scale),
                                        dW.ctypes.data, idx.ctypes.data, S.ctypes.data)
    assert rc == 0, rc
    return dW, idx, S


# ---- the layouts of the paper's own kernel (Section 2.4): X channel-last, dY unchanged, dW as OHWI or HWIO ----
OIHW, OHWI, HWIO = 0, 1, 2


def dw_shape(g, layout):
    return {OIHW: (g.K, g.C, g.R, g.S), OHWI: (g.K, g.R, g.S, g.C), HWIO: (g.R, g.S, g.C, g.K)}[layout]


def _check_nhwc(g, X, dY):
    Ho, Wo = out_hw(g)
    assert X.shape == (g.N, g.H, g.W, g.C), (X.shape, (g.N, g.H, g.W, g.C))
    assert dY.shape == (g.N, g.K, Ho, Wo), (dY.shape, (g.N, g.K, Ho, Wo))


def wgrad_exact_nhwc(g, X, dY, dw_layout=OHWI):
    """Exact filter gradient from X[n,h,w,c] and dY[n,k,h,w], in the given dW layout."""
    X, dY, dt = _pair(X, dY)
    _check_nhwc(g, X, dY)
    dW = np.empty(dw_shape(g, dw_layout), np.float64)
    rc = lib().oracle_wgrad_exact_nhwc(ctypes.byref(g), X.ctypes.data, dY.ctypes.data, dt, int(dw_layout),
                                       dW.ctypes.data)
    assert rc == 0, rc
    return dW


def wgrad_approx_nhwc(g, X, dY, scale=1.0, dw_layout=OHWI):
    """Algorithm 1 from X[n,h,w,c] and dY[n,k,h,w]; returns (dW in the given layout, idx, S)."""
    X, dY, dt = _pair(X, dY)
    _check_nhwc(g, X, dY)
    dW = np.empty(dw_shape(g, dw_layout), np.float64)
    idx = np.empty((g.N, g.K), np.int32)
    S = np.empty((g.N, g.K), np.float64)
    rc = lib().oracle_wgrad_approx_nhwc(ctypes.byref(g), X.ctypes.data, dY.ctypes.data, dt, int(dw_layout),
                                        float(scale), dW.ctypes.data, idx.ctypes.data, S.ctypes.data)
    assert rc == 0, rc
    return dW, idx, S


def x_to_nhwc(X):
    """X[n,c,h,w] -> X[n,h,w,c]: the paper's input transpose (Section 2.4)."""
    return np.ascontiguousarray(np.asarray(X).transpose(0, 2, 3, 1))


def x_to_nchw(X):
    """X[n,h,w,c] -> X[n,c,h,w]."""
    return np.ascontiguousarray(np.asarray(X).transpose(0, 3, 1, 2))


def dw_permute(dW, src, dst):
    """Filter gradient from layout src to layout dst (the paper's second transpose is OHWI -> HWIO)."""
    to_oihw = {OIHW: (0, 1, 2, 3), OHWI: (0, 3, 1, 2), HWIO: (3, 2, 0, 1)}[src]
    from_oihw = {OIHW: (0, 1, 2, 3), OHWI: (0, 2, 3, 1), HWIO: (2, 3, 1, 0)}[dst]
    return np.ascontiguousarray(np.asarray(dW).transpose(to_oihw).transpose(from_oihw))


def philox4x32_10(counter, key):
    c = np.ascontiguousarray(counter, np.uint32)
    k = np.ascontiguousarray(key, np.uint32)
    assert c.shape == (4,) and k.shape == (2,)
    out = np.empty(4, np.uint32)
    lib().oracle_philox4x32_10(c.ctypes.data, k.ctypes.data, out.ctypes.data)
    return out


def random_normal(seed, offset, count, sigma):
    out = np.empty(count, np.float64)
    lib().oracle_random_normal(seed, offset, count, float(sigma), out.ctypes.data)
    return out


def num_threads():
    return lib().oracle_num_threads()
