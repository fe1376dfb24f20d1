"""ctypes front end of the CPU oracle (``conv_ref.c``).

TEST INFRASTRUCTURE ONLY.  Tests, the smoke check and the benchmark's
``cpu_baseline`` leg import this module; the product package never does, and
this module imports nothing from the product package.

Arrays are numpy, contiguous: float32, float64, or uint16 holding bf16 bit
patterns.  Outputs are float64.  Shapes follow the operator definition in the
C file's header: x[N,C,H,W], w[K,C/groups,R,S], y/dy[N,K,P,Q].
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_ref.c")
_SRC_BN = os.path.join(_HERE, "bn_ref.c")
_LIB = os.path.join(_HERE, "libconvref.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc; returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_BN))
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, _SRC_BN, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        i = ctypes.c_int
        dims = [i] * 13  # N C H W K R S sh sw ph pw groups dtype
        for name in ("conv2d_fwd_ref", "conv2d_bwd_data_ref", "conv2d_bwd_weight_ref"):
            fn = getattr(_lib, name)
            fn.restype = i
            fn.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p] + dims
        for name in ("conv2d_fwd_ref_at", "conv2d_bwd_data_ref_at", "conv2d_bwd_weight_ref_at"):
            fn = getattr(_lib, name)
            fn.restype = i
            fn.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                           ctypes.c_void_p] + dims
        _lib.conv2d_fwd_bias_relu_ref.restype = i
        _lib.conv2d_fwd_bias_relu_ref.argtypes = [ctypes.c_void_p] * 4 + dims
        _lib.conv2d_bwd_data_relu_ref.restype = i
        _lib.conv2d_bwd_data_relu_ref.argtypes = [ctypes.c_void_p] * 4 + dims
        d = ctypes.c_double
        _lib.batchnorm2d_fwd_ref.restype = i
        _lib.batchnorm2d_fwd_ref.argtypes = [ctypes.c_void_p] * 6 + [i, i, i, i, d, i]
        _lib.batchnorm2d_bwd_ref.restype = i
        _lib.batchnorm2d_bwd_ref.argtypes = [ctypes.c_void_p] * 6 + [i, i, i, i, d, i]
        _lib.convref_num_threads.restype = i
    return _lib


def num_threads() -> int:
    return int(_load().convref_num_threads())


def out_hw(H, W, R, S, stride, pad):
    sh, sw = stride
    ph, pw = pad
    return (H + 2 * ph - R) // sh + 1, (W + 2 * pw - S) // sw + 1


def _pair(v):
    return (int(v), int(v)) if np.isscalar(v) else (int(v[0]), int(v[1]))


def _dtype_code(*arrs):
    dt = arrs[0].dtype
    for a in arrs:
        if a.dtype != dt:
            raise TypeError("oracle inputs must share one dtype")
        if not a.flags["C_CONTIGUOUS"]:
            raise ValueError("oracle inputs must be C-contiguous")
    if dt == np.float32:
        return 0
    if dt == np.uint16:
        return 1
    if dt == np.float64:
        return 2
    raise TypeError(f"unsupported oracle dtype {dt}")


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _check(rc):
    if rc != 0:
        raise ValueError(f"oracle rejected the problem (code {rc})")


def conv2d_fwd(x, w, stride=1, pad=0, groups=1):
    N, C, H, W = x.shape
    K, Cg, R, S = w.shape
    assert Cg * groups == C
    st, pd = _pair(stride), _pair(pad)
    P, Q = out_hw(H, W, R, S, st, pd)
    y = np.empty((N, K, P, Q), dtype=np.float64)
    _check(_load().conv2d_fwd_ref(_ptr(x), _ptr(w), _ptr(y), N, C, H, W, K, R, S,
                                  st[0], st[1], pd[0], pd[1], groups, _dtype_code(x, w)))
    return y


def conv2d_bwd_data(dy, w, x_shape, stride=1, pad=0, groups=1):
    N, C, H, W = x_shape
    K, Cg, R, S = w.shape
    assert Cg * groups == C
    st, pd = _pair(stride), _pair(pad)
    P, Q = out_hw(H, W, R, S, st, pd)
    assert dy.shape == (N, K, P, Q)
    dx = np.empty((N, C, H, W), dtype=np.float64)
    _check(_load().conv2d_bwd_data_ref(_ptr(dy), _ptr(w), _ptr(dx), N, C, H, W, K, R, S,
                                       st[0], st[1], pd[0], pd[1], groups, _dtype_code(dy, w)))
    return dx


def conv2d_bwd_weight(x, dy, w_shape, stride=1, pad=0, groups=1):
    N, C, H, W = x.shape
    K, Cg, R, S = w_shape
    assert Cg * groups == C
    st, pd = _pair(stride), _pair(pad)
    P, Q = out_hw(H, W, R, S, st, pd)
    assert dy.shape == (N, K, P, Q)
    dw = np.empty((K, Cg, R, S), dtype=np.float64)
    _check(_load().conv2d_bwd_weight_ref(_ptr(x), _ptr(dy), _ptr(dw), N, C, H, W, K, R, S,
                                         st[0], st[1], pd[0], pd[1], groups, _dtype_code(x, dy)))
    return dw


def _idx(idx):
    a = np.ascontiguousarray(idx, dtype=np.int64)
    return a, np.empty(a.shape, dtype=np.float64)


def conv2d_fwd_at(x, w, idx, stride=1, pad=0, groups=1):
    """Elements of y at flat indices ``idx`` (row-major over [N,K,P,Q])."""
    N, C, H, W = x.shape
    K, Cg, R, S = w.shape
    st, pd = _pair(stride), _pair(pad)
    a, out = _idx(idx)
    _check(_load().conv2d_fwd_ref_at(_ptr(x), _ptr(w), _ptr(a), a.size, _ptr(out), N, C, H, W, K, R, S,
                                     st[0], st[1], pd[0], pd[1], groups, _dtype_code(x, w)))
    return out


def conv2d_bwd_data_at(dy, w, x_shape, idx, stride=1, pad=0, groups=1):
    """Elements of dx at flat indices ``idx`` (row-major over [N,C,H,W])."""
    N, C, H, W = x_shape
    K, Cg, R, S = w.shape
    st, pd = _pair(stride), _pair(pad)
    a, out = _idx(idx)
    _check(_load().conv2d_bwd_data_ref_at(_ptr(dy), _ptr(w), _ptr(a), a.size, _ptr(out), N, C, H, W, K, R, S,
                                          st[0], st[1], pd[0], pd[1], groups, _dtype_code(dy, w)))
    return out


def conv2d_bwd_weight_at(x, dy, w_shape, idx, stride=1, pad=0, groups=1):
    """Elements of dw at flat indices ``idx`` (row-major over [K,C/groups,R,S])."""
    N, C, H, W = x.shape
    K, Cg, R, S = w_shape
    st, pd = _pair(stride), _pair(pad)
    a, out = _idx(idx)
    _check(_load().conv2d_bwd_weight_ref_at(_ptr(x), _ptr(dy), _ptr(a), a.size, _ptr(out), N, C, H, W, K, R, S,
                                            st[0], st[1], pd[0], pd[1], groups, _dtype_code(x, dy)))
    return out


def conv2d_fwd_bias_relu(x, w, bias, stride=1, pad=0, groups=1):
    """max(0, conv2d_fwd(x, w) + bias[k]); bias is widened to float64."""
    N, C, H, W = x.shape
    K, Cg, R, S = w.shape
    assert Cg * groups == C
    st, pd = _pair(stride), _pair(pad)
    P, Q = out_hw(H, W, R, S, st, pd)
    b = np.ascontiguousarray(bias, dtype=np.float64)
    assert b.shape == (K,)
    y = np.empty((N, K, P, Q), dtype=np.float64)
    _check(_load().conv2d_fwd_bias_relu_ref(_ptr(x), _ptr(w), _ptr(b), _ptr(y), N, C, H, W, K, R, S,
                                            st[0], st[1], pd[0], pd[1], groups, _dtype_code(x, w)))
    return y


def conv2d_bwd_data_relu(dy, w, act, stride=1, pad=0, groups=1):
    """conv2d_bwd_data(dy, w) where act > 0, else 0; act has the shape of x and the dtype of dy and w."""
    N, C, H, W = act.shape
    K, Cg, R, S = w.shape
    assert Cg * groups == C
    st, pd = _pair(stride), _pair(pad)
    P, Q = out_hw(H, W, R, S, st, pd)
    assert dy.shape == (N, K, P, Q)
    dx = np.empty((N, C, H, W), dtype=np.float64)
    _check(_load().conv2d_bwd_data_relu_ref(_ptr(dy), _ptr(w), _ptr(act), _ptr(dx), N, C, H, W, K, R, S,
                                            st[0], st[1], pd[0], pd[1], groups, _dtype_code(dy, w, act)))
    return dx


def batchnorm2d_fwd(x, gamma, beta, eps):
    """Training-mode batch normalisation.  Returns (y, mean, inv_std), all float64."""
    N, C, H, W = x.shape
    g = np.ascontiguousarray(gamma, dtype=np.float64)
    b = np.ascontiguousarray(beta, dtype=np.float64)
    assert g.shape == (C,) and b.shape == (C,)
    y = np.empty((N, C, H, W), dtype=np.float64)
    mean = np.empty(C, dtype=np.float64)
    inv_std = np.empty(C, dtype=np.float64)
    _check(_load().batchnorm2d_fwd_ref(_ptr(x), _ptr(g), _ptr(b), _ptr(y), _ptr(mean), _ptr(inv_std),
                                       N, C, H, W, float(eps), _dtype_code(x)))
    return y, mean, inv_std


def batchnorm2d_bwd(x, dy, gamma, eps):
    """Vector-Jacobian product of batchnorm2d_fwd.  Returns (dx, dgamma, dbeta), all float64."""
    N, C, H, W = x.shape
    assert dy.shape == x.shape
    g = np.ascontiguousarray(gamma, dtype=np.float64)
    assert g.shape == (C,)
    dx = np.empty((N, C, H, W), dtype=np.float64)
    dgamma = np.empty(C, dtype=np.float64)
    dbeta = np.empty(C, dtype=np.float64)
    _check(_load().batchnorm2d_bwd_ref(_ptr(x), _ptr(dy), _ptr(g), _ptr(dx), _ptr(dgamma), _ptr(dbeta),
                                       N, C, H, W, float(eps), _dtype_code(x, dy)))
    return dx, dgamma, dbeta
