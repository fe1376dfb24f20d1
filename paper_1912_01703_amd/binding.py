"""Thin ctypes binding of ``libmiconv.so`` (the C ABI in ``include/miconv.h``).

Argument marshalling only: every function has the name and argument order of
its C counterpart and launches the library's HIP kernels.  Tensor arguments
may be anything with a ``data_ptr()`` method (e.g. a torch tensor on the GPU)
or a raw integer device address.  There is no CPU fallback: if the library has
not been built the import of this module fails.
"""
from __future__ import annotations

import ctypes
import os

# A process must hold exactly one HIP runtime.  Device buffers and streams come
# from torch, whose wheel bundles its own libamdhip64; importing torch first
# makes the loader resolve this library's HIP dependency to that same copy.
import torch  # noqa: F401

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmiconv.so")

OK, ERR_NULL, ERR_SHAPE, ERR_GROUPS, ERR_DTYPE, ERR_WORKSPACE, ERR_LAUNCH, ERR_UNSUPPORTED = range(8)
F32, BF16_F32ACC, BF16_BF16OUT = 0, 1, 2
PASS_FWD, PASS_BWD_DATA, PASS_BWD_WEIGHT = 0, 1, 2
ALGO_AUTO, ALGO_DIRECT, ALGO_MFMA, ALGO_DEPTHWISE = 0, 1, 2, 3

if not os.path.exists(_LIB_PATH):
    raise ImportError(
        f"{_LIB_PATH} is missing: build it first with `python -m paper_1912_01703_amd.build` "
        "(there is no fallback path)")

_lib = ctypes.CDLL(_LIB_PATH)

_i = ctypes.c_int
_dims = [_i] * 12  # N C H W K R S stride_h stride_w pad_h pad_w groups
for _name in ("conv2d_fwd", "conv2d_bwd_data", "conv2d_bwd_weight"):
    _fn = getattr(_lib, _name)
    _fn.restype = _i
    _fn.argtypes = [ctypes.c_void_p] * 3 + _dims + [_i, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
for _name in ("conv2d_fwd_bias_relu", "conv2d_bwd_data_relu_mask"):
    _fn = getattr(_lib, _name)
    _fn.restype = _i
    _fn.argtypes = [ctypes.c_void_p] * 4 + _dims + [_i, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.miconv_epilogue_is_fused.restype = _i
_lib.miconv_epilogue_is_fused.argtypes = [_i] + _dims + [_i]
_f = ctypes.c_float
_lib.batchnorm2d_fwd.restype = _i
_lib.batchnorm2d_fwd.argtypes = [ctypes.c_void_p] * 6 + [_i, _i, _i, _i, _f, _i, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.batchnorm2d_bwd.restype = _i
_lib.batchnorm2d_bwd.argtypes = [ctypes.c_void_p] * 8 + [_i, _i, _i, _i, _i, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.batchnorm2d_workspace_bytes.restype = ctypes.c_size_t
_lib.batchnorm2d_workspace_bytes.argtypes = [_i] * 6
_lib.conv2d_bwd_weight_static_ws.restype = _i
_lib.conv2d_bwd_weight_static_ws.argtypes = [ctypes.c_void_p] * 3 + _dims + [_i, ctypes.c_void_p]
_lib.conv2d_workspace_bytes.restype = ctypes.c_size_t
_lib.conv2d_workspace_bytes.argtypes = [_i] + _dims + [_i]
_lib.miconv_kernel_path.restype = ctypes.c_char_p
_lib.miconv_kernel_path.argtypes = [_i] + _dims + [_i]
_lib.miconv_sample_shader_clock.restype = _i
_lib.miconv_sample_shader_clock.argtypes = [ctypes.c_void_p, ctypes.c_uint, ctypes.POINTER(_i), ctypes.c_void_p]
_lib.miconv_set_algo.restype = _i
_lib.miconv_set_algo.argtypes = [_i, _i]
_lib.miconv_last_algo.restype = _i
_lib.miconv_last_algo.argtypes = [_i]
_lib.miconv_last_error.restype = ctypes.c_char_p
_lib.miconv_last_error.argtypes = []


class MiconvError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"miconv status {code}: {message}")
        self.code = code


def _ptr(t):
    if t is None:
        return None
    if hasattr(t, "data_ptr"):
        return ctypes.c_void_p(t.data_ptr())
    return ctypes.c_void_p(int(t))


def _ws(workspace):
    if workspace is None:
        return None, 0
    if hasattr(workspace, "data_ptr"):
        return ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()
    ptr, nbytes = workspace
    return ctypes.c_void_p(int(ptr)), int(nbytes)


def _call(fn, a, b, out, dims, dtype, workspace, stream, check):
    wptr, wbytes = _ws(workspace)
    rc = fn(_ptr(a), _ptr(b), _ptr(out), *[int(d) for d in dims], int(dtype), wptr, wbytes,
            ctypes.c_void_p(int(stream)) if stream else None)
    if check and rc != OK:
        raise MiconvError(rc, last_error())
    return rc


def conv2d_fwd(x, w, y, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups,
               dtype=F32, workspace=None, stream=0, check=True):
    return _call(_lib.conv2d_fwd, x, w, y, (N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups),
                 dtype, workspace, stream, check)


def conv2d_bwd_data(dy, w, dx, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups,
                    dtype=F32, workspace=None, stream=0, check=True):
    return _call(_lib.conv2d_bwd_data, dy, w, dx, (N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups),
                 dtype, workspace, stream, check)


def conv2d_bwd_weight(x, dy, dw, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups,
                      dtype=F32, workspace=None, stream=0, check=True):
    return _call(_lib.conv2d_bwd_weight, x, dy, dw, (N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups),
                 dtype, workspace, stream, check)


def _call4(fn, a, b, c, out, dims, dtype, workspace, stream, check):
    wptr, wbytes = _ws(workspace)
    rc = fn(_ptr(a), _ptr(b), _ptr(c), _ptr(out), *[int(d) for d in dims], int(dtype), wptr, wbytes,
            ctypes.c_void_p(int(stream)) if stream else None)
    if check and rc != OK:
        raise MiconvError(rc, last_error())
    return rc


def conv2d_fwd_bias_relu(x, w, bias, y, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups,
                         dtype=F32, workspace=None, stream=0, check=True):
    return _call4(_lib.conv2d_fwd_bias_relu, x, w, bias, y,
                  (N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups), dtype, workspace, stream, check)


def conv2d_bwd_data_relu_mask(dy, w, act, dx, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups,
                              dtype=F32, workspace=None, stream=0, check=True):
    return _call4(_lib.conv2d_bwd_data_relu_mask, dy, w, act, dx,
                  (N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups), dtype, workspace, stream, check)


def miconv_epilogue_is_fused(pass_, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups, dtype=F32) -> bool:
    return bool(_lib.miconv_epilogue_is_fused(int(pass_), N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w,
                                              groups, int(dtype)))


def batchnorm2d_fwd(x, gamma, beta, y, save_mean, save_inv_std, N, C, H, W, eps, dtype=F32, workspace=None, stream=0,
                    check=True):
    wptr, wbytes = _ws(workspace)
    rc = _lib.batchnorm2d_fwd(_ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), _ptr(save_mean), _ptr(save_inv_std),
                              N, C, H, W, float(eps), int(dtype), wptr, wbytes,
                              ctypes.c_void_p(int(stream)) if stream else None)
    if check and rc != OK:
        raise MiconvError(rc, last_error())
    return rc


def batchnorm2d_bwd(x, dy, gamma, save_mean, save_inv_std, dx, dgamma, dbeta, N, C, H, W, dtype=F32, workspace=None,
                    stream=0, check=True):
    wptr, wbytes = _ws(workspace)
    rc = _lib.batchnorm2d_bwd(_ptr(x), _ptr(dy), _ptr(gamma), _ptr(save_mean), _ptr(save_inv_std), _ptr(dx),
                              _ptr(dgamma), _ptr(dbeta), N, C, H, W, int(dtype), wptr, wbytes,
                              ctypes.c_void_p(int(stream)) if stream else None)
    if check and rc != OK:
        raise MiconvError(rc, last_error())
    return rc


def batchnorm2d_workspace_bytes(pass_, N, C, H, W, dtype=F32):
    return int(_lib.batchnorm2d_workspace_bytes(int(pass_), N, C, H, W, int(dtype)))


def conv2d_bwd_weight_static_ws(x, dy, dw, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups,
                                dtype=F32, stream=0, check=True):
    rc = _lib.conv2d_bwd_weight_static_ws(_ptr(x), _ptr(dy), _ptr(dw), N, C, H, W, K, R, S, stride_h, stride_w,
                                          pad_h, pad_w, groups, int(dtype),
                                          ctypes.c_void_p(int(stream)) if stream else None)
    if check and rc != OK:
        raise MiconvError(rc, last_error())
    return rc


def conv2d_workspace_bytes(pass_, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups, dtype=F32):
    return int(_lib.conv2d_workspace_bytes(int(pass_), N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w,
                                           groups, int(dtype)))


def miconv_kernel_path(pass_, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups, dtype=F32) -> str:
    return _lib.miconv_kernel_path(int(pass_), N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups,
                                   int(dtype)).decode()


def miconv_sample_shader_clock(counts, duration_us, stream=0, check=True):
    """Returns the constant-rate counter's frequency in kHz; `counts` (2 x int64 on the device) is filled by the
    kernel once it has run."""
    khz = _i(0)
    rc = _lib.miconv_sample_shader_clock(_ptr(counts), int(duration_us), ctypes.byref(khz),
                                         ctypes.c_void_p(int(stream)) if stream else None)
    if check and rc != OK:
        raise MiconvError(rc, "miconv_sample_shader_clock failed")
    return int(khz.value)


def miconv_set_algo(pass_, algo):
    return int(_lib.miconv_set_algo(int(pass_), int(algo)))


def miconv_last_algo(pass_):
    return int(_lib.miconv_last_algo(int(pass_)))


def last_error() -> str:
    return _lib.miconv_last_error().decode()


miconv_last_error = last_error
