"""ctypes binding of the CPU oracle (oracle/lg_oracle.c) on NumPy arrays.

Test infrastructure only: the GPU library and its Python binding never import
this module.  Every wrapper passes host pointers of C-contiguous float32 arrays
straight to the C function of the same name; there is no arithmetic here.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_i64 = ctypes.c_int64
_fp = ctypes.POINTER(ctypes.c_float)
_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        L.lgo_conv_out_extent.restype = _i64
        L.lgo_conv_out_extent.argtypes = [_i64] * 4
        L.lgo_matmul.argtypes = [_fp, _fp, _fp] + [_i64] * 6 + [ctypes.c_int]
        L.lgo_conv2d_nhwc_hwcf.argtypes = [_fp, _fp, _fp] + [_i64] * 11 + [ctypes.c_int]
        L.lgo_im2col_nhwc.argtypes = [_fp, _fp] + [_i64] * 10
        L.lgo_dwconv1d_nwc_wc.argtypes = [_fp, _fp, _fp] + [_i64] * 6 + [ctypes.c_int]
        L.lgo_dwconv2d_nhwc_hwc.argtypes = [_fp, _fp, _fp] + [_i64] * 10 + [ctypes.c_int]
        L.lgo_reduce_rows.argtypes = [_fp, _fp] + [_i64] * 3 + [ctypes.c_int]
        L.lgo_reduce_cols.argtypes = [_fp, _fp] + [_i64] * 3 + [ctypes.c_int]
        L.lgo_transpose.argtypes = [_fp, _fp] + [_i64] * 4
        L.lgo_copy2d.argtypes = [_fp, _fp] + [_i64] * 4
        _lib = L
    return _lib


def _p(a):
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"], "float32 C-contiguous arrays only"
    return a.ctypes.data_as(_fp)


def _check(rc, name):
    if rc != 0:
        raise ValueError(f"{name}: oracle rejected the arguments (status {rc})")


def num_threads():
    return int(lib().lgo_num_threads())


def conv_out_extent(n_in, k, s, d):
    return int(lib().lgo_conv_out_extent(n_in, k, s, d))


def matmul(A, B, C=None, accumulate=False):
    """C[M,N] (+)= A[M,K] @ B[K,N]; returns C (allocated when not given)."""
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    if C is None:
        assert not accumulate
        C = np.empty((M, N), np.float32)
    assert C.shape == (M, N)
    _check(lib().lgo_matmul(_p(A), _p(B), _p(C), M, N, K, K, N, N, int(accumulate)), "matmul")
    return C


def conv2d_nhwc_hwcf(I, Kf, O=None, stride=(1, 1), dilation=(1, 1), accumulate=False):
    N, H, W, C = I.shape
    KH, KW, C2, F = Kf.shape
    assert C == C2
    OH = conv_out_extent(H, KH, stride[0], dilation[0])
    OW = conv_out_extent(W, KW, stride[1], dilation[1])
    if O is None:
        assert not accumulate
        O = np.empty((N, OH, OW, F), np.float32)
    assert O.shape == (N, OH, OW, F)
    _check(lib().lgo_conv2d_nhwc_hwcf(_p(I), _p(Kf), _p(O), N, H, W, C, KH, KW, F,
                                      stride[0], stride[1], dilation[0], dilation[1],
                                      int(accumulate)), "conv2d_nhwc_hwcf")
    return O


def im2col_nhwc(I, KH, KW, stride=(1, 1), dilation=(1, 1)):
    N, H, W, C = I.shape
    OH = conv_out_extent(H, KH, stride[0], dilation[0])
    OW = conv_out_extent(W, KW, stride[1], dilation[1])
    col = np.empty((N * OH * OW, KH * KW * C), np.float32)
    _check(lib().lgo_im2col_nhwc(_p(I), _p(col), N, H, W, C, KH, KW,
                                 stride[0], stride[1], dilation[0], dilation[1]), "im2col_nhwc")
    return col


def dwconv1d_nwc_wc(I, Kf, O=None, stride=1, dilation=1, accumulate=False):
    N, W, C = I.shape
    KW, C2 = Kf.shape
    assert C == C2
    OW = conv_out_extent(W, KW, stride, dilation)
    if O is None:
        assert not accumulate
        O = np.empty((N, OW, C), np.float32)
    assert O.shape == (N, OW, C)
    _check(lib().lgo_dwconv1d_nwc_wc(_p(I), _p(Kf), _p(O), N, W, C, KW, stride, dilation,
                                     int(accumulate)), "dwconv1d_nwc_wc")
    return O


def dwconv2d_nhwc_hwc(I, Kf, O=None, stride=(1, 1), dilation=(1, 1), accumulate=False):
    N, H, W, C = I.shape
    KH, KW, C2 = Kf.shape
    assert C == C2
    OH = conv_out_extent(H, KH, stride[0], dilation[0])
    OW = conv_out_extent(W, KW, stride[1], dilation[1])
    if O is None:
        assert not accumulate
        O = np.empty((N, OH, OW, C), np.float32)
    assert O.shape == (N, OH, OW, C)
    _check(lib().lgo_dwconv2d_nhwc_hwc(_p(I), _p(Kf), _p(O), N, H, W, C, KH, KW,
                                       stride[0], stride[1], dilation[0], dilation[1],
                                       int(accumulate)), "dwconv2d_nhwc_hwc")
    return O


def reduce_rows(x, out=None, accumulate=False):
    R, Cn = x.shape
    if out is None:
        assert not accumulate
        out = np.empty((R,), np.float32)
    assert out.shape == (R,)
    _check(lib().lgo_reduce_rows(_p(x), _p(out), R, Cn, Cn, int(accumulate)), "reduce_rows")
    return out


def reduce_cols(x, out=None, accumulate=False):
    R, Cn = x.shape
    if out is None:
        assert not accumulate
        out = np.empty((Cn,), np.float32)
    assert out.shape == (Cn,)
    _check(lib().lgo_reduce_cols(_p(x), _p(out), R, Cn, Cn, int(accumulate)), "reduce_cols")
    return out


def transpose(x):
    R, Cn = x.shape
    out = np.empty((Cn, R), np.float32)
    _check(lib().lgo_transpose(_p(x), _p(out), R, Cn, Cn, R), "transpose")
    return out


def copy2d(x):
    R, Cn = x.shape
    out = np.empty((R, Cn), np.float32)
    _check(lib().lgo_copy2d(_p(x), _p(out), R, Cn, Cn, Cn), "copy2d")
    return out
