"""ctypes binding of the CPU oracle (oracle/lg_oracle.c) on NumPy arrays.

`Oracle(path)` binds one compiled oracle library; the module-level functions use the default
build (oracle/liblg_oracle.so).  Tests that plant mistakes bind a mutant build the same way.

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


def _p(a):
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"], "float32 C-contiguous arrays only"
    return a.ctypes.data_as(_fp)


def _check(rc, name):
    if rc != 0:
        raise ValueError(f"{name}: oracle rejected the arguments (status {rc})")


class Oracle:
    """One loaded oracle library.  Every method passes host pointers straight to the C function."""

    _p = staticmethod(_p)

    def __init__(self, path):
        L = ctypes.CDLL(path)
        L.lgo_num_threads.restype = ctypes.c_int
        L.lgo_conv_out_extent.restype = _i64
        L.lgo_conv_out_extent.argtypes = [_i64] * 4
        L.lgo_matmul.argtypes = [_fp, _fp, _fp] + [_i64] * 6 + [ctypes.c_int]
        L.lgo_matmul_t.argtypes = [_fp, _fp, _fp] + [_i64] * 6 + [ctypes.c_int] * 3
        L.lgo_conv2d_nhwc_hwcf.argtypes = [_fp, _fp, _fp] + [_i64] * 11 + [ctypes.c_int]
        L.lgo_conv1d_nwc_wcf.argtypes = [_fp, _fp, _fp] + [_i64] * 7 + [ctypes.c_int]
        L.lgo_im2col_nhwc.argtypes = [_fp, _fp] + [_i64] * 10
        L.lgo_dwconv1d_nwc_wc.argtypes = [_fp, _fp, _fp] + [_i64] * 6 + [ctypes.c_int]
        L.lgo_dwconv2d_nhwc_hwc.argtypes = [_fp, _fp, _fp] + [_i64] * 10 + [ctypes.c_int]
        L.lgo_reduce_rows.argtypes = [_fp, _fp] + [_i64] * 3 + [ctypes.c_int]
        L.lgo_reduce_cols.argtypes = [_fp, _fp] + [_i64] * 3 + [ctypes.c_int]
        L.lgo_transpose.argtypes = [_fp, _fp] + [_i64] * 4
        L.lgo_transpose_batched.argtypes = [_fp, _fp] + [_i64] * 10
        L.lgo_copy2d.argtypes = [_fp, _fp] + [_i64] * 4
        self._lib = L

    def lib(self):
        return self._lib

    def num_threads(self):
        return int(self._lib.lgo_num_threads())

    def conv_out_extent(self, n_in, k, s, d):
        return int(self._lib.lgo_conv_out_extent(n_in, k, s, d))

    def matmul(self, A, B, C=None, accumulate=False):
        """C[M,N] (+)= A[M,K] @ B[K,N]; returns C (allocated when not given)."""
        M, K = A.shape
        K2, N = B.shape
        assert K == K2
        if C is None:
            assert not accumulate
            C = np.empty((M, N), np.float32)
        assert C.shape == (M, N)
        _check(self._lib.lgo_matmul(_p(A), _p(B), _p(C), M, N, K, K, N, N, int(accumulate)), "matmul")
        return C


    def matmul_t(self, A, B, trans_a=False, trans_b=False, C=None, accumulate=False):
        """C[M,N] (+)= op(A) @ op(B); A is [K,M] when trans_a, B is [N,K] when trans_b."""
        K, M = A.shape if trans_a else A.shape[::-1]
        N = B.shape[0] if trans_b else B.shape[1]
        assert tuple(B.shape) == ((N, K) if trans_b else (K, N))
        if C is None:
            assert not accumulate
            C = np.empty((M, N), np.float32)
        assert C.shape == (M, N)
        _check(self._lib.lgo_matmul_t(_p(A), _p(B), _p(C), M, N, K, A.shape[1], B.shape[1], N,
                                      int(trans_a), int(trans_b), int(accumulate)), "matmul_t")
        return C

    def conv2d_nhwc_hwcf(self, I, Kf, O=None, stride=(1, 1), dilation=(1, 1), accumulate=False):
        N, H, W, C = I.shape
        KH, KW, C2, F = Kf.shape
        assert C == C2
        OH = self.conv_out_extent(H, KH, stride[0], dilation[0])
        OW = self.conv_out_extent(W, KW, stride[1], dilation[1])
        if O is None:
            assert not accumulate
            O = np.empty((N, OH, OW, F), np.float32)
        assert O.shape == (N, OH, OW, F)
        _check(self._lib.lgo_conv2d_nhwc_hwcf(_p(I), _p(Kf), _p(O), N, H, W, C, KH, KW, F,
                                          stride[0], stride[1], dilation[0], dilation[1],
                                          int(accumulate)), "conv2d_nhwc_hwcf")
        return O


    def conv1d_nwc_wcf(self, I, Kf, O=None, stride=1, dilation=1, accumulate=False):
        N, W, C = I.shape
        KW, C2, F = Kf.shape
        assert C == C2
        OW = self.conv_out_extent(W, KW, stride, dilation)
        if O is None:
            assert not accumulate
            O = np.empty((N, OW, F), np.float32)
        assert O.shape == (N, OW, F)
        _check(self._lib.lgo_conv1d_nwc_wcf(_p(I), _p(Kf), _p(O), N, W, C, KW, F, stride, dilation,
                                            int(accumulate)), "conv1d_nwc_wcf")
        return O

    def im2col_nhwc(self, I, KH, KW, stride=(1, 1), dilation=(1, 1)):
        N, H, W, C = I.shape
        OH = self.conv_out_extent(H, KH, stride[0], dilation[0])
        OW = self.conv_out_extent(W, KW, stride[1], dilation[1])
        col = np.empty((N * OH * OW, KH * KW * C), np.float32)
        _check(self._lib.lgo_im2col_nhwc(_p(I), _p(col), N, H, W, C, KH, KW,
                                     stride[0], stride[1], dilation[0], dilation[1]), "im2col_nhwc")
        return col


    def dwconv1d_nwc_wc(self, I, Kf, O=None, stride=1, dilation=1, accumulate=False):
        N, W, C = I.shape
        KW, C2 = Kf.shape
        assert C == C2
        OW = self.conv_out_extent(W, KW, stride, dilation)
        if O is None:
            assert not accumulate
            O = np.empty((N, OW, C), np.float32)
        assert O.shape == (N, OW, C)
        _check(self._lib.lgo_dwconv1d_nwc_wc(_p(I), _p(Kf), _p(O), N, W, C, KW, stride, dilation,
                                         int(accumulate)), "dwconv1d_nwc_wc")
        return O


    def dwconv2d_nhwc_hwc(self, I, Kf, O=None, stride=(1, 1), dilation=(1, 1), accumulate=False):
        N, H, W, C = I.shape
        KH, KW, C2 = Kf.shape
        assert C == C2
        OH = self.conv_out_extent(H, KH, stride[0], dilation[0])
        OW = self.conv_out_extent(W, KW, stride[1], dilation[1])
        if O is None:
            assert not accumulate
            O = np.empty((N, OH, OW, C), np.float32)
        assert O.shape == (N, OH, OW, C)
        _check(self._lib.lgo_dwconv2d_nhwc_hwc(_p(I), _p(Kf), _p(O), N, H, W, C, KH, KW,
                                           stride[0], stride[1], dilation[0], dilation[1],
                                           int(accumulate)), "dwconv2d_nhwc_hwc")
        return O


    def reduce_rows(self, x, out=None, accumulate=False):
        R, Cn = x.shape
        if out is None:
            assert not accumulate
            out = np.empty((R,), np.float32)
        assert out.shape == (R,)
        _check(self._lib.lgo_reduce_rows(_p(x), _p(out), R, Cn, Cn, int(accumulate)), "reduce_rows")
        return out


    def reduce_cols(self, x, out=None, accumulate=False):
        R, Cn = x.shape
        if out is None:
            assert not accumulate
            out = np.empty((Cn,), np.float32)
        assert out.shape == (Cn,)
        _check(self._lib.lgo_reduce_cols(_p(x), _p(out), R, Cn, Cn, int(accumulate)), "reduce_cols")
        return out


    def transpose(self, x):
        R, Cn = x.shape
        out = np.empty((Cn, R), np.float32)
        _check(self._lib.lgo_transpose(_p(x), _p(out), R, Cn, Cn, R), "transpose")
        return out


    def transpose_batched(self, x, out, R, Cn, ld_in, ld_out, B0, B1, is0, is1, os0, os1):
        """x and out are flat float32 arrays; writes into out and returns it."""
        assert x.ndim == 1 and out.ndim == 1
        if R and Cn and B0 and B1:
            assert (B0 - 1) * is0 + (B1 - 1) * is1 + (R - 1) * ld_in + Cn <= x.size
            assert (B0 - 1) * os0 + (B1 - 1) * os1 + (Cn - 1) * ld_out + R <= out.size
        _check(self._lib.lgo_transpose_batched(_p(x), _p(out), R, Cn, ld_in, ld_out, B0, B1,
                                               is0, is1, os0, os1), "transpose_batched")
        return out

    def copy2d(self, x):
        R, Cn = x.shape
        out = np.empty((R, Cn), np.float32)
        _check(self._lib.lgo_copy2d(_p(x), _p(out), R, Cn, Cn, Cn), "copy2d")
        return out


_default = None


def default():
    global _default
    if _default is None:
        _default = Oracle(_build.build(force=False))
    return _default


def lib():
    return default().lib()


def __getattr__(name):          # module-level matmul(), transpose(), ... use the default build
    if name.startswith("__"):
        raise AttributeError(name)
    return getattr(default(), name)
