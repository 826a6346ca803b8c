"""ctypes binding of liblg.so on torch device tensors (argument marshalling only)."""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblg.so")

_i64 = ctypes.c_int64
_vp = ctypes.c_void_p
_int = ctypes.c_int
_sz = ctypes.c_size_t

_SIGNATURES = {
    "lg_version": (_int, []),
    "lg_status_string": (ctypes.c_char_p, [_int]),
    "lg_conv_out_extent": (_i64, [_i64] * 4),
    "lg_matmul": (_int, [_vp, _vp, _vp] + [_i64] * 6 + [_int, _vp, _sz, _vp]),
    "lg_matmul_t": (_int, [_vp, _vp, _vp] + [_i64] * 6 + [_int, _int, _int, _vp, _sz, _vp]),
    "lg_matmul_workspace_bytes": (_sz, [_i64] * 3),
    "lg_matmul_plan": (_int, [_i64] * 3 + [ctypes.POINTER(_int)] * 3),
    "lg_matmul_t_plan": (_int, [_i64] * 3 + [_int, _int] + [ctypes.POINTER(_int)] * 3),
    "lg_matmul_plan_tile_loop": (_int, [_i64] * 3),
    "lg_gemm_variants": (_int, []),
    "lg_gemm_variant_info": (_int, [_int] + [ctypes.POINTER(_int)] * 5),
    "lg_gemm_variant_workspace_bytes": (_sz, [_i64] * 3 + [_int, _int]),
    "lg_matmul_variant": (_int, [_vp, _vp, _vp] + [_i64] * 6 + [_int] * 5 + [_vp, _sz, _vp]),
    "lg_conv2d_nhwc_hwcf_variant": (_int, [_vp, _vp, _vp] + [_i64] * 11 + [_int] * 3 + [_vp, _sz, _vp]),
    "lg_conv2d_nhwc_hwcf": (_int, [_vp, _vp, _vp] + [_i64] * 11 + [_int, _vp, _sz, _vp]),
    "lg_conv2d_workspace_bytes": (_sz, [_i64] * 11),
    "lg_conv1d_nwc_wcf": (_int, [_vp, _vp, _vp] + [_i64] * 7 + [_int, _vp, _sz, _vp]),
    "lg_conv1d_workspace_bytes": (_sz, [_i64] * 7),
    "lg_dwconv1d_nwc_wc": (_int, [_vp, _vp, _vp] + [_i64] * 6 + [_int, _vp]),
    "lg_dwconv2d_nhwc_hwc": (_int, [_vp, _vp, _vp] + [_i64] * 10 + [_int, _vp]),
    "lg_reduce_rows": (_int, [_vp, _vp] + [_i64] * 3 + [_int, _vp]),
    "lg_reduce_rows_ws": (_int, [_vp, _vp] + [_i64] * 3 + [_int, _vp, _sz, _vp]),
    "lg_reduce_rows_workspace_bytes": (_sz, [_i64] * 2),
    "lg_reduce_cols": (_int, [_vp, _vp] + [_i64] * 3 + [_int, _vp, _sz, _vp]),
    "lg_reduce_cols_workspace_bytes": (_sz, [_i64] * 2),
    "lg_reduce_cols_static": (_int, [_vp, _vp] + [_i64] * 3 + [_int, _vp]),
    "lg_transpose": (_int, [_vp, _vp] + [_i64] * 4 + [_vp]),
    "lg_transpose_batched": (_int, [_vp, _vp] + [_i64] * 10 + [_vp]),
    "lg_copy2d": (_int, [_vp, _vp] + [_i64] * 4 + [_vp]),
    "lg_mfma_probe": (_int, [_vp, _i64, _i64, _vp]),
    "lg_mfma_probe_out_elems": (_i64, []),
    "lg_mfma_probe_flops": (ctypes.c_double, [_i64]),
    "lg_stream_probe": (_int, [_int, _vp, _vp, _i64, _int, _int, _int, _vp]),
}

_lib = None


class LgError(RuntimeError):
    def __init__(self, name, status):
        self.status = status
        super().__init__(f"{name} failed: {lg_status_string(status)} ({status})")


def lib():
    """The loaded liblg.so; raises when it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2202_03293_amd.build` "
                              "(or __graft_entry__.build()) first")
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def exported_symbols():
    return sorted(_SIGNATURES)


def _ptr(t):
    if t is None:
        return None
    if not (t.is_cuda and t.dtype == torch.float32):
        raise TypeError("liblg takes float32 tensors in device memory")
    return t.data_ptr()


# torch.cuda.current_stream() builds a Stream object through several Python layers (~3 us, as much
# as the launch itself); the raw handle of the same stream is one C call away.
_raw_current_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream(stream):
    if stream is None:
        if _raw_current_stream is not None:
            return _raw_current_stream(torch.cuda.current_device())
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _ws(workspace):
    if workspace is None:
        return None, 0
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("workspace must be a contiguous device tensor")
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def _ld(t):
    """Row stride of a 2-D row-major tensor (last stride must be 1)."""
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("expected a 2-D tensor with unit stride in the last dimension")
    return t.stride(0) if t.shape[0] > 1 else t.shape[1]


def _dense(t):
    if not t.is_contiguous():
        raise ValueError("operands of this op must be dense (contiguous)")


def _check(name, status):
    if status != 0:
        raise LgError(name, status)


def lg_version():
    return lib().lg_version()


def lg_status_string(status):
    return lib().lg_status_string(status).decode()


def lg_conv_out_extent(n_in, k, stride, dilation):
    return lib().lg_conv_out_extent(n_in, k, stride, dilation)


def lg_matmul_workspace_bytes(M, N, K):
    return lib().lg_matmul_workspace_bytes(M, N, K)


def lg_matmul_plan(M, N, K):
    """(block_m, block_n, k_splits) the library picks for an M x N x K contraction."""
    bm, bn, sp = _int(), _int(), _int()
    _check("lg_matmul_plan", lib().lg_matmul_plan(M, N, K, ctypes.byref(bm), ctypes.byref(bn), ctypes.byref(sp)))
    return bm.value, bn.value, sp.value


def lg_matmul_t_plan(M, N, K, trans_a=False, trans_b=False):
    """(block_m, block_n, k_splits) for lg_matmul_t in the given operand layout."""
    bm, bn, sp = _int(), _int(), _int()
    _check("lg_matmul_t_plan", lib().lg_matmul_t_plan(M, N, K, int(trans_a), int(trans_b),
                                                      ctypes.byref(bm), ctypes.byref(bn), ctypes.byref(sp)))
    return bm.value, bn.value, sp.value


def lg_matmul(A, B, C, accumulate=False, workspace=None, stream=None):
    """C[M,N] (+)= A[M,K] @ B[K,N] on the device, in place in C."""
    M, K = A.shape
    K2, N = B.shape
    if K != K2 or tuple(C.shape) != (M, N):
        raise ValueError("matmul shapes do not agree")
    wp, wb = _ws(workspace)
    _check("lg_matmul", lib().lg_matmul(_ptr(A), _ptr(B), _ptr(C), M, N, K, _ld(A), _ld(B), _ld(C),
                                        int(accumulate), wp, wb, _stream(stream)))
    return C


def lg_matmul_t(A, B, C, trans_a=False, trans_b=False, accumulate=False, workspace=None, stream=None):
    """C[M,N] (+)= op(A) @ op(B); A is stored [K,M] when trans_a, B is stored [N,K] when trans_b."""
    M, N = C.shape
    K = A.shape[0] if trans_a else A.shape[1]
    if tuple(A.shape) != ((K, M) if trans_a else (M, K)) or tuple(B.shape) != ((N, K) if trans_b else (K, N)):
        raise ValueError("matmul shapes do not agree")
    wp, wb = _ws(workspace)
    _check("lg_matmul_t", lib().lg_matmul_t(_ptr(A), _ptr(B), _ptr(C), M, N, K, _ld(A), _ld(B), _ld(C),
                                            int(trans_a), int(trans_b), int(accumulate), wp, wb, _stream(stream)))
    return C


def lg_matmul_plan_tile_loop(M, N, K):
    """Whether lg_matmul's plan for (M, N, K) walks several tiles per workgroup."""
    return bool(lib().lg_matmul_plan_tile_loop(M, N, K))


def lg_gemm_variants():
    """Number of compiled GEMM decompositions; variants are numbered from 0."""
    return lib().lg_gemm_variants()


def lg_gemm_variant_info(variant):
    """(block_m, block_n, block_k, k_parts, tile_loop) of a variant."""
    v = [_int() for _ in range(5)]
    _check("lg_gemm_variant_info", lib().lg_gemm_variant_info(variant, *[ctypes.byref(x) for x in v]))
    return tuple(x.value for x in v)


def lg_gemm_variant_workspace_bytes(M, N, K, variant, k_splits=1):
    return lib().lg_gemm_variant_workspace_bytes(M, N, K, variant, k_splits)


def lg_matmul_variant(A, B, C, variant, k_splits=1, trans_a=False, trans_b=False, accumulate=False,
                      workspace=None, stream=None):
    """lg_matmul_t run by one chosen kernel variant and k-split instead of the planner's choice."""
    M, N = C.shape
    K = A.shape[0] if trans_a else A.shape[1]
    if tuple(A.shape) != ((K, M) if trans_a else (M, K)) or tuple(B.shape) != ((N, K) if trans_b else (K, N)):
        raise ValueError("matmul shapes do not agree")
    wp, wb = _ws(workspace)
    _check("lg_matmul_variant",
           lib().lg_matmul_variant(_ptr(A), _ptr(B), _ptr(C), M, N, K, _ld(A), _ld(B), _ld(C), int(trans_a),
                                   int(trans_b), int(accumulate), variant, k_splits, wp, wb, _stream(stream)))
    return C


def lg_conv2d_nhwc_hwcf_variant(I, Kf, O, variant, k_splits=1, stride=(1, 1), dilation=(1, 1), accumulate=False,
                                workspace=None, stream=None):
    """lg_conv2d_nhwc_hwcf run by one chosen kernel variant and k-split."""
    N, H, W, C = I.shape
    KH, KW, C2, F = Kf.shape
    if C != C2:
        raise ValueError("channel extents do not agree")
    for t in (I, Kf, O):
        _dense(t)
    OH = lg_conv_out_extent(H, KH, stride[0], dilation[0])
    OW = lg_conv_out_extent(W, KW, stride[1], dilation[1])
    if tuple(O.shape) != (N, OH, OW, F):
        raise ValueError(f"output must have shape {(N, OH, OW, F)}")
    wp, wb = _ws(workspace)
    _check("lg_conv2d_nhwc_hwcf_variant",
           lib().lg_conv2d_nhwc_hwcf_variant(_ptr(I), _ptr(Kf), _ptr(O), N, H, W, C, KH, KW, F,
                                             stride[0], stride[1], dilation[0], dilation[1],
                                             int(accumulate), variant, k_splits, wp, wb, _stream(stream)))
    return O


def lg_conv2d_workspace_bytes(N, H, W, C, KH, KW, F, SH=1, SW=1, DH=1, DW=1):
    return lib().lg_conv2d_workspace_bytes(N, H, W, C, KH, KW, F, SH, SW, DH, DW)


def lg_conv2d_nhwc_hwcf(I, Kf, O, stride=(1, 1), dilation=(1, 1), accumulate=False, workspace=None,
                        stream=None):
    """O[N,OH,OW,F] (+)= conv(I[N,H,W,C], Kf[KH,KW,C,F]), no padding."""
    N, H, W, C = I.shape
    KH, KW, C2, F = Kf.shape
    if C != C2:
        raise ValueError("channel extents do not agree")
    for t in (I, Kf, O):
        _dense(t)
    OH = lg_conv_out_extent(H, KH, stride[0], dilation[0])
    OW = lg_conv_out_extent(W, KW, stride[1], dilation[1])
    if tuple(O.shape) != (N, OH, OW, F):
        raise ValueError(f"output must have shape {(N, OH, OW, F)}")
    wp, wb = _ws(workspace)
    _check("lg_conv2d_nhwc_hwcf",
           lib().lg_conv2d_nhwc_hwcf(_ptr(I), _ptr(Kf), _ptr(O), N, H, W, C, KH, KW, F,
                                     stride[0], stride[1], dilation[0], dilation[1],
                                     int(accumulate), wp, wb, _stream(stream)))
    return O


def lg_conv1d_workspace_bytes(N, W, C, KW, F, SW=1, DW=1):
    return lib().lg_conv1d_workspace_bytes(N, W, C, KW, F, SW, DW)


def lg_conv1d_nwc_wcf(I, Kf, O, stride=1, dilation=1, accumulate=False, workspace=None, stream=None):
    """O[N,OW,F] (+)= conv(I[N,W,C], Kf[KW,C,F]), no padding."""
    N, W, C = I.shape
    KW, C2, F = Kf.shape
    if C != C2:
        raise ValueError("channel extents do not agree")
    for t in (I, Kf, O):
        _dense(t)
    OW = lg_conv_out_extent(W, KW, stride, dilation)
    if tuple(O.shape) != (N, OW, F):
        raise ValueError(f"output must have shape {(N, OW, F)}")
    wp, wb = _ws(workspace)
    _check("lg_conv1d_nwc_wcf",
           lib().lg_conv1d_nwc_wcf(_ptr(I), _ptr(Kf), _ptr(O), N, W, C, KW, F, stride, dilation,
                                   int(accumulate), wp, wb, _stream(stream)))
    return O


def lg_dwconv1d_nwc_wc(I, Kf, O, stride=1, dilation=1, accumulate=False, stream=None):
    """O[N,OW,C] (+)= depthwise conv(I[N,W,C], Kf[KW,C])."""
    N, W, C = I.shape
    KW, C2 = Kf.shape
    if C != C2:
        raise ValueError("channel extents do not agree")
    for t in (I, Kf, O):
        _dense(t)
    OW = lg_conv_out_extent(W, KW, stride, dilation)
    if tuple(O.shape) != (N, OW, C):
        raise ValueError(f"output must have shape {(N, OW, C)}")
    _check("lg_dwconv1d_nwc_wc",
           lib().lg_dwconv1d_nwc_wc(_ptr(I), _ptr(Kf), _ptr(O), N, W, C, KW, stride, dilation,
                                    int(accumulate), _stream(stream)))
    return O


def lg_dwconv2d_nhwc_hwc(I, Kf, O, stride=(1, 1), dilation=(1, 1), accumulate=False, stream=None):
    """O[N,OH,OW,C] (+)= depthwise conv(I[N,H,W,C], Kf[KH,KW,C])."""
    N, H, W, C = I.shape
    KH, KW, C2 = Kf.shape
    if C != C2:
        raise ValueError("channel extents do not agree")
    for t in (I, Kf, O):
        _dense(t)
    OH = lg_conv_out_extent(H, KH, stride[0], dilation[0])
    OW = lg_conv_out_extent(W, KW, stride[1], dilation[1])
    if tuple(O.shape) != (N, OH, OW, C):
        raise ValueError(f"output must have shape {(N, OH, OW, C)}")
    _check("lg_dwconv2d_nhwc_hwc",
           lib().lg_dwconv2d_nhwc_hwc(_ptr(I), _ptr(Kf), _ptr(O), N, H, W, C, KH, KW,
                                      stride[0], stride[1], dilation[0], dilation[1],
                                      int(accumulate), _stream(stream)))
    return O


def lg_reduce_rows(x, out, accumulate=False, stream=None):
    """out[R] (+)= sum over the last dimension of x[R,Cn]."""
    R, Cn = x.shape
    if tuple(out.shape) != (R,) or not out.is_contiguous():
        raise ValueError("out must be a dense vector with one entry per row")
    _check("lg_reduce_rows", lib().lg_reduce_rows(_ptr(x), _ptr(out), R, Cn, _ld(x), int(accumulate),
                                                  _stream(stream)))
    return out


def lg_reduce_rows_workspace_bytes(R, Cn):
    return lib().lg_reduce_rows_workspace_bytes(R, Cn)


def lg_reduce_rows_ws(x, out, accumulate=False, workspace=None, stream=None):
    """lg_reduce_rows with a workspace, which lets a handful of very long rows use the whole GPU."""
    R, Cn = x.shape
    if tuple(out.shape) != (R,) or not out.is_contiguous():
        raise ValueError("out must be a dense vector with one entry per row")
    wp, wb = _ws(workspace)
    _check("lg_reduce_rows_ws", lib().lg_reduce_rows_ws(_ptr(x), _ptr(out), R, Cn, _ld(x), int(accumulate),
                                                        wp, wb, _stream(stream)))
    return out


def lg_reduce_cols_workspace_bytes(R, Cn):
    return lib().lg_reduce_cols_workspace_bytes(R, Cn)


def lg_reduce_cols(x, out, accumulate=False, workspace=None, stream=None):
    """out[Cn] (+)= sum over the first dimension of x[R,Cn]."""
    R, Cn = x.shape
    if tuple(out.shape) != (Cn,) or not out.is_contiguous():
        raise ValueError("out must be a dense vector with one entry per column")
    wp, wb = _ws(workspace)
    _check("lg_reduce_cols", lib().lg_reduce_cols(_ptr(x), _ptr(out), R, Cn, _ld(x), int(accumulate),
                                                  wp, wb, _stream(stream)))
    return out


def lg_reduce_cols_static(x, out, accumulate=False, stream=None):
    """lg_reduce_cols without a workspace: partial sums go to the library's own fixed device array."""
    R, Cn = x.shape
    if tuple(out.shape) != (Cn,) or not out.is_contiguous():
        raise ValueError("out must be a dense vector with one entry per column")
    _check("lg_reduce_cols_static", lib().lg_reduce_cols_static(_ptr(x), _ptr(out), R, Cn, _ld(x), int(accumulate),
                                                                _stream(stream)))
    return out


def lg_transpose(x, out, stream=None):
    """out[Cn,R] = x[R,Cn] transposed, bit for bit."""
    R, Cn = x.shape
    if tuple(out.shape) != (Cn, R):
        raise ValueError("out must have the transposed shape")
    _check("lg_transpose", lib().lg_transpose(_ptr(x), _ptr(out), R, Cn, _ld(x), _ld(out), _stream(stream)))
    return out


def lg_copy2d(x, out, stream=None):
    """out[R,Cn] = x[R,Cn], bit for bit."""
    R, Cn = x.shape
    if tuple(out.shape) != (R, Cn):
        raise ValueError("out must have the same shape")
    _check("lg_copy2d", lib().lg_copy2d(_ptr(x), _ptr(out), R, Cn, _ld(x), _ld(out), _stream(stream)))
    return out


def lg_mfma_probe_out_elems():
    return int(lib().lg_mfma_probe_out_elems())


def lg_mfma_probe_flops(iters):
    return float(lib().lg_mfma_probe_flops(int(iters)))


def lg_mfma_probe(out, iters, stream=None):
    """Enqueue the register-only MFMA issue loop; `out` takes one checksum per lane."""
    _check("lg_mfma_probe", lib().lg_mfma_probe(_ptr(out), out.numel(), int(iters), _stream(stream)))
    return out


def lg_stream_probe(mode, x, out, threads=256, unroll=1, hint=3, stream=None):
    """Enqueue one HBM stream probe: mode "read" (x -> sink), "write" (-> out) or "copy" (x -> out)."""
    m = {"read": 0, "write": 1, "copy": 2}[mode]
    n = out.numel() if m == 1 else x.numel()
    if m == 2 and out.numel() != n:
        raise ValueError("copy probe: x and out must have the same number of elements")
    if m == 0 and out.numel() < 1024:
        raise ValueError("read probe: out is a sink of at least 1024 floats")
    _check("lg_stream_probe", lib().lg_stream_probe(m, _ptr(x), _ptr(out), n, threads, unroll, hint, _stream(stream)))
    return out


def lg_transpose_batched(x, out, R, Cn, ld_in, ld_out, B0, B1, in_strides, out_strides, stream=None):
    """B0 x B1 transposes of R x Cn matrices inside the flat tensors x and out; batch (b0, b1) starts
    at element b0*in_strides[0] + b1*in_strides[1] of x and likewise of out."""
    if x.dim() != 1 or out.dim() != 1:
        raise ValueError("x and out are passed flat (view(-1))")
    for t in (x, out):
        _dense(t)
    if R and Cn and B0 and B1:
        if (B0 - 1) * in_strides[0] + (B1 - 1) * in_strides[1] + (R - 1) * ld_in + Cn > x.numel():
            raise ValueError("batched transpose reads past the end of x")
        if (B0 - 1) * out_strides[0] + (B1 - 1) * out_strides[1] + (Cn - 1) * ld_out + R > out.numel():
            raise ValueError("batched transpose writes past the end of out")
    _check("lg_transpose_batched",
           lib().lg_transpose_batched(_ptr(x), _ptr(out), R, Cn, ld_in, ld_out, B0, B1,
                                      in_strides[0], in_strides[1], out_strides[0], out_strides[1],
                                      _stream(stream)))
    return out
