"""Seeded synthetic inputs shared by the parity tests, the smoke check and the benchmark.

This module holds none of the ops' arithmetic.  It only produces host arrays:
tensor `t` of a configuration with seed `s` is stream (s, t) of a counter-based
generator, in row-major element order, so the CPU oracle and the GPU library see
byte-identical data regardless of how a tensor is chunked or which side asks first.

Generator: the SplitMix64 output function (Steele, Lea, Flood 2014) applied to
`key(s, t) + (i + 1) * 0x9E3779B97F4A7C15 mod 2^64` for element index i, where
`key` is the same function applied to a mix of seed and tensor id.  The top 24
bits give u = bits * 2^-24 in [0, 1), exactly representable in fp32.
"""
import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 24


def _mix(z):
    z = z ^ (z >> np.uint64(30))
    z = z * _M1
    z = z ^ (z >> np.uint64(27))
    z = z * _M2
    z = z ^ (z >> np.uint64(31))
    return z


def _key(seed, tensor_id):
    with np.errstate(over="ignore"):
        s = np.array([seed], dtype=np.uint64) * _GAMMA + np.array([tensor_id], dtype=np.uint64) * _M1
        return _mix(s + np.uint64(1))[0]


def bits24(seed, tensor_id, count, start=0):
    """24 random bits per element for indices start .. start+count-1 of stream (seed, tensor_id)."""
    out = np.empty(count, dtype=np.uint32)
    key = _key(seed, tensor_id)
    with np.errstate(over="ignore"):
        for lo in range(0, count, _CHUNK):
            hi = min(count, lo + _CHUNK)
            idx = np.arange(start + lo + 1, start + hi + 1, dtype=np.uint64)
            out[lo:hi] = (_mix(key + idx * _GAMMA) >> np.uint64(40)).astype(np.uint32)
    return out


def uniform(seed, tensor_id, shape, lo=0.0, hi=1.0):
    """float32 array of `shape`, i.i.d. uniform on [lo, hi) on a 2^-24-spaced grid."""
    count = int(np.prod(shape, dtype=np.int64)) if len(shape) else 1
    u = bits24(seed, tensor_id, count).astype(np.float32) * np.float32(2.0 ** -24)
    if lo != 0.0 or hi != 1.0:
        u = u * np.float32(hi - lo) + np.float32(lo)
    return u.reshape(shape)


def small_integers(seed, tensor_id, shape, lo=-4, hi=4):
    """float32 array of integers in [lo, hi]; sums of products of these are exact in fp32."""
    count = int(np.prod(shape, dtype=np.int64)) if len(shape) else 1
    b = bits24(seed, tensor_id, count).astype(np.int64)
    return (b % (hi - lo + 1) + lo).astype(np.float32).reshape(shape)


# ---------------------------------------------------------------------------
# Workload shapes.  Index = position in the benchmark configuration list:
# 0 small matmul, 1 memory-bound ops, 2 matmul sweep, 3 conv2d, 4 depthwise.
# ---------------------------------------------------------------------------
MATMUL_SMALL = (256, 256, 256)                       # seed 0
REDUCE_SHAPE = (4096, 16384)                         # seed 1, tensor 0
TRANSPOSE_SHAPE = (8192, 8192)                       # seed 1, tensor 1
MATMUL_SWEEP = [(1024, 1024, 1024), (4096, 4096, 4096), (8192, 8192, 8192),
                (16384, 512, 2048), (4096, 4096, 64)]  # (M, N, K), seed 2
# (N, H, W, C, F, KH, KW, stride), seed 3, dilation 1, no padding
CONV2D_SHAPES = [(8, 58, 58, 64, 64, 3, 3, 1), (8, 16, 16, 256, 256, 3, 3, 1),
                 (8, 56, 56, 256, 512, 1, 1, 2)]
# a conv large enough to fill the machine (118 GFLOP); not one of the configurations' shapes
CONV2D_LARGE = (32, 58, 58, 256, 256, 3, 3, 1)
DWCONV1D_SHAPE = (32, 4098, 512, 3)                  # (N, W, C, KW), seed 4
DWCONV2D_SHAPE = (8, 114, 114, 96, 3, 3)             # (N, H, W, C, KH, KW), seed 4


def matmul_inputs(seed, M, N, K, case=0):
    """A[M,K], B[K,N] uniform on [-1, 1)."""
    return (uniform(seed, 2 * case, (M, K), -1.0, 1.0),
            uniform(seed, 2 * case + 1, (K, N), -1.0, 1.0))


def conv2d_inputs(seed, N, H, W, C, F, KH, KW, case=0):
    """I[N,H,W,C], K[KH,KW,C,F] uniform on [-1, 1)."""
    return (uniform(seed, 2 * case, (N, H, W, C), -1.0, 1.0),
            uniform(seed, 2 * case + 1, (KH, KW, C, F), -1.0, 1.0))


def dwconv1d_inputs(seed, N, W, C, KW):
    return (uniform(seed, 0, (N, W, C), -1.0, 1.0), uniform(seed, 1, (KW, C), -1.0, 1.0))


def dwconv2d_inputs(seed, N, H, W, C, KH, KW):
    return (uniform(seed, 2, (N, H, W, C), -1.0, 1.0), uniform(seed, 3, (KH, KW, C), -1.0, 1.0))
