"""Pins for the CPU oracle: everything here runs without a GPU.

The oracle is the naive loop nest of each op's definition; these tests tie it to
things that are not the oracle: hand-worked literals, facts the paper states,
closed forms, exact rational arithmetic, NumPy/SciPy library routines on the
special cases that reduce to them, and identities between different oracle
functions.  Shapes are asymmetric everywhere (M != N != K, KH != KW, SH != SW,
DH != DW) so that a transposed operand or swapped index fails.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy import signal

import seeded_inputs as si

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_examples.txt")


def golden(tag):
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            t, _cite, data = [s.strip() for s in line.split("|")]
            if t == tag:
                rows.append([int(x) for x in data.split()])
    assert rows
    return rows


def ulp32(x):
    x = np.abs(np.asarray(x, np.float64))
    e = np.floor(np.log2(np.maximum(x, 2.0 ** -126)))
    return 2.0 ** (e - 23)


def assert_half_ulp(got, exact):
    """got (fp32) is the fp32 rounding of exact (fp64 or Fraction-derived) up to fp64 noise."""
    got = np.asarray(got, np.float64)
    exact = np.asarray(exact, np.float64)
    assert np.all(np.abs(got - exact) <= 0.5 * ulp32(exact) * (1 + 1e-6) + 1e-300)


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


# --------------------------------------------------------------------------- matmul

def test_matmul_hand_literals(lgo):
    A = np.array([[1, 2], [3, 4]], np.float32)
    B = np.array([[5, 6], [7, 8]], np.float32)
    assert lgo.matmul(A, B).tolist() == [[19, 22], [43, 50]]
    A = np.array([[1, -2, 3], [0, 4, -1]], np.float32)          # 2x3
    B = np.array([[2, 1, 0, -1], [1, 0, 3, 2], [-2, 5, 1, 0]], np.float32)  # 3x4
    # row0: [2-2-6, 1+0+15, 0-6+3, -1-4+0]; row1: [0+4+2, 0+0-5, 0+12-1, 0+8+0]
    assert lgo.matmul(A, B).tolist() == [[-6, 16, -3, -5], [6, -5, 11, 8]]
    assert lgo.matmul(np.array([[3]], np.float32), np.array([[-7]], np.float32)).tolist() == [[-21]]


def test_matmul_all_ones_paper_example(lgo):
    for M, K, N, expect in golden("matmul_all_ones"):
        C = np.zeros((M, N), np.float32)
        lgo.matmul(np.ones((M, K), np.float32), np.ones((K, N), np.float32), C)
        assert np.all(C == np.float32(expect))


def test_matmul_identity_and_permutation_bit_exact(lgo):
    A = si.uniform(11, 0, (37, 23), -1, 1)
    assert np.array_equal(bits(lgo.matmul(A, np.eye(23, dtype=np.float32))), bits(A))
    assert np.array_equal(bits(lgo.matmul(np.eye(37, dtype=np.float32), A)), bits(A))
    perm = np.random.default_rng(5).permutation(37)
    P = np.zeros((37, 37), np.float32)
    P[np.arange(37), perm] = 1            # (P A)[i] = A[perm[i]]
    assert np.array_equal(bits(lgo.matmul(P, A)), bits(A[perm]))
    permc = np.random.default_rng(6).permutation(23)
    Q = np.zeros((23, 23), np.float32)
    Q[permc, np.arange(23)] = 1           # (A Q)[:, j] = A[:, permc[j]]
    assert np.array_equal(bits(lgo.matmul(A, Q)), bits(A[:, permc]))


def test_matmul_closed_form(lgo):
    M, N, K = 19, 31, 13
    A = np.repeat(np.arange(M, dtype=np.float32)[:, None], K, 1)      # A[m,k] = m
    B = np.repeat(np.arange(N, dtype=np.float32)[None, :], K, 0)      # B[k,n] = n
    C = lgo.matmul(A, B)
    assert np.array_equal(C, (K * np.outer(np.arange(M), np.arange(N))).astype(np.float32))
    # A[m,k] = k+1, B[k,n] = (n+1): C = (n+1) * K(K+1)/2 ; catches a dropped k term
    A = np.repeat(np.arange(1, K + 1, dtype=np.float32)[None, :], M, 0)
    B = np.repeat(np.arange(1, N + 1, dtype=np.float32)[None, :], K, 0)
    C = lgo.matmul(A, B)
    assert np.array_equal(C, np.repeat(((K * (K + 1) // 2) * np.arange(1, N + 1))[None, :], M, 0)
                          .astype(np.float32))


def test_matmul_exact_rational_bruteforce(lgo):
    M, N, K = 5, 7, 11
    A, B = si.matmul_inputs(21, M, N, K)
    C = lgo.matmul(A, B)
    for m in range(M):
        for n in range(N):
            ex = sum(Fraction(float(A[m, k])) * Fraction(float(B[k, n])) for k in range(K))
            assert_half_ulp(C[m, n], float(ex))


def test_matmul_vs_numpy_fp64(lgo):
    for (M, N, K) in [(64, 48, 200), (33, 130, 1), (1, 1, 777), (130, 3, 65)]:
        A, B = si.matmul_inputs(22, M, N, K)
        C = lgo.matmul(A, B)
        assert_half_ulp(C, A.astype(np.float64) @ B.astype(np.float64))


def test_matmul_leading_dims_and_accumulate(lgo):
    M, N, K = 9, 14, 6
    A, B = si.matmul_inputs(23, M, N, K)
    C0 = si.uniform(23, 9, (M, N), -1, 1)
    ref = lgo.matmul(A, B)
    Ap = np.full((M, K + 3), np.nan, np.float32); Ap[:, :K] = A
    Bp = np.full((K, N + 5), np.nan, np.float32); Bp[:, :N] = B
    Cp = np.full((M, N + 2), 7.0, np.float32)
    rc = lgo.lib().lgo_matmul(lgo._p(Ap), lgo._p(Bp), lgo._p(Cp), M, N, K, K + 3, N + 5, N + 2, 0)
    assert rc == 0
    assert np.array_equal(bits(Cp[:, :N]), bits(ref)) and np.all(Cp[:, N:] == 7.0)
    C = C0.copy()
    lgo.matmul(A, B, C, accumulate=True)
    assert_half_ulp(C, A.astype(np.float64) @ B.astype(np.float64) + C0.astype(np.float64))
    # zero reduction extent: overwrite gives the neutral element, accumulate leaves C alone
    Z = np.full((3, 4), 5.0, np.float32)
    lgo.matmul(np.empty((3, 0), np.float32), np.empty((0, 4), np.float32), Z)
    assert np.all(Z == 0)
    Z = np.full((3, 4), 5.0, np.float32)
    lgo.matmul(np.empty((3, 0), np.float32), np.empty((0, 4), np.float32), Z, accumulate=True)
    assert np.all(Z == 5.0)
    assert lgo.lib().lgo_matmul(lgo._p(Ap), lgo._p(Bp), lgo._p(Cp), M, N, K, K - 1, N, N, 0) == -1


def test_matmul_linearity_power_of_two(lgo):
    A, B = si.matmul_inputs(24, 12, 10, 40)
    assert np.array_equal(bits(lgo.matmul(A * np.float32(4), B)), bits(lgo.matmul(A, B) * np.float32(4)))


def test_matmul_transposed_operands(lgo):
    # hand literal: A stored K x M = [[1,2],[3,4],[5,6]] (K=3, M=2), B stored K x N = [[1,0],[0,1],[1,1]]
    At = np.array([[1, 2], [3, 4], [5, 6]], np.float32)
    B = np.array([[1, 0], [0, 1], [1, 1]], np.float32)
    # C[m,n] = sum_k At[k,m] B[k,n]: row0 = [1+5, 3+5], row1 = [2+6, 4+6]
    assert lgo.matmul_t(At, B, trans_a=True).tolist() == [[6, 8], [8, 10]]
    # A stored M x K = [[1,2,3]], B stored N x K = [[4,5,6],[7,8,9]] : C = [[32, 50]]
    assert lgo.matmul_t(np.array([[1, 2, 3]], np.float32), np.array([[4, 5, 6], [7, 8, 9]], np.float32),
                        trans_b=True).tolist() == [[32, 50]]
    # Section 4.6.1: the transposed variants are the plain product after a transpose -> bit-exact
    M, N, K = 13, 9, 21
    A, B = si.matmul_inputs(25, M, N, K)
    ref = lgo.matmul(A, B)
    assert np.array_equal(bits(lgo.matmul_t(lgo.transpose(A), B, trans_a=True)), bits(ref))
    assert np.array_equal(bits(lgo.matmul_t(A, lgo.transpose(B), trans_b=True)), bits(ref))
    assert np.array_equal(bits(lgo.matmul_t(A, B)), bits(ref))
    assert_half_ulp(lgo.matmul_t(lgo.transpose(A), B, trans_a=True), A.astype(np.float64) @ B.astype(np.float64))
    # accumulate and leading dimensions
    C0 = si.uniform(25, 9, (M, N), -1, 1)
    C = C0.copy()
    lgo.matmul_t(A, lgo.transpose(B), trans_b=True, C=C, accumulate=True)
    assert_half_ulp(C, A.astype(np.float64) @ B.astype(np.float64) + C0)
    Atp = np.full((K, M + 3), np.nan, np.float32); Atp[:, :M] = A.T
    Cp = np.full((M, N + 1), 7.0, np.float32)
    rc = lgo.lib().lgo_matmul_t(lgo._p(Atp), lgo._p(B), lgo._p(Cp), M, N, K, M + 3, N, N + 1, 1, 0, 0)
    assert rc == 0 and np.array_equal(bits(Cp[:, :N]), bits(ref)) and np.all(Cp[:, N:] == 7.0)
    assert lgo.lib().lgo_matmul_t(lgo._p(Atp), lgo._p(B), lgo._p(Cp), M, N, K, M - 1, N, N + 1, 1, 0, 0) == -1
    assert lgo.lib().lgo_matmul_t(lgo._p(Atp), lgo._p(B), lgo._p(Cp), M, N, K, M + 3, N, N + 1, 1, 1, 0) == -1


# --------------------------------------------------------------------------- conv2d

def test_conv_out_extent_closed_forms(lgo):
    assert lgo.conv_out_extent(58, 3, 1, 1) == 56
    assert lgo.conv_out_extent(16, 3, 1, 1) == 14
    assert lgo.conv_out_extent(56, 1, 2, 1) == 28
    assert lgo.conv_out_extent(4098, 3, 1, 1) == 4096
    assert lgo.conv_out_extent(114, 3, 1, 1) == 112
    assert lgo.conv_out_extent(10, 3, 2, 2) == 3      # taps at 0,2,4 ; starts 0,2,4 ; 4+4=8<=9
    assert lgo.conv_out_extent(5, 3, 1, 2) == 1       # taps 0,2,4 only fit once
    assert lgo.conv_out_extent(4, 3, 1, 2) == 0       # dilated window of 5 does not fit
    # brute force: largest extent with every access in bounds
    for n_in in range(1, 20):
        for k in range(1, 5):
            for s in range(1, 4):
                for d in range(1, 4):
                    cnt = 0
                    while cnt * s + (k - 1) * d <= n_in - 1:
                        cnt += 1
                    assert lgo.conv_out_extent(n_in, k, s, d) == cnt


def test_conv2d_hand_literal(lgo):
    I = np.arange(1, 10, dtype=np.float32).reshape(1, 3, 3, 1)       # 1..9
    Kf = np.array([[1, 2], [3, 4]], np.float32).reshape(2, 2, 1, 1)
    # no kernel flip (cross-correlation): O[0,0] = 1*1+2*2+4*3+5*4 = 37
    assert lgo.conv2d_nhwc_hwcf(I, Kf).reshape(2, 2).tolist() == [[37, 47], [67, 77]]
    # two channels, two filters: K[0,0,c,f] = [[1,10],[100,1000]] on a 1x1 window
    I = np.array([[2, 3], [5, 7]], np.float32).reshape(1, 1, 2, 2)   # pixels (2,3),(5,7)
    Kf = np.array([[1, 10], [100, 1000]], np.float32).reshape(1, 1, 2, 2)
    assert lgo.conv2d_nhwc_hwcf(I, Kf).reshape(2, 2).tolist() == [[302, 3020], [705, 7050]]


CONV_CASES = [
    # N, H, W, C, F, KH, KW, (SH,SW), (DH,DW)
    (2, 7, 9, 3, 5, 3, 2, (1, 1), (1, 1)),
    (1, 11, 8, 4, 2, 2, 3, (2, 1), (1, 2)),
    (3, 9, 13, 2, 3, 3, 3, (1, 3), (2, 1)),
    (1, 6, 6, 5, 4, 1, 1, (2, 2), (1, 1)),
    (2, 1, 12, 3, 4, 1, 4, (1, 2), (1, 3)),
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv2d_equals_im2col_matmul_bit_exact(lgo, case):
    N, H, W, C, F, KH, KW, st, dl = case
    I, Kf = si.conv2d_inputs(31, N, H, W, C, F, KH, KW)
    O = lgo.conv2d_nhwc_hwcf(I, Kf, stride=st, dilation=dl)
    col = lgo.im2col_nhwc(I, KH, KW, st, dl)
    O2 = lgo.matmul(col, Kf.reshape(KH * KW * C, F))
    assert np.array_equal(bits(O.reshape(-1, F)), bits(O2))


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv2d_vs_numpy_sliding_window_fp64(lgo, case):
    N, H, W, C, F, KH, KW, (SH, SW), (DH, DW) = case
    I, Kf = si.conv2d_inputs(32, N, H, W, C, F, KH, KW)
    O = lgo.conv2d_nhwc_hwcf(I, Kf, stride=(SH, SW), dilation=(DH, DW))
    Id = I.astype(np.float64)
    # windows[n, y, x, c, a, b] = I[n, y+a, x+b, c] for the dilated span, then subsample
    span_h, span_w = DH * (KH - 1) + 1, DW * (KW - 1) + 1
    win = np.lib.stride_tricks.sliding_window_view(Id, (span_h, span_w), axis=(1, 2))
    win = win[:, ::SH, ::SW, :, ::DH, ::DW]
    ref = np.einsum("nyxcab,abcf->nyxf", win, Kf.astype(np.float64))
    assert O.shape == ref.shape
    assert_half_ulp(O, ref)


def test_conv2d_vs_scipy_correlate2d(lgo):
    H, W, KH, KW = 12, 17, 3, 5
    I = si.uniform(33, 0, (1, H, W, 1), -1, 1)
    Kf = si.uniform(33, 1, (KH, KW, 1, 1), -1, 1)
    ref = signal.correlate2d(I[0, :, :, 0].astype(np.float64), Kf[:, :, 0, 0].astype(np.float64), "valid")
    assert_half_ulp(lgo.conv2d_nhwc_hwcf(I, Kf)[0, :, :, 0], ref)
    # stride = subsampling of the stride-1 result
    O = lgo.conv2d_nhwc_hwcf(I, Kf, stride=(2, 3))
    assert_half_ulp(O[0, :, :, 0], ref[::2, ::3])
    # dilation = correlation with a zero-stuffed filter
    Kz = np.zeros((2 * (KH - 1) + 1, 3 * (KW - 1) + 1))
    Kz[::2, ::3] = Kf[:, :, 0, 0]
    refd = signal.correlate2d(I[0, :, :, 0].astype(np.float64), Kz, "valid")
    assert_half_ulp(lgo.conv2d_nhwc_hwcf(I, Kf, dilation=(2, 3))[0, :, :, 0], refd)


def test_conv2d_1x1_is_matmul_bit_exact(lgo):
    N, H, W, C, F = 2, 5, 7, 6, 9
    I, Kf = si.conv2d_inputs(34, N, H, W, C, F, 1, 1)
    O = lgo.conv2d_nhwc_hwcf(I, Kf)
    assert np.array_equal(bits(O.reshape(-1, F)), bits(lgo.matmul(I.reshape(-1, C), Kf.reshape(C, F))))


def test_conv2d_delta_filter_is_shifted_crop(lgo):
    N, H, W, C = 2, 9, 10, 4
    I = si.uniform(35, 0, (N, H, W, C), -1, 1)
    KH, KW, kh0, kw0 = 3, 4, 2, 1
    Kf = np.zeros((KH, KW, C, C), np.float32)
    Kf[kh0, kw0] = np.eye(C, dtype=np.float32)
    SH, SW, DH, DW = 2, 1, 1, 2
    O = lgo.conv2d_nhwc_hwcf(I, Kf, stride=(SH, SW), dilation=(DH, DW))
    OH, OW = O.shape[1:3]
    crop = I[:, kh0 * DH: kh0 * DH + (OH - 1) * SH + 1: SH, kw0 * DW: kw0 * DW + (OW - 1) * SW + 1: SW, :]
    assert np.array_equal(bits(O), bits(crop))


def test_conv2d_h1_reduces_to_conv1d(lgo):
    # Section 4.6.2: tiling H and K_h by 1 turns the 2-D op into the 1-D op
    # O[n,w,f] = sum I[n, w*S + kw*D, c] K[kw,c,f]; compare with a NumPy 1-D evaluation.
    N, W, C, F, KW, S, D = 2, 15, 3, 4, 3, 2, 2
    I = si.uniform(36, 0, (N, 1, W, C), -1, 1)
    Kf = si.uniform(36, 1, (1, KW, C, F), -1, 1)
    O = lgo.conv2d_nhwc_hwcf(I, Kf, stride=(1, S), dilation=(1, D))
    OW = O.shape[2]
    ref = np.zeros((N, OW, F))
    for w in range(OW):
        for kw in range(KW):
            ref[:, w, :] += I[:, 0, w * S + kw * D, :].astype(np.float64) @ Kf[0, kw].astype(np.float64)
    assert_half_ulp(O[:, 0], ref)


def test_conv2d_accumulate_and_errors(lgo):
    N, H, W, C, F, KH, KW = 1, 5, 6, 2, 3, 2, 2
    I, Kf = si.conv2d_inputs(37, N, H, W, C, F, KH, KW)
    O0 = si.uniform(37, 9, (N, H - 1, W - 1, F), -1, 1)
    O = O0.copy()
    lgo.conv2d_nhwc_hwcf(I, Kf, O, accumulate=True)
    col = lgo.im2col_nhwc(I, KH, KW).astype(np.float64)
    assert_half_ulp(O.reshape(-1, F), col @ Kf.reshape(-1, F).astype(np.float64) + O0.reshape(-1, F))
    with pytest.raises(ValueError):
        lgo.conv2d_nhwc_hwcf(np.zeros((1, 2, 2, 1), np.float32), np.zeros((3, 3, 1, 1), np.float32))


# --------------------------------------------------------------------------- conv1d

def test_conv1d_hand_literal(lgo):
    # one channel, one filter, no flip: [1,2,3,4,5] with taps [1,10,100]
    I = np.arange(1, 6, dtype=np.float32).reshape(1, 5, 1)
    Kf = np.array([1, 10, 100], np.float32).reshape(3, 1, 1)
    assert lgo.conv1d_nwc_wcf(I, Kf).ravel().tolist() == [321, 432, 543]
    assert lgo.conv1d_nwc_wcf(I, Kf, stride=2).ravel().tolist() == [321, 543]
    assert lgo.conv1d_nwc_wcf(I, Kf, dilation=2).ravel().tolist() == [531]
    # two channels -> two filters at one tap: K[0,c,f] = [[1,10],[100,1000]]
    I = np.array([[2, 3], [5, 7]], np.float32).reshape(1, 2, 2)
    Kf = np.array([[1, 10], [100, 1000]], np.float32).reshape(1, 2, 2)
    assert lgo.conv1d_nwc_wcf(I, Kf).reshape(2, 2).tolist() == [[302, 3020], [705, 7050]]


@pytest.mark.parametrize("S,D", [(1, 1), (2, 1), (1, 2), (2, 2), (3, 2)])
def test_conv1d_vs_numpy_fp64_and_conv2d(lgo, S, D):
    # the paper's sweep point (N, C, F, K_w) = (1, 32, 64, 3) at a ragged width, plus a batch
    for N, W, C, F, KW in [(1, 55, 32, 64, 3), (3, 23, 5, 7, 4)]:
        I = si.uniform(38, 0, (N, W, C), -1, 1)
        Kf = si.uniform(38, 1, (KW, C, F), -1, 1)
        O = lgo.conv1d_nwc_wcf(I, Kf, stride=S, dilation=D)
        span = D * (KW - 1) + 1
        win = np.lib.stride_tricks.sliding_window_view(I.astype(np.float64), span, axis=1)[:, ::S, :, ::D]
        ref = np.einsum("nwck,kcf->nwf", win, Kf.astype(np.float64))
        assert O.shape == ref.shape
        assert_half_ulp(O, ref)
        # Section 4.6.2: the 2-D op with H = K_h = 1 is this op (same summation order: bit-exact)
        O2 = lgo.conv2d_nhwc_hwcf(I[:, None], Kf[None], stride=(1, S), dilation=(1, D))
        assert np.array_equal(bits(O), bits(O2[:, 0]))


def test_conv1d_scipy_accumulate_and_errors(lgo):
    W, KW = 40, 5
    I = si.uniform(39, 0, (1, W, 1), -1, 1)
    Kf = si.uniform(39, 1, (KW, 1, 1), -1, 1)
    ref = signal.correlate(I[0, :, 0].astype(np.float64), Kf[:, 0, 0].astype(np.float64), "valid")
    assert_half_ulp(lgo.conv1d_nwc_wcf(I, Kf)[0, :, 0], ref)
    O0 = si.uniform(39, 9, (1, W - KW + 1, 1), -1, 1)
    O = O0.copy()
    lgo.conv1d_nwc_wcf(I, Kf, O, accumulate=True)
    assert_half_ulp(O[0, :, 0], ref + O0[0, :, 0])
    with pytest.raises(ValueError):
        lgo.conv1d_nwc_wcf(np.zeros((1, 4, 1), np.float32), np.zeros((3, 1, 1), np.float32), dilation=2)


# --------------------------------------------------------------------------- depthwise

def test_dwconv1d_hand_literal(lgo):
    I = np.array([[1, 10], [2, 20], [3, 30], [4, 40]], np.float32).reshape(1, 4, 2)
    Kf = np.array([[1, -1], [2, 0], [3, 1]], np.float32)       # K[kw, c]
    # c=0: 1*1+2*2+3*3=14, 2+6+12=20 ; c=1: -10+0+30=20, -20+0+40=20
    assert lgo.dwconv1d_nwc_wc(I, Kf).reshape(2, 2).tolist() == [[14, 20], [20, 20]]


@pytest.mark.parametrize("S,D", [(1, 1), (2, 1), (1, 2), (3, 2)])
def test_dwconv1d_vs_scipy_per_channel(lgo, S, D):
    N, W, C, KW = 2, 23, 5, 3
    I, Kf = si.dwconv1d_inputs(41, N, W, C, KW)
    O = lgo.dwconv1d_nwc_wc(I, Kf, stride=S, dilation=D)
    for n in range(N):
        for c in range(C):
            kz = np.zeros(D * (KW - 1) + 1)
            kz[::D] = Kf[:, c]
            ref = signal.correlate(I[n, :, c].astype(np.float64), kz, "valid")[::S]
            assert_half_ulp(O[n, :, c], ref)


def test_dwconv_equals_conv2d_with_diagonal_filter_bit_exact(lgo):
    N, H, W, C, KH, KW = 2, 8, 9, 5, 3, 2
    I, Kf = si.dwconv2d_inputs(42, N, H, W, C, KH, KW)
    Kfull = np.zeros((KH, KW, C, C), np.float32)
    for c in range(C):
        Kfull[:, :, c, c] = Kf[:, :, c]
    for st, dl in [((1, 1), (1, 1)), ((2, 1), (1, 2)), ((1, 2), (2, 1))]:
        O = lgo.dwconv2d_nhwc_hwc(I, Kf, stride=st, dilation=dl)
        assert np.array_equal(bits(O), bits(lgo.conv2d_nhwc_hwcf(I, Kfull, stride=st, dilation=dl)))
    # 1-D: same identity through H = KH = 1
    I1, K1 = si.dwconv1d_inputs(43, 3, 17, 4, 3)
    K1full = np.zeros((1, 3, 4, 4), np.float32)
    for c in range(4):
        K1full[0, :, c, c] = K1[:, c]
    O1 = lgo.dwconv1d_nwc_wc(I1, K1, stride=2, dilation=3)
    O2 = lgo.conv2d_nhwc_hwcf(I1.reshape(3, 1, 17, 4), K1full, stride=(1, 2), dilation=(1, 3))
    assert np.array_equal(bits(O1), bits(O2[:, 0]))


def test_dwconv2d_h1_equals_dwconv1d_and_scipy(lgo):
    N, W, C, KW = 2, 19, 6, 4
    I, Kf = si.dwconv1d_inputs(44, N, W, C, KW)
    O1 = lgo.dwconv1d_nwc_wc(I, Kf, stride=2, dilation=2)
    O2 = lgo.dwconv2d_nhwc_hwc(I.reshape(N, 1, W, C), Kf.reshape(1, KW, C), stride=(1, 2), dilation=(1, 2))
    assert np.array_equal(bits(O1), bits(O2[:, 0]))
    I2, K2 = si.dwconv2d_inputs(45, 1, 10, 12, 3, 3, 2)
    O = lgo.dwconv2d_nhwc_hwc(I2, K2, stride=(2, 1))
    for c in range(3):
        ref = signal.correlate2d(I2[0, :, :, c].astype(np.float64), K2[:, :, c].astype(np.float64), "valid")
        assert_half_ulp(O[0, :, :, c], ref[::2, :])


def test_dwconv_delta_and_accumulate(lgo):
    N, H, W, C = 1, 7, 8, 3
    I = si.uniform(46, 0, (N, H, W, C), -1, 1)
    Kf = np.zeros((3, 3, C), np.float32)
    Kf[1, 2, :] = 1
    O = lgo.dwconv2d_nhwc_hwc(I, Kf)
    assert np.array_equal(bits(O), bits(I[:, 1:1 + H - 2, 2:2 + W - 2, :]))
    O0 = si.uniform(46, 1, O.shape, -1, 1)
    Oa = O0.copy()
    lgo.dwconv2d_nhwc_hwc(I, Kf, Oa, accumulate=True)
    assert_half_ulp(Oa, O.astype(np.float64) + O0)
    I1 = si.uniform(46, 2, (2, 9, 4), -1, 1)
    K1 = np.zeros((3, 4), np.float32); K1[0] = 1
    O1 = lgo.dwconv1d_nwc_wc(I1, K1)
    assert np.array_equal(bits(O1), bits(I1[:, :7]))
    O1a = np.ones_like(O1)
    lgo.dwconv1d_nwc_wc(I1, K1, O1a, accumulate=True)
    assert_half_ulp(O1a, O1.astype(np.float64) + 1)


# --------------------------------------------------------------------------- reductions

def test_reduce_output_extents_paper_example(lgo):
    for R, Cn, rows_len, cols_len in golden("reduce_output_extent"):
        x = np.ones((R, Cn), np.float32)
        r, c = lgo.reduce_rows(x), lgo.reduce_cols(x)
        assert r.shape == (rows_len,) and c.shape == (cols_len,)
        assert np.all(r == Cn) and np.all(c == R)       # all-ones reduces to the extent


def test_reduce_all_ones_at_config_extents(lgo):
    x = np.ones((3, 16384), np.float32)
    assert np.all(lgo.reduce_rows(x) == 16384)
    x = np.ones((4096, 5), np.float32)
    assert np.all(lgo.reduce_cols(x) == 4096)


def test_reduce_closed_forms(lgo):
    R, Cn = 13, 29
    x = np.repeat(np.arange(Cn, dtype=np.float32)[None, :], R, 0)   # in[i,j] = j
    assert np.all(lgo.reduce_rows(x) == Cn * (Cn - 1) // 2)
    assert np.array_equal(lgo.reduce_cols(x), (R * np.arange(Cn)).astype(np.float32))
    y = np.repeat(np.arange(R, dtype=np.float32)[:, None], Cn, 1)   # in[i,j] = i
    assert np.array_equal(lgo.reduce_rows(y), (Cn * np.arange(R)).astype(np.float32))
    assert np.all(lgo.reduce_cols(y) == R * (R - 1) // 2)


def test_reduce_vs_exactly_rounded_sum(lgo):
    x = si.uniform(51, 0, (7, 3001), 0, 1)
    r = lgo.reduce_rows(x)
    c = lgo.reduce_cols(x)
    for i in range(7):
        assert_half_ulp(r[i], math.fsum(float(v) for v in x[i]))
    for j in range(0, 3001, 97):
        assert_half_ulp(c[j], math.fsum(float(v) for v in x[:, j]))


def test_reduce_identities_between_ops(lgo):
    x = si.uniform(52, 0, (41, 67), 0, 1)
    # Section 4.5.1: a row reduction is a transpose followed by a column reduction
    assert np.array_equal(bits(lgo.reduce_cols(x)), bits(lgo.reduce_rows(lgo.transpose(x))))
    assert np.array_equal(bits(lgo.reduce_rows(x)), bits(lgo.reduce_cols(lgo.transpose(x))))
    # a row reduction is a matrix-vector product with ones
    assert np.array_equal(bits(lgo.reduce_rows(x)), bits(lgo.matmul(x, np.ones((67, 1), np.float32))[:, 0]))
    assert np.array_equal(bits(lgo.reduce_cols(x)), bits(lgo.matmul(np.ones((1, 41), np.float32), x)[0]))


def test_reduce_ld_accumulate_and_empty(lgo):
    x = si.uniform(53, 0, (6, 10), 0, 1)
    xp = np.full((6, 13), np.nan, np.float32); xp[:, :10] = x
    out = np.empty(6, np.float32)
    assert lgo.lib().lgo_reduce_rows(lgo._p(xp), lgo._p(out), 6, 10, 13, 0) == 0
    assert np.array_equal(bits(out), bits(lgo.reduce_rows(x)))
    outc = np.empty(10, np.float32)
    assert lgo.lib().lgo_reduce_cols(lgo._p(xp), lgo._p(outc), 6, 10, 13, 0) == 0
    assert np.array_equal(bits(outc), bits(lgo.reduce_cols(x)))
    acc = np.full(6, 2.0, np.float32)
    lgo.reduce_rows(x, acc, accumulate=True)
    assert_half_ulp(acc, x.astype(np.float64).sum(1) + 2.0)
    acc = np.full(10, -1.0, np.float32)
    lgo.reduce_cols(x, acc, accumulate=True)
    assert_half_ulp(acc, x.astype(np.float64).sum(0) - 1.0)
    # empty reduction extent gives the neutral element
    assert np.all(lgo.reduce_rows(np.empty((4, 0), np.float32)) == 0)
    assert np.all(lgo.reduce_cols(np.empty((0, 4), np.float32)) == 0)
    assert lgo.lib().lgo_reduce_rows(lgo._p(xp), lgo._p(out), 6, 10, 9, 0) == -1


# --------------------------------------------------------------------------- transpose / copy

def special_bits(shape, seed):
    """uint32 patterns incl. -0.0, infinities, denormals and NaNs with payloads."""
    n = int(np.prod(shape))
    b = (si.bits24(seed, 0, n).astype(np.uint32) << np.uint32(8)) | si.bits24(seed, 1, n).astype(np.uint32) & np.uint32(0xFF)
    specials = np.array([0x80000000, 0x7F800000, 0xFF800000, 0x7FC00001, 0xFFC12345, 0x7F800001,
                         0x00000001, 0x807FFFFF, 0x00800000], np.uint32)
    k = min(len(specials), len(b[::2]))
    b[::2][:k] = specials[:k]
    return b.reshape(shape)


def test_transpose_hand_literal_and_numpy(lgo):
    x = np.array([[1, 2, 3], [4, 5, 6]], np.float32)
    assert lgo.transpose(x).tolist() == [[1, 4], [2, 5], [3, 6]]
    xb = special_bits((37, 53), 61)
    x = xb.view(np.float32)
    t = lgo.transpose(x)
    assert t.shape == (53, 37)
    assert np.array_equal(bits(t), xb.T)                        # bit patterns survive, NaN payloads too
    assert np.array_equal(bits(lgo.transpose(t)), xb)           # involution
    v = special_bits((1, 19), 62).view(np.float32)
    assert np.array_equal(bits(lgo.transpose(v)).ravel(), bits(v).ravel())
    s = si.uniform(63, 0, (9, 9), 0, 1)
    s = (s + s.T).astype(np.float32)
    assert np.array_equal(bits(lgo.transpose(s)), bits(s))      # symmetric matrix is a fixed point


def test_transpose_and_copy_leading_dims(lgo):
    xb = special_bits((5, 8), 64)
    xp = np.zeros((5, 11), np.uint32); xp[:, :8] = xb
    out = np.full((8, 9), 0xDEADBEEF, np.uint32)
    rc = lgo.lib().lgo_transpose(lgo._p(xp.view(np.float32)), lgo._p(out.view(np.float32)), 5, 8, 11, 9)
    assert rc == 0 and np.array_equal(out[:, :5], xb.T) and np.all(out[:, 5:] == 0xDEADBEEF)
    out = np.full((5, 10), 0xDEADBEEF, np.uint32)
    rc = lgo.lib().lgo_copy2d(lgo._p(xp.view(np.float32)), lgo._p(out.view(np.float32)), 5, 8, 11, 10)
    assert rc == 0 and np.array_equal(out[:, :8], xb) and np.all(out[:, 8:] == 0xDEADBEEF)
    assert np.array_equal(bits(lgo.copy2d(xb.view(np.float32))), xb)
    assert lgo.lib().lgo_transpose(lgo._p(xp.view(np.float32)), lgo._p(out.view(np.float32)), 5, 8, 11, 4) == -1


def test_transpose_batched_paper_4d_example(lgo):
    # Section 4.4: [i,j,k,l] -> [k,j,l,i] as j x k transposes of (i, l) matrices
    Ni, Nj, Nk, Nl = 5, 3, 4, 7
    xb = special_bits((Ni, Nj, Nk, Nl), 65)
    out = np.full(Nk * Nj * Nl * Ni, 0xDEADBEEF, np.uint32)
    lgo.transpose_batched(xb.view(np.float32).ravel(), out.view(np.float32),
                          Ni, Nl, Nj * Nk * Nl, Ni, Nj, Nk, Nk * Nl, Nl, Nl * Ni, Nj * Nl * Ni)
    assert np.array_equal(out.reshape(Nk, Nj, Nl, Ni), np.transpose(xb, (2, 1, 3, 0)))
    # hand literal: two 2x2 matrices stored back to back
    x = np.array([1, 2, 3, 4, 5, 6, 7, 8], np.float32)
    o = np.zeros(8, np.float32)
    lgo.transpose_batched(x, o, 2, 2, 2, 2, 1, 2, 0, 4, 0, 4)
    assert o.tolist() == [1, 3, 2, 4, 5, 7, 6, 8]
    # a batch of one equals the plain transpose; [b,i,j] -> [j,b,i] through the outer batch index
    x2 = special_bits((6, 9), 66)
    o2 = np.zeros(54, np.uint32)
    lgo.transpose_batched(x2.view(np.float32).ravel(), o2.view(np.float32), 6, 9, 9, 6, 1, 1, 0, 0, 0, 0)
    assert np.array_equal(o2.reshape(9, 6), x2.T)
    x3 = special_bits((4, 3, 5), 67)
    o3 = np.zeros(60, np.uint32)
    lgo.transpose_batched(x3.view(np.float32).ravel(), o3.view(np.float32), 3, 5, 5, 12, 4, 1, 15, 0, 3, 0)
    assert np.array_equal(o3.reshape(5, 4, 3), np.transpose(x3, (2, 0, 1)))
    assert lgo.lib().lgo_transpose_batched(lgo._p(x), lgo._p(o), 2, 2, 1, 2, 1, 2, 0, 4, 0, 4) == -1


# --------------------------------------------------------------------------- inputs

def test_seeded_inputs_are_reproducible_and_in_range():
    a = si.uniform(1, 0, (1000, 33), 0, 1)
    assert a.dtype == np.float32 and a.min() >= 0 and a.max() < 1
    assert abs(float(a.mean()) - 0.5) < 0.01
    b = si.uniform(2, 0, (4097,), -1, 1)
    assert b.min() >= -1 and b.max() < 1 and abs(float(b.mean())) < 0.05
    assert np.array_equal(si.uniform(1, 0, (1000, 33), 0, 1), a)
    assert not np.array_equal(si.uniform(1, 1, (1000, 33), 0, 1), a)
    # chunk-independent: a sub-range equals the slice of the full stream
    assert np.array_equal(si.bits24(3, 2, 100, start=50), si.bits24(3, 2, 150)[50:])
