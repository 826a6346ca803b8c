"""GPU parity on shapes drawn from a fixed-seed generator: extents around the tile sizes (64, 128,
256), k around the slice depths and the split-k granule, ragged tails, odd channel counts, random
strides and dilations, padded leading dimensions.  Same bar as the hand-picked cases: the oracle
on identical seeded inputs, outputs between canary guard bands."""
import random

import numpy as np
import pytest
import torch

import seeded_inputs as si
from gpu_util import Guarded, assert_close, bits, dev, workspace

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lg():
    import paper_2202_03293_amd as pkg
    pkg.lib()
    return pkg


def near(rng, anchors, spread):
    """An extent next to one of the anchors (tile and slice boundaries are where indexing breaks)."""
    return max(1, rng.choice(anchors) + rng.randint(-spread, spread))


def matmul_cases():
    rng = random.Random(20220203)
    cases = []
    for i in range(36):
        M = near(rng, [1, 64, 128, 256, 384, 1000], 9)
        N = near(rng, [1, 64, 128, 256, 512], 9)
        K = near(rng, [1, 16, 32, 64, 128, 640, 2048], 7)
        if i % 3 == 0:                 # the aligned fast path: multiples of 4
            M, N, K = 4 * ((M + 3) // 4), 4 * ((N + 3) // 4), 4 * ((K + 3) // 4)
        cases.append((M, N, K, ("nn", "tn", "nt")[i % 3], i % 4 == 1, i % 5 == 2))
    return cases


@pytest.mark.parametrize("M,N,K,layout,accumulate,padded", matmul_cases())
def test_matmul_random(lg, lgo, M, N, K, layout, accumulate, padded):
    A, B = si.matmul_inputs(900 + M, M, N, K, case=K % 7)
    C0 = si.uniform(901, N, (M, N), -1, 1) if accumulate else None
    ref = C0.copy() if accumulate else None
    ref = lgo.matmul(A, B, ref, accumulate=accumulate) if accumulate else lgo.matmul(A, B)
    As = np.ascontiguousarray(A.T) if layout == "tn" else A          # stored K x M for A^T B
    Bs = np.ascontiguousarray(B.T) if layout == "nt" else B          # stored N x K for A B^T
    pad = 4 if padded else 0                                          # leading dimensions wider than the rows

    def padded_dev(x):
        if not pad:
            return dev(x)
        full = torch.full((x.shape[0], x.shape[1] + pad), float("nan"), device="cuda")
        full[:, :x.shape[1]] = dev(x)
        return full[:, :x.shape[1]]

    out = Guarded((M, N), init=C0 if accumulate else np.full((M, N), np.nan, np.float32))
    ws = workspace(lg.lg_matmul_workspace_bytes(M, N, K))
    lg.lg_matmul_t(padded_dev(As), padded_dev(Bs), out.t, trans_a=layout == "tn", trans_b=layout == "nt",
                   accumulate=accumulate, workspace=ws)
    torch.cuda.synchronize()
    out.check()
    assert_close(out.host(), ref, K, f"matmul {layout} {(M, N, K)} acc={accumulate} pad={pad}")


def conv_cases():
    rng = random.Random(3293)
    cases = []
    for i in range(24):
        KH, KW = rng.choice([1, 2, 3, 5]), rng.choice([1, 2, 3, 4])
        st = (rng.choice([1, 1, 2, 3]), rng.choice([1, 1, 2]))
        dl = (rng.choice([1, 1, 2]), rng.choice([1, 2, 3]))
        H = dl[0] * (KH - 1) + 1 + rng.randint(0, 20)
        W = dl[1] * (KW - 1) + 1 + rng.randint(0, 30)
        C = rng.choice([1, 3, 4, 8, 12, 16, 20, 32, 48, 64])
        F = rng.choice([1, 5, 8, 16, 60, 64, 72, 128])
        cases.append((rng.randint(1, 5), H, W, C, F, KH, KW, st, dl, i % 4 == 3))
    return cases


@pytest.mark.parametrize("N,H,W,C,F,KH,KW,st,dl,accumulate", conv_cases())
def test_conv2d_random(lg, lgo, N, H, W, C, F, KH, KW, st, dl, accumulate):
    I, Kf = si.conv2d_inputs(910 + C, N, H, W, C, F, KH, KW)
    OH, OW = lg.lg_conv_out_extent(H, KH, st[0], dl[0]), lg.lg_conv_out_extent(W, KW, st[1], dl[1])
    O0 = si.uniform(911, F, (N, OH, OW, F), -1, 1) if accumulate else None
    ref = lgo.conv2d_nhwc_hwcf(I, Kf, O0.copy(), stride=st, dilation=dl, accumulate=True) if accumulate \
        else lgo.conv2d_nhwc_hwcf(I, Kf, stride=st, dilation=dl)
    out = Guarded((N, OH, OW, F), init=O0 if accumulate else np.full((N, OH, OW, F), np.nan, np.float32))
    ws = workspace(lg.lg_conv2d_workspace_bytes(N, H, W, C, KH, KW, F, *st, *dl))
    lg.lg_conv2d_nhwc_hwcf(dev(I), dev(Kf), out.t, stride=st, dilation=dl, accumulate=accumulate, workspace=ws)
    torch.cuda.synchronize()
    out.check()
    assert_close(out.host(), ref, KH * KW * C, f"conv {(N, H, W, C, F, KH, KW, st, dl)}")


def dwconv_cases():
    rng = random.Random(47)
    cases = []
    for i in range(20):
        KH, KW = rng.choice([1, 1, 3, 3, 5]), rng.choice([1, 2, 3, 3, 7])
        st = (rng.choice([1, 1, 2]), rng.choice([1, 1, 2, 3]))
        dl = (rng.choice([1, 1, 2]), rng.choice([1, 1, 2]))
        H = dl[0] * (KH - 1) + 1 + rng.randint(0, 24)
        W = dl[1] * (KW - 1) + 1 + rng.randint(0, 40)
        cases.append((rng.randint(1, 4), H, W, rng.choice([1, 4, 6, 8, 24, 32, 96, 100]), KH, KW, st, dl, i % 3 == 2))
    return cases


@pytest.mark.parametrize("N,H,W,C,KH,KW,st,dl,accumulate", dwconv_cases())
def test_dwconv2d_random(lg, lgo, N, H, W, C, KH, KW, st, dl, accumulate):
    I, Kf = si.dwconv2d_inputs(920 + C, N, H, W, C, KH, KW)
    OH, OW = lg.lg_conv_out_extent(H, KH, st[0], dl[0]), lg.lg_conv_out_extent(W, KW, st[1], dl[1])
    O0 = si.uniform(921, C, (N, OH, OW, C), -1, 1) if accumulate else None
    ref = lgo.dwconv2d_nhwc_hwc(I, Kf, O0.copy(), stride=st, dilation=dl, accumulate=True) if accumulate \
        else lgo.dwconv2d_nhwc_hwc(I, Kf, stride=st, dilation=dl)
    out = Guarded((N, OH, OW, C), init=O0 if accumulate else np.full((N, OH, OW, C), np.nan, np.float32))
    lg.lg_dwconv2d_nhwc_hwc(dev(I), dev(Kf), out.t, stride=st, dilation=dl, accumulate=accumulate)
    torch.cuda.synchronize()
    out.check()
    assert_close(out.host(), ref, KH * KW, f"dwconv {(N, H, W, C, KH, KW, st, dl)}")


def plane_cases():
    rng = random.Random(8192)
    return [(near(rng, [1, 4, 64, 128, 256, 600, 2100], 5), near(rng, [1, 4, 64, 128, 256, 1024, 4100], 5))
            for _ in range(24)]


@pytest.mark.parametrize("R,Cn", plane_cases())
def test_reduce_and_move_random(lg, lgo, R, Cn):
    x = si.uniform(930 + R, Cn % 11, (R, Cn), 0, 1)
    xd = dev(x)
    rows, cols = Guarded((R,)), Guarded((Cn,))
    lg.lg_reduce_rows(xd, rows.t)
    lg.lg_reduce_cols(xd, cols.t, workspace=workspace(lg.lg_reduce_cols_workspace_bytes(R, Cn)))
    tr, cp = Guarded((Cn, R)), Guarded((R, Cn))
    lg.lg_transpose(xd, tr.t)
    lg.lg_copy2d(xd, cp.t)
    torch.cuda.synchronize()
    for g in (rows, cols, tr, cp):
        g.check()
    assert_close(rows.host(), lgo.reduce_rows(x), Cn, f"reduce_rows {(R, Cn)}")
    assert_close(cols.host(), lgo.reduce_cols(x), R, f"reduce_cols {(R, Cn)}")
    assert np.array_equal(bits(tr.host()), bits(lgo.transpose(x)))
    assert np.array_equal(bits(cp.host()), bits(x))
