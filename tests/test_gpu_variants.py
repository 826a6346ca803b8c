"""GPU parity of every GEMM kernel variant on shapes the planner would never give it: each of the
eight LDS tiles (with and without a k-split), each register-direct variant and each tile-loop variant
runs ragged, tiny and unaligned matmuls in the three layouts and convolutions with aligned and odd
channel counts, against the CPU oracle on the same seeded inputs, between canary guard bands; the
tile-loop variants also run shapes with several output blocks per workgroup."""
import numpy as np
import pytest
import torch

import seeded_inputs as si
from gpu_util import Guarded, assert_close, dev, workspace

pytestmark = pytest.mark.gpu

N_VARIANTS = 20            # checked against the library in test_variant_menu


@pytest.fixture(scope="module")
def lg():
    import paper_2202_03293_amd as pkg
    pkg.lib()
    return pkg


def test_variant_menu(lg):
    assert lg.lg_gemm_variants() == N_VARIANTS
    infos = [lg.lg_gemm_variant_info(v) for v in range(N_VARIANTS)]
    assert len(set(infos)) == N_VARIANTS                     # all different
    assert sum(1 for bm, bn, bk, kp, loop in infos if bm == 16) == 9
    assert sum(1 for bm, bn, bk, kp, loop in infos if loop) == 3
    with pytest.raises(lg.LgError):
        lg.lg_gemm_variant_info(N_VARIANTS)
    a = torch.zeros((4, 4), device="cuda")
    with pytest.raises(lg.LgError):
        lg.lg_matmul_variant(a, a.clone(), torch.empty((4, 4), device="cuda"), N_VARIANTS)
    for v in range(N_VARIANTS):                              # register-direct and tile-loop variants take no k-split
        if infos[v][0] == 16 or infos[v][4]:
            with pytest.raises(lg.LgError):
                lg.lg_matmul_variant(a, a.clone(), torch.empty((4, 4), device="cuda"), v, k_splits=2)


# (M, N, K, layout, accumulate, padded leading dimensions)
MATMUL_SHAPES = [
    (1, 1, 1, "nn", False, False),
    (17, 33, 5, "nn", True, False),
    (100, 70, 130, "nn", False, True),
    (64, 64, 288, "nn", False, False),
    (131, 257, 67, "tn", False, False),
    (96, 48, 200, "tn", True, True),
    (75, 130, 150, "nt", False, False),
    (128, 32, 272, "nt", True, True),
    (300, 20, 27, "nn", False, False),
]


@pytest.mark.parametrize("variant", range(N_VARIANTS))
@pytest.mark.parametrize("M,N,K,layout,accumulate,padded", MATMUL_SHAPES)
def test_matmul_every_variant(lg, lgo, variant, M, N, K, layout, accumulate, padded):
    info = lg.lg_gemm_variant_info(variant)
    direct = info[0] == 16 or info[4] == 1                   # no k-split
    A, B = si.matmul_inputs(1200 + M, M, N, K, case=K % 7)
    C0 = si.uniform(1201, N, (M, N), -1, 1) if accumulate else None
    ref = lgo.matmul(A, B, C0.copy(), accumulate=True) if accumulate else lgo.matmul(A, B)
    As = np.ascontiguousarray(A.T) if layout == "tn" else A
    Bs = np.ascontiguousarray(B.T) if layout == "nt" else B
    pad = 4 if padded else 0

    def padded_dev(x):
        if not pad:
            return dev(x)
        full = torch.full((x.shape[0], x.shape[1] + pad), float("nan"), device="cuda")
        full[:, :x.shape[1]] = dev(x)
        return full[:, :x.shape[1]]

    Ad, Bd = padded_dev(As), padded_dev(Bs)
    for k_splits in ((1,) if direct else (1, 3)):
        out = Guarded((M, N), init=C0 if accumulate else np.full((M, N), np.nan, np.float32))
        ws = workspace(lg.lg_gemm_variant_workspace_bytes(M, N, K, variant, k_splits))
        lg.lg_matmul_variant(Ad, Bd, out.t, variant, k_splits, trans_a=layout == "tn", trans_b=layout == "nt",
                             accumulate=accumulate, workspace=ws)
        torch.cuda.synchronize()
        out.check()
        assert_close(out.host(), ref, K, f"variant {variant} splits {k_splits} {layout} {(M, N, K)}")


# (N, H, W, C, F, KH, KW, stride, dilation, accumulate)
CONV_SHAPES = [
    (2, 12, 13, 3, 20, 3, 3, (1, 1), (1, 1), False),      # three channels: every quad straddles taps
    (1, 16, 16, 32, 64, 3, 3, (1, 1), (1, 1), False),     # the paper's batch-1 sweep shape
    (3, 11, 17, 20, 33, 2, 3, (2, 1), (1, 2), True),      # C % 4 == 0, C % 16 != 0, odd F
    (2, 9, 9, 7, 5, 5, 4, (1, 2), (1, 1), False),
    (1, 20, 20, 16, 16, 1, 1, (1, 1), (1, 1), True),      # 1x1, stride 1: runs as a plain matmul
    (2, 15, 15, 8, 24, 1, 1, (2, 2), (1, 1), False),      # 1x1, strided
    # contractions past 512: the register-direct kernel walks the taps per lane instead of reading
    # the host's table of tap offsets
    (1, 9, 10, 64, 16, 3, 3, (1, 1), (1, 1), False),      # K = 576, aligned
    (2, 8, 8, 63, 9, 3, 3, (1, 1), (1, 2), True),         # K = 567, nothing aligned
]


@pytest.mark.parametrize("variant", range(N_VARIANTS))
@pytest.mark.parametrize("N,H,W,C,F,KH,KW,st,dl,accumulate", CONV_SHAPES)
def test_conv2d_every_variant(lg, lgo, variant, N, H, W, C, F, KH, KW, st, dl, accumulate):
    info = lg.lg_gemm_variant_info(variant)
    direct = info[0] == 16 or info[4] == 1                   # no k-split
    I, Kf = si.conv2d_inputs(1210 + C, N, H, W, C, F, KH, KW)
    OH, OW = lg.lg_conv_out_extent(H, KH, st[0], dl[0]), lg.lg_conv_out_extent(W, KW, st[1], dl[1])
    O0 = si.uniform(1211, F, (N, OH, OW, F), -1, 1) if accumulate else None
    ref = lgo.conv2d_nhwc_hwcf(I, Kf, O0.copy(), stride=st, dilation=dl, accumulate=True) if accumulate \
        else lgo.conv2d_nhwc_hwcf(I, Kf, stride=st, dilation=dl)
    Id, Kd = dev(I), dev(Kf)
    for k_splits in ((1,) if direct else (1, 2)):
        out = Guarded((N, OH, OW, F), init=O0 if accumulate else np.full((N, OH, OW, F), np.nan, np.float32))
        ws = workspace(lg.lg_gemm_variant_workspace_bytes(N * OH * OW, F, KH * KW * C, variant, k_splits))
        lg.lg_conv2d_nhwc_hwcf_variant(Id, Kd, out.t, variant, k_splits, stride=st, dilation=dl,
                                       accumulate=accumulate, workspace=ws)
        torch.cuda.synchronize()
        out.check()
        assert_close(out.host(), ref, KH * KW * C, f"variant {variant} splits {k_splits} conv {(N, H, W, C, F, KH, KW)}")


# The tile loop proper: the forced variants run a third as many workgroups as there are output blocks, so
# every workgroup walks over about three.  (M, N, K, accumulate, padded leading dimensions)
LOOP_SHAPES = [
    (1024, 512, 64, False, False),     # whole blocks; four slices of 16 (the ring runs on across blocks) or two of 32
    (1024, 512, 128, False, False),
    (1000, 520, 64, False, False),     # ragged edges: predicated epilogues between the counted ones
    (1152, 576, 96, False, True),      # six slices of 16: the next block's first transfers go out after the last step
    (1024, 512, 200, False, False),    # a k tail after the ring
    (1024, 512, 64, True, False),      # accumulating: no epilogue is counted
    (2048, 1024, 16, False, False),    # a single slice
    (896, 640, 256, False, False),
    (520, 1000, 32, False, True),
    (2048, 2048, 64, False, False),    # more blocks than the chip holds workgroups of the larger tiles
]


@pytest.mark.parametrize("layout", ["nn", "tn"])
@pytest.mark.parametrize("M,N,K,accumulate,padded", LOOP_SHAPES)
def test_matmul_tile_loop(lg, lgo, M, N, K, accumulate, padded, layout):
    A, B = si.matmul_inputs(1240 + K, M, N, K, case=K % 7)
    C0 = si.uniform(1241, N, (M, N), -1, 1) if accumulate else None
    ref = lgo.matmul(A, B, C0.copy(), accumulate=True) if accumulate else lgo.matmul(A, B)
    pad = 8 if padded else 0

    def padded_dev(x):
        full = torch.full((x.shape[0], x.shape[1] + pad), float("nan"), device="cuda")
        full[:, :x.shape[1]] = dev(x)
        return full[:, :x.shape[1]]

    Ad, Bd = padded_dev(np.ascontiguousarray(A.T) if layout == "tn" else A), padded_dev(B)
    loops = [v for v in range(N_VARIANTS) if lg.lg_gemm_variant_info(v)[4]]
    assert len(loops) == 3
    for variant in loops:
        for rep in range(2):                                 # twice: the second run finds the caches warm, other timing
            out = Guarded((M, N), init=C0 if accumulate else np.full((M, N), np.nan, np.float32))
            lg.lg_matmul_variant(Ad, Bd, out.t, variant, trans_a=layout == "tn", accumulate=accumulate)
            torch.cuda.synchronize()
            out.check()
            assert_close(out.host(), ref, K, f"tile-loop variant {variant} {layout} {(M, N, K)} run {rep}")


def test_planner_takes_the_tile_loop_for_short_contractions(lg, lgo):
    """4096 x 4096 x 64 through lg_matmul itself (the planner's tile loop on the chip's fill of workgroups),
    every element against the oracle; and the same with a ragged edge."""
    for M, N, K in [(4096, 4096, 64), (4000, 4128, 128)]:
        assert lg.lg_matmul_plan(M, N, K)[:2] in ((128, 128), (128, 64), (64, 128))
        assert lg.lg_matmul_plan_tile_loop(M, N, K)
        A, B = si.matmul_inputs(1250, M, N, K, case=2)
        ref = lgo.matmul(A, B)
        out = Guarded((M, N), init=np.full((M, N), np.nan, np.float32))
        lg.lg_matmul(dev(A), dev(B), out.t)
        torch.cuda.synchronize()
        out.check()
        assert_close(out.host(), ref, K, f"planned tile loop {(M, N, K)}")
        out = Guarded((M, N), init=np.full((M, N), np.nan, np.float32))    # A^T B takes the same plan
        lg.lg_matmul_t(dev(np.ascontiguousarray(A.T)), dev(B), out.t, trans_a=True)
        torch.cuda.synchronize()
        out.check()
        assert_close(out.host(), ref, K, f"planned tile loop, A^T B {(M, N, K)}")


def random_cases():
    import random
    rng = random.Random(1503)
    mm, cv = [], []
    for i in range(14):
        M = rng.choice([1, 15, 16, 17, 63, 64, 100, 250])
        N = rng.choice([1, 4, 15, 16, 31, 64, 65, 128, 200])
        K = rng.choice([1, 4, 15, 16, 17, 48, 64, 100, 513, 700])
        if i % 2 == 0:                                       # the aligned paths
            N, K = 4 * ((N + 3) // 4), 4 * ((K + 3) // 4)
        mm.append((M, N, K, ("nn", "tn", "nt")[i % 3], i % 4 == 1))
    for i in range(10):
        KH, KW = rng.choice([1, 2, 3]), rng.choice([1, 3, 5])
        st = (rng.choice([1, 2]), rng.choice([1, 2, 3]))
        dl = (rng.choice([1, 2]), rng.choice([1, 2]))
        H = dl[0] * (KH - 1) + 1 + rng.randint(0, 9)
        W = dl[1] * (KW - 1) + 1 + rng.randint(0, 12)
        C = rng.choice([1, 3, 4, 8, 20, 36, 64])             # 64 x 3 x 5 = 960: past the tap table
        F = rng.choice([1, 4, 6, 16, 40, 64])
        cv.append((rng.randint(1, 3), H, W, C, F, KH, KW, st, dl, i % 3 == 2))
    return mm, cv


@pytest.mark.parametrize("M,N,K,layout,accumulate", random_cases()[0])
def test_matmul_random_shapes_every_variant(lg, lgo, M, N, K, layout, accumulate):
    A, B = si.matmul_inputs(1220 + M, M, N, K, case=K % 7)
    C0 = si.uniform(1221, N, (M, N), -1, 1) if accumulate else None
    ref = lgo.matmul(A, B, C0.copy(), accumulate=True) if accumulate else lgo.matmul(A, B)
    Ad = dev(np.ascontiguousarray(A.T) if layout == "tn" else A)
    Bd = dev(np.ascontiguousarray(B.T) if layout == "nt" else B)
    for variant in range(N_VARIANTS):
        out = Guarded((M, N), init=C0 if accumulate else np.full((M, N), np.nan, np.float32))
        lg.lg_matmul_variant(Ad, Bd, out.t, variant, trans_a=layout == "tn", trans_b=layout == "nt", accumulate=accumulate)
        torch.cuda.synchronize()
        out.check()
        assert_close(out.host(), ref, K, f"variant {variant} {layout} {(M, N, K)}")


@pytest.mark.parametrize("N,H,W,C,F,KH,KW,st,dl,accumulate", random_cases()[1])
def test_conv2d_random_shapes_every_variant(lg, lgo, N, H, W, C, F, KH, KW, st, dl, accumulate):
    I, Kf = si.conv2d_inputs(1230 + C, N, H, W, C, F, KH, KW)
    OH, OW = lg.lg_conv_out_extent(H, KH, st[0], dl[0]), lg.lg_conv_out_extent(W, KW, st[1], dl[1])
    O0 = si.uniform(1231, F, (N, OH, OW, F), -1, 1) if accumulate else None
    ref = lgo.conv2d_nhwc_hwcf(I, Kf, O0.copy(), stride=st, dilation=dl, accumulate=True) if accumulate \
        else lgo.conv2d_nhwc_hwcf(I, Kf, stride=st, dilation=dl)
    Id, Kd = dev(I), dev(Kf)
    for variant in range(N_VARIANTS):
        out = Guarded((N, OH, OW, F), init=O0 if accumulate else np.full((N, OH, OW, F), np.nan, np.float32))
        lg.lg_conv2d_nhwc_hwcf_variant(Id, Kd, out.t, variant, stride=st, dilation=dl, accumulate=accumulate)
        torch.cuda.synchronize()
        out.check()
        assert_close(out.host(), ref, KH * KW * C, f"variant {variant} conv {(N, H, W, C, F, KH, KW, st, dl)}")


# matrix times one to four vectors: the planner's entry points send these to the weighted
# row-reduction kernel (AB and A B^T); A^T B and shapes below its thresholds take the MFMA kernels
@pytest.mark.parametrize("M,N,K,layout,accumulate,padded", [
    (1024, 1, 1024, "nn", False, False), (2000, 3, 1501, "nn", True, False), (1500, 4, 2048, "nt", False, False),
    (1031, 2, 4096, "nt", True, True), (4096, 1, 1030, "nn", False, True), (1024, 4, 1024, "tn", False, False),
    (1023, 1, 5000, "nn", False, False), (3000, 2, 1000, "nn", False, False)])
def test_matrix_times_few_vectors(lg, lgo, M, N, K, layout, accumulate, padded):
    A, B = si.matmul_inputs(1240 + N, M, N, K, case=K % 7)
    C0 = si.uniform(1241, N, (M, N), -1, 1) if accumulate else None
    ref = lgo.matmul(A, B, C0.copy(), accumulate=True) if accumulate else lgo.matmul(A, B)
    As = np.ascontiguousarray(A.T) if layout == "tn" else A
    Bs = np.ascontiguousarray(B.T) if layout == "nt" else B
    pad = 4 if padded else 0

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
    assert_close(out.host(), ref, K, f"{layout} {(M, N, K)}")
