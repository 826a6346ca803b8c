"""GPU parity: every liblg entry point against the CPU oracle on identical seeded inputs.

fp32 ops: max |err| <= 1e-4*sqrt(K) (K = reduction length of one output element) and relative
Frobenius error <= 1e-5.  Transpose / copy: bit-exact.  All calls go through the C ABI via the
thin ctypes binding; outputs sit between canary guard bands.
"""
import numpy as np
import pytest
import torch

import seeded_inputs as si
from gpu_util import Guarded, assert_close, bits, dev, workspace

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lg():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2202_03293_amd as lg_
    lg_.lib()
    return lg_


def sync():
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------- matmul

def run_matmul(lg, A, B, C0=None, accumulate=False):
    M, K = A.shape
    N = B.shape[1]
    out = Guarded((M, N), init=C0 if C0 is not None else np.full((M, N), np.nan, np.float32))
    ws = workspace(lg.lg_matmul_workspace_bytes(M, N, K))
    lg.lg_matmul(dev(A), dev(B), out.t, accumulate=accumulate, workspace=ws)
    sync()
    out.check()
    return out.host()


MATMUL_SHAPES = [
    (256, 256, 256),        # benchmark config 0
    (1, 1, 1), (3, 5, 7), (64, 64, 16), (65, 63, 17), (100, 36, 52),
    (128, 128, 128), (257, 255, 129), (300, 520, 40), (512, 768, 64),
    (1000, 24, 2000),       # split-k, ragged everywhere
    (2048, 2048, 96), (4100, 4104, 36),   # big tile with ragged edges
    (33, 4096, 8),
    (2048, 2048, 192), (1024, 1024, 320), (1020, 1000, 264), (2048, 1024, 100),   # mid-size tiles, deep slices
    (6272, 512, 256), (16384, 512, 128),
    # whole tiles whose k is not a multiple of the slice depth: transfer ring + one predicated tail slice
    (256, 256, 1000), (512, 384, 2052), (256, 512, 72), (128, 128, 20), (128, 128, 12), (1024, 1024, 1028),
    (4096, 4096, 56), (2048, 1024, 4104),
]


@pytest.mark.parametrize("M,N,K", MATMUL_SHAPES)
def test_matmul_matches_oracle(lg, lgo, M, N, K):
    A, B = si.matmul_inputs(0 if (M, N, K) == (256, 256, 256) else 100 + M % 7, M, N, K)
    C = run_matmul(lg, A, B)
    assert_close(C, lgo.matmul(A, B), K, f"matmul {M}x{N}x{K}")


@pytest.mark.parametrize("M,N,K", [(129, 67, 45), (256, 256, 64), (520, 516, 132)])
def test_matmul_accumulate(lg, lgo, M, N, K):
    A, B = si.matmul_inputs(111, M, N, K)
    C0 = si.uniform(111, 7, (M, N), -1, 1)
    C = run_matmul(lg, A, B, C0=C0, accumulate=True)
    ref = C0.copy()
    lgo.matmul(A, B, ref, accumulate=True)
    assert_close(C, ref, K, "matmul accumulate")


def test_matmul_exact_cases(lg, lgo):
    # integer-valued operands: every product and partial sum is exact in fp32, any order
    A = si.small_integers(112, 0, (200, 96))
    B = si.small_integers(112, 1, (96, 136))
    assert np.array_equal(run_matmul(lg, A, B), lgo.matmul(A, B))
    # identity and permutation: one non-zero term per sum -> bit-exact
    X = si.uniform(113, 0, (192, 192), -1, 1)
    eye = np.eye(192, dtype=np.float32)
    assert np.array_equal(bits(run_matmul(lg, X, eye)), bits(X))
    assert np.array_equal(bits(run_matmul(lg, eye, X)), bits(X))
    perm = np.random.default_rng(3).permutation(192)
    assert np.array_equal(bits(run_matmul(lg, eye[perm], X)), bits(X[perm]))
    # the paper's all-ones example: every entry equals K
    assert np.all(run_matmul(lg, np.ones((70, 300), np.float32), np.ones((300, 50), np.float32)) == 300)


def test_matmul_leading_dimensions(lg, lgo):
    M, N, K = 150, 200, 72
    A, B = si.matmul_inputs(114, M, N, K)
    ref = lgo.matmul(A, B)
    for pa, pb, pc in [(8, 4, 12), (3, 5, 1)]:      # aligned (vector path) and odd (scalar path)
        Ad = torch.full((M, K + pa), float("nan"), device="cuda"); Ad[:, :K] = dev(A)
        Bd = torch.full((K, N + pb), float("nan"), device="cuda"); Bd[:, :N] = dev(B)
        Cd = torch.full((M, N + pc), 7.0, device="cuda")
        lg.lg_matmul(Ad[:, :K], Bd[:, :N], Cd[:, :N], workspace=workspace(lg.lg_matmul_workspace_bytes(M, N, K)))
        sync()
        Ch = Cd.cpu().numpy()
        assert_close(Ch[:, :N], ref, K, "matmul ld")
        assert np.all(Ch[:, N:] == 7.0)


def test_matmul_zero_extents(lg):
    C = Guarded((5, 6), init=np.full((5, 6), 3.0, np.float32))
    lg.lg_matmul(torch.empty((5, 0), device="cuda"), torch.empty((0, 6), device="cuda"), C.t)
    sync(); C.check()
    assert np.all(C.host() == 0)
    C = Guarded((5, 6), init=np.full((5, 6), 3.0, np.float32))
    lg.lg_matmul(torch.empty((5, 0), device="cuda"), torch.empty((0, 6), device="cuda"), C.t, accumulate=True)
    sync(); C.check()
    assert np.all(C.host() == 3.0)
    lg.lg_matmul(torch.empty((0, 4), device="cuda"), torch.empty((4, 6), device="cuda"), torch.empty((0, 6), device="cuda"))


def test_matmul_is_deterministic(lg):
    A, B = si.matmul_inputs(115, 384, 640, 1000)
    c1 = run_matmul(lg, A, B)
    c2 = run_matmul(lg, A, B)
    assert np.array_equal(bits(c1), bits(c2))


def test_matmul_workspace_errors(lg):
    # a shape the planner splits along k (found, not assumed: the plan is the library's business)
    shape = next((s for s in [(784, 512, 4608), (512, 1024, 8192), (1024, 1024, 16384), (640, 640, 32768)]
                  if lg.lg_matmul_workspace_bytes(*s) > 0), None)
    assert shape is not None, "no candidate shape is split along k"
    M, N, K = shape
    need = lg.lg_matmul_workspace_bytes(M, N, K)
    A = torch.zeros((M, K), device="cuda"); B = torch.zeros((K, N), device="cuda"); C = torch.zeros((M, N), device="cuda")
    with pytest.raises(lg.LgError) as e:
        lg.lg_matmul(A, B, C)
    assert e.value.status == -3
    with pytest.raises(lg.LgError):
        lg.lg_matmul(A, B, C, workspace=workspace(need - 4))
    # and with the split forced on a small shape
    need = lg.lg_gemm_variant_workspace_bytes(256, 256, 1024, 3, 4)
    assert need == 4 * 256 * 256 * 4
    A = torch.zeros((256, 1024), device="cuda"); B = torch.zeros((1024, 256), device="cuda"); C = torch.zeros((256, 256), device="cuda")
    with pytest.raises(lg.LgError) as e:
        lg.lg_matmul_variant(A, B, C, 3, 4)
    assert e.value.status == -3
    with pytest.raises(lg.LgError):
        lg.lg_matmul_variant(A, B, C, 3, 4, workspace=workspace(need - 4))
    # a workspace that overlaps an operand or the output would silently corrupt the product: rejected
    big = torch.zeros(need // 4 + 256 * 256, device="cuda")
    for victim in ("A", "B", "C"):
        n = 256 * 1024 if victim != "C" else 256 * 256
        t = big[:n].view((256, 1024) if victim == "A" else (1024, 256) if victim == "B" else (256, 256))
        ops = dict(A=A, B=B, C=C)
        ops[victim] = t
        with pytest.raises(lg.LgError) as e:
            lg.lg_matmul_variant(ops["A"], ops["B"], ops["C"], 3, 4, workspace=big[64:64 + need // 4])
        assert e.value.status == -1, victim
    lg.lg_matmul_variant(A, B, C, 3, 4, workspace=workspace(need))
    sync()
    assert bool((C == 0).all())


@pytest.mark.parametrize("case,shape", list(enumerate(si.MATMUL_SWEEP)))
def test_matmul_full_size_sampled(lg, lgo, case, shape):
    """Benchmark sweep shapes, in the launch configuration the benchmark times.  What the oracle
    checks element by element: the WHOLE output for 1024^3 and 4096 x 4096 x 64 (2 GFLOP each);
    for 4096^3, 8192^3 and 16384 x 512 x 2048 a sample of at least 256 full rows (all N columns)
    that holds the two rows on either side of every boundary between workgroup tiles along M
    (block_m from the library's plan query), the first and the last row, and seeded random rows
    for the rest -- 34 GFLOP of naive loop nest for 8192^3.  Every element must be finite (the
    output is pre-filled with NaN)."""
    M, N, K = shape
    A, B = si.matmul_inputs(2, M, N, K, case=case)
    Cd = torch.full((M, N), float("nan"), device="cuda")
    ws = workspace(lg.lg_matmul_workspace_bytes(M, N, K))
    lg.lg_matmul(dev(A), dev(B), Cd, workspace=ws)
    sync()
    assert bool(torch.isfinite(Cd).all())
    if 2.0 * M * N * K <= 3e9:
        assert_close(Cd.cpu().numpy(), lgo.matmul(A, B), K, f"matmul {shape} (whole output)")
        return
    bm = lg.lg_matmul_plan(M, N, K)[0]
    rows = {0, M - 1}
    for b in range(bm, M, bm):
        rows.update((b - 1, b))
    rng = np.random.default_rng(1000 + case)
    while len(rows) < 256:
        rows.add(int(rng.integers(0, M)))
    rows = np.array(sorted(rows))
    ref = lgo.matmul(np.ascontiguousarray(A[rows]), B)
    got = Cd[torch.from_numpy(rows).cuda()].cpu().numpy()
    assert_close(got, ref, K, f"matmul {shape}, {len(rows)} rows incl. every {bm}-row tile boundary")


MATMUL_T_SHAPES = [(1, 1, 1), (5, 7, 3), (64, 64, 64), (130, 70, 50), (256, 256, 256), (300, 520, 136),
                   (1000, 24, 2000), (1024, 1024, 320), (2048, 1024, 128), (516, 260, 1028), (4100, 4104, 36)]


@pytest.mark.parametrize("M,N,K", MATMUL_T_SHAPES)
@pytest.mark.parametrize("trans", ["a", "b"])
def test_matmul_transposed_matches_oracle(lg, lgo, M, N, K, trans):
    A, B = si.matmul_inputs(116, M, N, K)
    ta, tb = trans == "a", trans == "b"
    As = np.ascontiguousarray(A.T) if ta else A          # stored K x M
    Bs = np.ascontiguousarray(B.T) if tb else B          # stored N x K
    out = Guarded((M, N), init=np.full((M, N), np.nan, np.float32))
    ws = workspace(lg.lg_matmul_workspace_bytes(M, N, K))
    lg.lg_matmul_t(dev(As), dev(Bs), out.t, trans_a=ta, trans_b=tb, workspace=ws)
    sync(); out.check()
    assert_close(out.host(), lgo.matmul_t(As, Bs, trans_a=ta, trans_b=tb), K, f"matmul_t {trans} {M}x{N}x{K}")


def test_matmul_transposed_accumulate_ld_exact(lg, lgo):
    M, N, K = 136, 200, 72
    A, B = si.matmul_inputs(117, M, N, K)
    C0 = si.uniform(117, 7, (M, N), -1, 1)
    for ta, tb in [(True, False), (False, True)]:
        As = np.ascontiguousarray(A.T) if ta else A
        Bs = np.ascontiguousarray(B.T) if tb else B
        ref = C0.copy(); lgo.matmul_t(As, Bs, trans_a=ta, trans_b=tb, C=ref, accumulate=True)
        for pad in (4, 3):        # aligned and odd leading dimensions
            Ad = torch.full((As.shape[0], As.shape[1] + pad), float("nan"), device="cuda"); Ad[:, :As.shape[1]] = dev(As)
            Bd = torch.full((Bs.shape[0], Bs.shape[1] + pad), float("nan"), device="cuda"); Bd[:, :Bs.shape[1]] = dev(Bs)
            Cd = torch.full((M, N + pad), 7.0, device="cuda"); Cd[:, :N] = dev(C0)
            lg.lg_matmul_t(Ad[:, :As.shape[1]], Bd[:, :Bs.shape[1]], Cd[:, :N], trans_a=ta, trans_b=tb, accumulate=True,
                           workspace=workspace(lg.lg_matmul_workspace_bytes(M, N, K)))
            sync()
            Ch = Cd.cpu().numpy()
            assert_close(Ch[:, :N], ref, K, "matmul_t accumulate/ld")
            assert np.all(Ch[:, N:] == 7.0)
    # integer-valued operands: exact in any order
    Ai = si.small_integers(118, 0, (96, 200)); Bi = si.small_integers(118, 1, (96, 136))      # A stored K x M
    out = Guarded((200, 136)); lg.lg_matmul_t(dev(Ai), dev(Bi), out.t, trans_a=True); sync(); out.check()
    assert np.array_equal(out.host(), lgo.matmul_t(Ai, Bi, trans_a=True))
    with pytest.raises(lg.LgError) as e:
        lg.lg_matmul_t(dev(Ai), dev(Bi.T.copy()), out.t, trans_a=True, trans_b=True)
    assert e.value.status == -2


def test_matmul_transposed_full_size_sampled(lg, lgo):
    M = N = K = 4096
    A, B = si.matmul_inputs(2, M, N, K, case=1)
    for ta, tb in [(True, False), (False, True)]:
        As = np.ascontiguousarray(A.T) if ta else A
        Bs = np.ascontiguousarray(B.T) if tb else B
        Cd = torch.full((M, N), float("nan"), device="cuda")
        lg.lg_matmul_t(dev(As), dev(Bs), Cd, trans_a=ta, trans_b=tb, workspace=workspace(lg.lg_matmul_workspace_bytes(M, N, K)))
        sync()
        for r0 in (0, 252, M - 8):
            ref = lgo.matmul(np.ascontiguousarray(A[r0:r0 + 8]), B)
            assert_close(Cd[r0:r0 + 8].cpu().numpy(), ref, K, f"matmul_t full rows {r0}")
        assert bool(torch.isfinite(Cd).all())


# ------------------------------------------------------------------------------- conv2d

def run_conv(lg, I, Kf, stride=(1, 1), dilation=(1, 1), O0=None, accumulate=False):
    N, H, W, C = I.shape
    KH, KW, _, F = Kf.shape
    OH = lg.lg_conv_out_extent(H, KH, stride[0], dilation[0])
    OW = lg.lg_conv_out_extent(W, KW, stride[1], dilation[1])
    out = Guarded((N, OH, OW, F), init=O0 if O0 is not None else np.full((N, OH, OW, F), np.nan, np.float32))
    ws = workspace(lg.lg_conv2d_workspace_bytes(N, H, W, C, KH, KW, F, *stride, *dilation))
    lg.lg_conv2d_nhwc_hwcf(dev(I), dev(Kf), out.t, stride=stride, dilation=dilation,
                           accumulate=accumulate, workspace=ws)
    sync()
    out.check()
    return out.host()


CONV_SMALL = [
    # N, H, W, C, F, KH, KW, stride, dilation
    (2, 12, 14, 8, 16, 3, 3, (1, 1), (1, 1)),
    (1, 9, 9, 3, 5, 3, 2, (1, 1), (1, 1)),          # C, F not multiples of 4 -> scalar path
    (2, 20, 17, 12, 20, 2, 3, (2, 1), (1, 2)),
    (3, 15, 15, 4, 8, 3, 3, (1, 3), (2, 1)),
    (1, 30, 30, 20, 72, 1, 1, (2, 2), (1, 1)),
    (2, 1, 40, 8, 12, 1, 5, (1, 2), (1, 3)),        # 1-D convolution as H = KH = 1
    (4, 18, 18, 32, 64, 3, 3, (1, 1), (1, 1)),      # the paper's channel/filter counts (C, F) = (32, 64)
    (1, 40, 40, 16, 136, 3, 3, (1, 1), (1, 1)),
    (3, 17, 19, 24, 40, 1, 1, (1, 1), (1, 1)),      # 1x1 at stride 1: runs as the plain matmul
    (2, 33, 31, 64, 64, 1, 1, (1, 1), (2, 3)),      # dilation is irrelevant to a 1x1 filter
    (2, 9, 9, 5, 3, 1, 1, (1, 1), (1, 1)),
    (4, 34, 34, 24, 64, 3, 3, (1, 1), (1, 1)),      # K = 216: thirteen whole slices and a tail of 8
    (4, 20, 20, 20, 128, 3, 3, (2, 2), (1, 1)),     # K = 180
    (2, 40, 40, 36, 64, 5, 5, (1, 1), (2, 2)),      # K = 900
]


@pytest.mark.parametrize("case", CONV_SMALL)
def test_conv2d_matches_oracle(lg, lgo, case):
    N, H, W, C, F, KH, KW, st, dl = case
    I, Kf = si.conv2d_inputs(120, N, H, W, C, F, KH, KW)
    O = run_conv(lg, I, Kf, st, dl)
    assert_close(O, lgo.conv2d_nhwc_hwcf(I, Kf, stride=st, dilation=dl), KH * KW * C, f"conv {case}")


def test_conv2d_accumulate_and_exact(lg, lgo):
    N, H, W, C, F, KH, KW = 2, 10, 11, 8, 12, 3, 3
    I, Kf = si.conv2d_inputs(121, N, H, W, C, F, KH, KW)
    O0 = si.uniform(121, 9, (N, H - 2, W - 2, F), -1, 1)
    O = run_conv(lg, I, Kf, O0=O0, accumulate=True)
    ref = O0.copy()
    lgo.conv2d_nhwc_hwcf(I, Kf, ref, accumulate=True)
    assert_close(O, ref, KH * KW * C, "conv accumulate")
    Ii = si.small_integers(122, 0, (2, 9, 9, 8))
    Ki = si.small_integers(122, 1, (3, 3, 8, 8))
    assert np.array_equal(run_conv(lg, Ii, Ki, (2, 1), (1, 2)), lgo.conv2d_nhwc_hwcf(Ii, Ki, stride=(2, 1), dilation=(1, 2)))
    # delta filter: the output is a strided crop of the input, bit for bit
    Kd = np.zeros((3, 3, 8, 8), np.float32)
    Kd[2, 1] = np.eye(8, dtype=np.float32)
    X = si.uniform(123, 0, (1, 12, 12, 8), -1, 1)
    assert np.array_equal(bits(run_conv(lg, X, Kd)), bits(X[:, 2:12, 1:11, :]))


@pytest.mark.parametrize("case,shape", list(enumerate(si.CONV2D_SHAPES + [si.CONV2D_LARGE])))
def test_conv2d_full_size(lg, lgo, case, shape):
    N, H, W, C, F, KH, KW, s = shape
    I, Kf = si.conv2d_inputs(3, N, H, W, C, F, KH, KW, case=case)
    O = run_conv(lg, I, Kf, (s, s))
    # all images, the whole output (1.6-1.9 GFLOP of naive loop nest per configuration)
    ref = lgo.conv2d_nhwc_hwcf(I, Kf, stride=(s, s))
    assert_close(O, ref, KH * KW * C, f"conv {shape} (whole output)")


# ------------------------------------------------------------------------------- conv1d

def run_conv1d(lg, I, Kf, s=1, d=1, O0=None, accumulate=False):
    N, W, C = I.shape
    KW, _, F = Kf.shape
    OW = lg.lg_conv_out_extent(W, KW, s, d)
    out = Guarded((N, OW, F), init=O0 if O0 is not None else np.full((N, OW, F), np.nan, np.float32))
    ws = workspace(lg.lg_conv1d_workspace_bytes(N, W, C, KW, F, s, d))
    lg.lg_conv1d_nwc_wcf(dev(I), dev(Kf), out.t, stride=s, dilation=d, accumulate=accumulate, workspace=ws)
    sync(); out.check()
    return out.host()


# the paper's 1-D sweep (Section 4.6.2): (N, C, F, K_w) = (1, 32, 64, 3), strides and dilations 1 and 2,
# widths including the ragged 20 and 55; plus batches, odd channel counts and a long signal
@pytest.mark.parametrize("N,W,C,F,KW", [(1, 20, 32, 64, 3), (1, 55, 32, 64, 3), (1, 256, 32, 64, 3),
                                        (3, 77, 5, 7, 4), (2, 5000, 48, 96, 5)])
@pytest.mark.parametrize("s,d", [(1, 1), (2, 1), (1, 2), (2, 2)])
def test_conv1d_matches_oracle(lg, lgo, N, W, C, F, KW, s, d):
    I = si.uniform(125, 0, (N, W, C), -1, 1)
    Kf = si.uniform(125, 1, (KW, C, F), -1, 1)
    assert_close(run_conv1d(lg, I, Kf, s, d), lgo.conv1d_nwc_wcf(I, Kf, stride=s, dilation=d), KW * C,
                 f"conv1d {(N, W, C, F, KW, s, d)}")


def test_conv1d_accumulate_and_exact(lg, lgo):
    I = si.uniform(126, 0, (2, 60, 8), -1, 1)
    Kf = si.uniform(126, 1, (3, 8, 12), -1, 1)
    O0 = si.uniform(126, 9, (2, 28, 12), -1, 1)
    ref = O0.copy(); lgo.conv1d_nwc_wcf(I, Kf, ref, stride=2, dilation=2, accumulate=True)
    assert_close(run_conv1d(lg, I, Kf, 2, 2, O0=O0, accumulate=True), ref, 24, "conv1d accumulate")
    Ii = si.small_integers(127, 0, (2, 33, 8))
    Ki = si.small_integers(127, 1, (3, 8, 8))
    assert np.array_equal(run_conv1d(lg, Ii, Ki, 2, 1), lgo.conv1d_nwc_wcf(Ii, Ki, stride=2))


# the paper's 2-D sweep: (N, C, F, K_h, K_w) = (1, 32, 64, 3, 3), strides and dilations 1 and 2
@pytest.mark.parametrize("HW", [20, 55])
@pytest.mark.parametrize("s,d", [(1, 1), (2, 1), (1, 2), (2, 2)])
def test_conv2d_paper_sweep(lg, lgo, HW, s, d):
    I, Kf = si.conv2d_inputs(128, 1, HW, HW, 32, 64, 3, 3)
    assert_close(run_conv(lg, I, Kf, (s, s), (d, d)), lgo.conv2d_nhwc_hwcf(I, Kf, stride=(s, s), dilation=(d, d)),
                 288, f"conv2d sweep {(HW, s, d)}")


# ------------------------------------------------------------------------------- depthwise

def run_dw1(lg, I, Kf, s=1, d=1, O0=None, accumulate=False):
    N, W, C = I.shape
    OW = lg.lg_conv_out_extent(W, Kf.shape[0], s, d)
    out = Guarded((N, OW, C), init=O0 if O0 is not None else np.full((N, OW, C), np.nan, np.float32))
    lg.lg_dwconv1d_nwc_wc(dev(I), dev(Kf), out.t, stride=s, dilation=d, accumulate=accumulate)
    sync(); out.check()
    return out.host()


def run_dw2(lg, I, Kf, st=(1, 1), dl=(1, 1), O0=None, accumulate=False):
    N, H, W, C = I.shape
    OH = lg.lg_conv_out_extent(H, Kf.shape[0], st[0], dl[0])
    OW = lg.lg_conv_out_extent(W, Kf.shape[1], st[1], dl[1])
    out = Guarded((N, OH, OW, C), init=O0 if O0 is not None else np.full((N, OH, OW, C), np.nan, np.float32))
    lg.lg_dwconv2d_nhwc_hwc(dev(I), dev(Kf), out.t, stride=st, dilation=dl, accumulate=accumulate)
    sync(); out.check()
    return out.host()


@pytest.mark.parametrize("N,W,C,KW,s,d", [
    (1, 40, 32, 3, 1, 1),          # the paper's (N, C, K_w) = (1, 32, 3)
    (3, 100, 64, 3, 1, 1), (2, 19, 8, 3, 1, 1), (2, 3, 4, 3, 1, 1),
    (2, 50, 12, 3, 2, 1), (2, 50, 12, 3, 1, 2), (1, 64, 20, 5, 2, 2),
    (2, 33, 7, 3, 1, 1), (1, 17, 1, 2, 1, 1), (4, 1000, 512, 3, 1, 1),
    # the paper's stride x dilation sweep at (N, C, K_w) = (1, 32, 3), Section 4.7
    (1, 259, 32, 3, 2, 1), (1, 259, 32, 3, 1, 2), (1, 259, 32, 3, 2, 2), (3, 700, 256, 7, 3, 2),
])
def test_dwconv1d_matches_oracle(lg, lgo, N, W, C, KW, s, d):
    I, Kf = si.dwconv1d_inputs(130, N, W, C, KW)
    assert_close(run_dw1(lg, I, Kf, s, d), lgo.dwconv1d_nwc_wc(I, Kf, stride=s, dilation=d), KW, "dwconv1d")


@pytest.mark.parametrize("N,H,W,C,KH,KW,st,dl", [
    (1, 20, 20, 32, 3, 3, (1, 1), (1, 1)),      # the paper's (N, C, K_h, K_w) = (1, 32, 3, 3)
    (2, 11, 13, 8, 3, 3, (1, 1), (1, 1)), (1, 3, 3, 4, 3, 3, (1, 1), (1, 1)),
    (2, 35, 37, 96, 3, 3, (1, 1), (1, 1)), (2, 14, 15, 12, 3, 3, (2, 1), (1, 2)),
    (1, 16, 16, 6, 2, 4, (1, 2), (2, 1)), (2, 10, 9, 5, 3, 3, (1, 1), (1, 1)),
    (2, 1, 30, 8, 1, 3, (1, 1), (1, 1)),
    # the paper's stride x dilation sweep at (N, C, K_h, K_w) = (1, 32, 3, 3), Section 4.7
    (1, 41, 43, 32, 3, 3, (2, 2), (1, 1)), (1, 41, 43, 32, 3, 3, (1, 1), (2, 2)),
    (1, 41, 43, 32, 3, 3, (2, 2), (2, 2)), (2, 60, 57, 128, 5, 4, (2, 3), (3, 2)),
])
def test_dwconv2d_matches_oracle(lg, lgo, N, H, W, C, KH, KW, st, dl):
    I, Kf = si.dwconv2d_inputs(131, N, H, W, C, KH, KW)
    assert_close(run_dw2(lg, I, Kf, st, dl), lgo.dwconv2d_nhwc_hwc(I, Kf, stride=st, dilation=dl), KH * KW, "dwconv2d")


# every register-window instantiation (filter width 3, 5, 7; stride and dilation 1 or 2), ragged
# extents so that the last run of every phase is partial, overwrite and accumulate
@pytest.mark.parametrize("KW", [3, 5, 7])
@pytest.mark.parametrize("s,d", [(1, 1), (2, 1), (1, 2), (2, 2)])
def test_dwconv1d_window_kernels(lg, lgo, KW, s, d):
    for N, W, C in [(3, 261, 24), (1, (KW - 1) * d + 1, 8), (2, (KW - 1) * d + 1 + 3 * s, 4)]:
        I, Kf = si.dwconv1d_inputs(134 + KW, N, W, C, KW)
        ref = lgo.dwconv1d_nwc_wc(I, Kf, stride=s, dilation=d)
        assert_close(run_dw1(lg, I, Kf, s, d), ref, KW, f"dwconv1d window {(N, W, C, KW, s, d)}")
        O0 = si.uniform(135, KW, ref.shape, -1, 1)
        ref2 = O0.copy(); lgo.dwconv1d_nwc_wc(I, Kf, ref2, stride=s, dilation=d, accumulate=True)
        assert_close(run_dw1(lg, I, Kf, s, d, O0=O0, accumulate=True), ref2, KW, "dwconv1d window accumulate")


@pytest.mark.parametrize("s,d", [(1, 1), (2, 1), (1, 2), (2, 2)])
def test_dwconv2d_window_kernels(lg, lgo, s, d):
    for N, H, W, C in [(2, 37, 41, 24), (1, 2 * d + 1, 2 * d + 1, 4), (1, 2 * d + 1 + 5 * s, 2 * d + 1 + s, 8)]:
        I, Kf = si.dwconv2d_inputs(136, N, H, W, C, 3, 3)
        ref = lgo.dwconv2d_nhwc_hwc(I, Kf, stride=(s, s), dilation=(d, d))
        assert_close(run_dw2(lg, I, Kf, (s, s), (d, d)), ref, 9, f"dwconv2d window {(N, H, W, C, s, d)}")
        O0 = si.uniform(137, s, ref.shape, -1, 1)
        ref2 = O0.copy(); lgo.dwconv2d_nhwc_hwc(I, Kf, ref2, stride=(s, s), dilation=(d, d), accumulate=True)
        assert_close(run_dw2(lg, I, Kf, (s, s), (d, d), O0=O0, accumulate=True), ref2, 9, "dwconv2d window accumulate")


# the row-streaming kernel: filter widths 2 ... 9 at horizontal stride and dilation 1, any height,
# vertical stride and dilation; short runs (small problems) and long runs, ragged last run, accumulate
@pytest.mark.parametrize("N,H,W,C,KH,KW,sh,dh", [
    (2, 20, 23, 64, 5, 5, 1, 1), (1, 16, 19, 96, 7, 7, 1, 1), (2, 9, 40, 64, 1, 9, 1, 1), (3, 14, 11, 68, 2, 4, 2, 1),
    (2, 17, 13, 128, 3, 6, 1, 2), (1, 12, 9, 64, 4, 8, 3, 3), (2, 8, 10, 72, 3, 2, 1, 1), (1, 7, 7, 64, 7, 7, 1, 1),
    (8, 70, 70, 256, 7, 7, 1, 1), (4, 64, 133, 128, 5, 5, 2, 1),
    # channel counts that are not a multiple of 4: one channel per lane
    (2, 20, 23, 65, 3, 3, 1, 1), (1, 16, 19, 97, 7, 7, 1, 1), (3, 1, 300, 130, 1, 5, 1, 1), (2, 9, 33, 67, 3, 3, 2, 2),
    (4, 70, 140, 255, 3, 3, 1, 1),
    # 32 ... 63 channels: one channel per lane whether or not they are a multiple of 4
    (1, 12, 9, 60, 4, 8, 3, 3), (2, 20, 23, 33, 5, 5, 1, 1), (2, 20, 23, 48, 5, 5, 1, 1), (2, 1, 200, 32, 1, 4, 1, 1),
    # fewer than 32 channels: the general kernels take these
    (2, 20, 23, 8, 5, 5, 1, 1), (2, 20, 23, 31, 5, 5, 1, 1)])
def test_dwconv_row_streaming_kernel(lg, lgo, N, H, W, C, KH, KW, sh, dh):
    I, Kf = si.dwconv2d_inputs(139 + KW, N, H, W, C, KH, KW)
    ref = lgo.dwconv2d_nhwc_hwc(I, Kf, stride=(sh, 1), dilation=(dh, 1))
    assert_close(run_dw2(lg, I, Kf, (sh, 1), (dh, 1)), ref, KH * KW, f"dwconv rows {(N, H, W, C, KH, KW, sh, dh)}")
    if N * H * W * C < 400000:
        O0 = si.uniform(139, KW, ref.shape, -1, 1)
        ref2 = O0.copy(); lgo.dwconv2d_nhwc_hwc(I, Kf, ref2, stride=(sh, 1), dilation=(dh, 1), accumulate=True)
        assert_close(run_dw2(lg, I, Kf, (sh, 1), (dh, 1), O0=O0, accumulate=True), ref2, KH * KW, "dwconv rows accumulate")


# the row-streaming kernel at horizontal stride / dilation 2 (widths 3, 5, 7): 128-bit and one-channel
# lanes, ragged last runs, unequal vertical and horizontal strides, 1-D signals, accumulate
@pytest.mark.parametrize("N,H,W,C,KH,KW,st,dl", [
    (2, 23, 25, 64, 5, 5, (2, 2), (1, 1)), (1, 30, 31, 96, 5, 5, (1, 1), (2, 2)), (2, 21, 22, 72, 7, 7, (2, 2), (2, 2)),
    (2, 17, 19, 65, 3, 3, (2, 2), (1, 1)), (1, 19, 27, 67, 3, 3, (1, 1), (2, 2)), (2, 19, 21, 130, 5, 5, (2, 2), (2, 2)),
    (3, 12, 40, 64, 3, 5, (1, 2), (1, 1)), (2, 15, 33, 100, 2, 7, (3, 1), (1, 2)), (2, 11, 16, 64, 3, 3, (1, 2), (2, 1)),
    (4, 1, 301, 63, 1, 5, (1, 2), (1, 2)), (2, 1, 64, 129, 1, 7, (1, 2), (1, 1)), (8, 61, 61, 144, 5, 5, (2, 2), (1, 1)),
    (2, 23, 25, 50, 5, 5, (2, 2), (1, 1)), (2, 23, 25, 36, 7, 7, (1, 1), (2, 2)), (2, 23, 25, 31, 5, 5, (2, 2), (1, 1))])
def test_dwconv_row_streaming_kernel_strided(lg, lgo, N, H, W, C, KH, KW, st, dl):
    I, Kf = si.dwconv2d_inputs(170 + KW, N, H, W, C, KH, KW)
    ref = lgo.dwconv2d_nhwc_hwc(I, Kf, stride=st, dilation=dl)
    assert_close(run_dw2(lg, I, Kf, st, dl), ref, KH * KW, f"dwconv rows strided {(N, H, W, C, KH, KW, st, dl)}")
    if N * H * W * C < 400000:
        O0 = si.uniform(170, KW, ref.shape, -1, 1)
        ref2 = O0.copy(); lgo.dwconv2d_nhwc_hwc(I, Kf, ref2, stride=st, dilation=dl, accumulate=True)
        assert_close(run_dw2(lg, I, Kf, st, dl, O0=O0, accumulate=True), ref2, KH * KW, "dwconv rows strided accumulate")


# the 2-D depthwise sizes of Section 4.7: batch-1 MobileNet layers (output extent x channels), each
# at strides and dilations 1 and 2
@pytest.mark.parametrize("size,C", [(112, 32), (112, 64), (56, 128), (28, 256), (14, 512), (7, 1024)])
@pytest.mark.parametrize("s,d", [(1, 1), (2, 1), (1, 2), (2, 2)])
def test_dwconv2d_mobilenet_layers(lg, lgo, size, C, s, d):
    H = (size - 1) * s + 2 * d + 1
    I, Kf = si.dwconv2d_inputs(138 + C, 1, H, H, C, 3, 3)
    ref = lgo.dwconv2d_nhwc_hwc(I, Kf, stride=(s, s), dilation=(d, d))
    assert ref.shape == (1, size, size, C)
    assert_close(run_dw2(lg, I, Kf, (s, s), (d, d)), ref, 9, f"dwconv2d {size}x{size}x{C} s{s} d{d}")


def test_dwconv_accumulate_and_delta(lg, lgo):
    I, Kf = si.dwconv1d_inputs(132, 2, 50, 16, 3)
    O0 = si.uniform(132, 9, (2, 48, 16), -1, 1)
    ref = O0.copy(); lgo.dwconv1d_nwc_wc(I, Kf, ref, accumulate=True)
    assert_close(run_dw1(lg, I, Kf, O0=O0, accumulate=True), ref, 3, "dwconv1d accumulate")
    I2, K2 = si.dwconv2d_inputs(133, 2, 12, 12, 8, 3, 3)
    O0 = si.uniform(133, 9, (2, 10, 10, 8), -1, 1)
    ref = O0.copy(); lgo.dwconv2d_nhwc_hwc(I2, K2, ref, accumulate=True)
    assert_close(run_dw2(lg, I2, K2, O0=O0, accumulate=True), ref, 9, "dwconv2d accumulate")
    I3, K3 = si.dwconv2d_inputs(134, 2, 21, 20, 16, 3, 3)
    O0 = si.uniform(134, 9, (2, 9, 8, 16), -1, 1)
    ref = O0.copy(); lgo.dwconv2d_nhwc_hwc(I3, K3, ref, stride=(2, 2), dilation=(2, 2), accumulate=True)
    assert_close(run_dw2(lg, I3, K3, (2, 2), (2, 2), O0=O0, accumulate=True), ref, 9, "dwconv2d strided accumulate")
    Kd = np.zeros((3, 3, 8), np.float32); Kd[1, 2] = 1
    assert np.array_equal(bits(run_dw2(lg, I2, Kd)), bits(I2[:, 1:11, 2:12, :]))
    K1 = np.zeros((3, 16), np.float32); K1[2] = 1
    assert np.array_equal(bits(run_dw1(lg, I, K1)), bits(I[:, 2:50]))


# the 3 x 3 kernel that stages 8 x 16 pixel x 32 channel tiles through LDS: exact tile multiples, ragged
# extents whose last tiles are moved inwards (and overlap their neighbours), the smallest extents it
# takes (one tile in either direction), one and several channel slabs, several images; next to them the
# shapes just outside it (fewer than 8 output rows or 16 columns, channels not a multiple of 32,
# accumulation), which must land on the other kernels with the same results
@pytest.mark.parametrize("N,H,W,C,accumulate", [
    (1, 10, 18, 32, False), (1, 18, 34, 32, False), (2, 26, 50, 64, False),
    (1, 11, 19, 32, False), (2, 17, 33, 96, False), (3, 25, 41, 32, False), (1, 58, 58, 128, False),
    (2, 31, 100, 160, False), (1, 114, 114, 96, False), (1, 9, 40, 32, False), (1, 40, 17, 32, False),
    (1, 40, 40, 48, False), (1, 40, 40, 36, False), (2, 26, 50, 64, True), (1, 11, 19, 32, True),
])
def test_dwconv2d_tile_kernel_shapes(lg, lgo, N, H, W, C, accumulate):
    I, Kf = si.dwconv2d_inputs(136, N, H, W, C, 3, 3)
    O0 = si.uniform(136, 9, (N, H - 2, W - 2, C), -1, 1) if accumulate else None
    got = run_dw2(lg, I, Kf, O0=O0, accumulate=accumulate)
    ref = lgo.dwconv2d_nhwc_hwc(I, Kf).astype(np.float64)
    if accumulate:
        ref = ref + O0.astype(np.float64)
    assert_close(got, ref, 9, f"dwconv2d tile {N}x{H}x{W}x{C} acc={accumulate}")


# the same staging at stride and dilation 2 (patch rows and columns gcd(S, D) apart): exact tile multiples,
# ragged extents with tiles moved inwards, the smallest extents a tile takes, extents whose moved tiles would
# recompute too much (they stay on the register-window kernel), several slabs and images
@pytest.mark.parametrize("st,dl", [(2, 1), (1, 2), (2, 2)])
@pytest.mark.parametrize("N,OH,OW,C", [(1, 8, 16, 32), (2, 16, 32, 64), (1, 9, 17, 32), (2, 23, 45, 96), (1, 56, 56, 128),
                                       (3, 13, 30, 32), (1, 27, 27, 64), (1, 4, 16, 32), (1, 7, 40, 32), (2, 20, 15, 32)])
def test_dwconv2d_tile_kernel_strides_dilations(lg, lgo, N, OH, OW, C, st, dl):
    H, W = (OH - 1) * st + 2 * dl + 1 + (st - 1), (OW - 1) * st + 2 * dl + 1        # a spare row at stride 2: floor in the extent
    I, Kf = si.dwconv2d_inputs(138, N, H, W, C, 3, 3)
    got = run_dw2(lg, I, Kf, st=(st, st), dl=(dl, dl))
    assert got.shape == (N, OH, OW, C)
    assert_close(got, lgo.dwconv2d_nhwc_hwc(I, Kf, stride=(st, st), dilation=(dl, dl)), 9,
                 f"dwconv2d tile {N}x{H}x{W}x{C} stride {st} dilation {dl}")


def test_dwconv2d_tile_kernel_delta_filter_is_a_crop(lg):
    """A filter with a single 1.0 tap copies a shifted crop of the input: bit-exact, every tap position
    (a wrong LDS row or column in the tile kernel's window shows as a shifted image)."""
    N, H, W, C = 2, 27, 37, 64
    I = si.uniform(137, 0, (N, H, W, C), -1, 1)
    for a in range(3):
        for b in range(3):
            Kf = np.zeros((3, 3, C), np.float32)
            Kf[a, b, :] = 1.0
            got = run_dw2(lg, I, Kf)
            assert np.array_equal(bits(got), bits(np.ascontiguousarray(I[:, a:a + H - 2, b:b + W - 2, :]))), (a, b)


def test_dwconv_full_size(lg, lgo):
    N, W, C, KW = si.DWCONV1D_SHAPE
    I, Kf = si.dwconv1d_inputs(4, N, W, C, KW)
    O = run_dw1(lg, I, Kf)
    assert_close(O, lgo.dwconv1d_nwc_wc(I, Kf), KW, "dwconv1d full (all 32 batches)")
    N, H, W, C, KH, KW = si.DWCONV2D_SHAPE
    I, Kf = si.dwconv2d_inputs(4, N, H, W, C, KH, KW)
    O = run_dw2(lg, I, Kf)
    assert_close(O, lgo.dwconv2d_nhwc_hwc(I, Kf), KH * KW, "dwconv2d full")


# ------------------------------------------------------------------------------- reductions

def run_rows(lg, x, out0=None, accumulate=False):
    out = Guarded((x.shape[0],), init=out0 if out0 is not None else np.full(x.shape[0], np.nan, np.float32))
    lg.lg_reduce_rows(dev(x), out.t, accumulate=accumulate)
    sync(); out.check()
    return out.host()


def run_cols(lg, x, out0=None, accumulate=False):
    out = Guarded((x.shape[1],), init=out0 if out0 is not None else np.full(x.shape[1], np.nan, np.float32))
    ws = workspace(lg.lg_reduce_cols_workspace_bytes(*x.shape))
    lg.lg_reduce_cols(dev(x), out.t, accumulate=accumulate, workspace=ws)
    sync(); out.check()
    return out.host()


RED_SHAPES = [(250, 960), (1, 1), (7, 5), (64, 4096), (100, 4100), (33, 8191), (513, 64),
              (1000, 3), (5, 20000), (300, 1024), (4096, 8), (129, 260),
              (2500, 1000), (2049, 260), (4100, 37), (2048, 4096),
              # short rows / narrow inputs: several rows per wavefront (128-bit and scalar variants)
              (70001, 64), (5000, 128), (3001, 100), (9000, 12), (4097, 4), (20000, 1), (777, 31),
              (2600, 33), (1500, 256), (999, 63), (100003, 2),
              # a few long rows: 16-wavefront workgroups per row (128-bit and scalar); small inputs whose column
              # sums take one launch
              (3, 100000), (5, 65537), (700, 32768), (767, 32770), (100, 4098), (5001, 4), (257, 63)]


@pytest.mark.parametrize("R,Cn", RED_SHAPES)
def test_reductions_match_oracle(lg, lgo, R, Cn):
    x = si.uniform(1, 5, (R, Cn), 0, 1)
    assert_close(run_rows(lg, x), lgo.reduce_rows(x), Cn, f"reduce_rows {R}x{Cn}")
    assert_close(run_cols(lg, x), lgo.reduce_cols(x), R, f"reduce_cols {R}x{Cn}")


def test_reductions_all_ones_accumulate_ld_and_empty(lg, lgo):
    ones = np.ones((300, 4096), np.float32)
    assert np.all(run_rows(lg, ones) == 4096) and np.all(run_cols(lg, ones) == 300)
    x = si.uniform(1, 6, (260, 520), 0, 1)
    r0 = si.uniform(1, 7, (260,), -1, 1); c0 = si.uniform(1, 8, (520,), -1, 1)
    rr = r0.copy(); lgo.reduce_rows(x, rr, accumulate=True)
    cc = c0.copy(); lgo.reduce_cols(x, cc, accumulate=True)
    assert_close(run_rows(lg, x, r0, True), rr, 520, "rows accumulate")
    assert_close(run_cols(lg, x, c0, True), cc, 260, "cols accumulate")
    for pad in (4, 3):
        xd = torch.full((260, 520 + pad), float("nan"), device="cuda"); xd[:, :520] = dev(x)
        o = torch.empty(260, device="cuda"); lg.lg_reduce_rows(xd[:, :520], o)
        oc = torch.empty(520, device="cuda")
        lg.lg_reduce_cols(xd[:, :520], oc, workspace=workspace(lg.lg_reduce_cols_workspace_bytes(260, 520)))
        sync()
        assert_close(o.cpu().numpy(), lgo.reduce_rows(x), 520, "rows ld")
        assert_close(oc.cpu().numpy(), lgo.reduce_cols(x), 260, "cols ld")
    e = torch.full((4,), 5.0, device="cuda")
    lg.lg_reduce_rows(torch.empty((4, 0), device="cuda"), e); sync()
    assert np.all(e.cpu().numpy() == 0)
    e = torch.full((4,), 5.0, device="cuda")
    lg.lg_reduce_cols(torch.empty((0, 4), device="cuda"), e); sync()
    assert np.all(e.cpu().numpy() == 0)


# a handful of very long rows: lg_reduce_rows_ws cuts them into pieces (one workgroup each) and adds
# the piece sums in a second pass; ragged last piece, unaligned, padded rows, accumulate
@pytest.mark.parametrize("R,Cn,pad", [(1, 1000000, 0), (3, 333333, 0), (7, 200004, 4), (2, 32768, 0), (100, 70000, 0),
                                      (511, 40000, 8), (5, 32767, 0), (512, 40000, 0), (1, 9000, 0)])
def test_reduce_rows_with_workspace(lg, lgo, R, Cn, pad):
    x = si.uniform(150 + R, 0, (R, Cn), 0, 1)
    need = lg.lg_reduce_rows_workspace_bytes(R, Cn)
    assert (need > 0) == (R < 512 and Cn >= 32768)
    xd = torch.full((R, Cn + pad), float("nan"), device="cuda")
    xd[:, :Cn] = dev(x)
    ref = lgo.reduce_rows(x)
    out = Guarded((R,))
    lg.lg_reduce_rows_ws(xd[:, :Cn], out.t, workspace=workspace(need)); sync(); out.check()
    assert_close(out.host(), ref, Cn, f"reduce_rows_ws {R}x{Cn}")
    o0 = si.uniform(151, R, (R,), -1, 1)
    acc = Guarded((R,), init=o0)
    lg.lg_reduce_rows_ws(xd[:, :Cn], acc.t, accumulate=True, workspace=workspace(need)); sync(); acc.check()
    assert_close(acc.host(), ref + o0, Cn, f"reduce_rows_ws accumulate {R}x{Cn}")
    again = Guarded((R,))
    lg.lg_reduce_rows_ws(xd[:, :Cn], again.t, workspace=workspace(need)); sync()
    assert np.array_equal(bits(again.host()), bits(out.host()))              # same pieces, same order
    if need:
        with pytest.raises(lg.LgError) as e:
            lg.lg_reduce_rows_ws(xd[:, :Cn], out.t)
        assert e.value.status == -3
        with pytest.raises(lg.LgError):
            lg.lg_reduce_rows_ws(xd[:, :Cn], out.t, workspace=workspace(need - 4))


def test_reductions_full_size(lg, lgo):
    x = si.uniform(1, 0, si.REDUCE_SHAPE, 0, 1)
    assert_close(run_rows(lg, x), lgo.reduce_rows(x), x.shape[1], "reduce_rows full")
    assert_close(run_cols(lg, x), lgo.reduce_cols(x), x.shape[0], "reduce_cols full")


# ------------------------------------------------------------------------------- transpose / copy

def special_bits(shape, seed):
    n = int(np.prod(shape))
    b = (si.bits24(seed, 0, n) << np.uint32(8)) | (si.bits24(seed, 1, n) & np.uint32(0xFF))
    sp = np.array([0x80000000, 0x7F800000, 0xFF800000, 0x7FC00001, 0xFFC12345, 0x7F800001,
                   0x00000001, 0x807FFFFF, 0x00800000], np.uint32)
    k = min(len(sp), len(b[::2]))
    b[::2][:k] = sp[:k]
    return b.reshape(shape)


@pytest.mark.parametrize("R,Cn", [(64, 64), (1, 1), (1, 19), (19, 1), (37, 53), (128, 256), (100, 260),
                                  (250, 960), (1000, 1000), (1027, 765), (4, 4096), (4096, 4),
                                  # thin matrices: the one-element-per-lane kernel on both of its sides
                                  (1, 100003), (100003, 1), (3, 70001), (70001, 3), (15, 257), (257, 15),
                                  (16, 300), (300, 16),
                                  # dense, more than 2^20 elements, not a multiple of 4: 128-bit body + scalar tail copy
                                  (1025, 1031), (1, 1048579)])
def test_transpose_and_copy_bit_exact(lg, lgo, R, Cn):
    xb = special_bits((R, Cn), 140)
    x = xb.view(np.float32)
    out = Guarded((Cn, R))
    lg.lg_transpose(dev(x), out.t); sync(); out.check()
    assert np.array_equal(bits(out.host()), bits(lgo.transpose(x)))
    back = Guarded((R, Cn))
    lg.lg_transpose(out.t, back.t); sync(); back.check()
    assert np.array_equal(bits(back.host()), xb)                 # transpose twice = identity
    cp = Guarded((R, Cn))
    lg.lg_copy2d(dev(x), cp.t); sync(); cp.check()
    assert np.array_equal(bits(cp.host()), bits(lgo.copy2d(x)))


@pytest.mark.parametrize("R,Cn", [(130, 200), (5, 999), (999, 5)])
def test_transpose_copy_leading_dims(lg, lgo, R, Cn):
    xb = special_bits((R, Cn), 141)
    for pi, po in [(8, 4), (3, 5)]:
        xd = torch.zeros((R, Cn + pi), dtype=torch.int32, device="cuda").view(torch.float32)
        xd[:, :Cn] = dev(xb.view(np.float32))
        od = torch.full((Cn, R + po), 0x5EADBEEF, dtype=torch.int32, device="cuda").view(torch.float32)
        lg.lg_transpose(xd[:, :Cn], od[:, :R]); sync()
        oh = od.view(torch.int32).cpu().numpy().view(np.uint32)
        assert np.array_equal(oh[:, :R], xb.T) and np.all(oh[:, R:] == 0x5EADBEEF)
        cd = torch.full((R, Cn + po), 0x5EADBEEF, dtype=torch.int32, device="cuda").view(torch.float32)
        lg.lg_copy2d(xd[:, :Cn], cd[:, :Cn]); sync()
        ch = cd.view(torch.int32).cpu().numpy().view(np.uint32)
        assert np.array_equal(ch[:, :Cn], xb) and np.all(ch[:, Cn:] == 0x5EADBEEF)


def run_transpose_batched(lg, lgo, xb, out_shape, R, Cn, ld_in, ld_out, B0, B1, ist, ost):
    """Runs both sides on the same bits; untouched output words must keep their fill pattern."""
    n_out = int(np.prod(out_shape))
    ref = np.full(n_out, 0x5EADBEEF, np.uint32)
    lgo.transpose_batched(np.ascontiguousarray(xb).view(np.float32).ravel(), ref.view(np.float32),
                          R, Cn, ld_in, ld_out, B0, B1, ist[0], ist[1], ost[0], ost[1])
    od = torch.full((n_out,), 0x5EADBEEF, dtype=torch.int32, device="cuda").view(torch.float32)
    lg.lg_transpose_batched(dev(np.ascontiguousarray(xb).view(np.float32).ravel()), od, R, Cn, ld_in, ld_out,
                            B0, B1, ist, ost)
    sync()
    got = od.view(torch.int32).cpu().numpy().view(np.uint32)
    assert np.array_equal(got, ref)
    return got.reshape(out_shape)


@pytest.mark.parametrize("dims", [(5, 3, 4, 7), (64, 6, 5, 128), (130, 2, 3, 260), (256, 9, 8, 256), (1, 1, 1, 1)])
def test_transpose_batched_4d_paper_permutation(lg, lgo, dims):
    # Section 4.4: [i,j,k,l] -> [k,j,l,i] as j x k transposes of (i, l) matrices
    Ni, Nj, Nk, Nl = dims
    xb = special_bits(dims, 142)
    got = run_transpose_batched(lg, lgo, xb, (Nk, Nj, Nl, Ni), Ni, Nl, Nj * Nk * Nl, Ni, Nj, Nk,
                                (Nk * Nl, Nl), (Nl * Ni, Nj * Nl * Ni))
    assert np.array_equal(got, np.transpose(xb, (2, 1, 3, 0)))


@pytest.mark.parametrize("N,H,W,C", [(5, 17, 19, 3), (2, 40, 33, 1), (3, 9, 8, 15)])
def test_transpose_batched_few_channels(lg, lgo, N, H, W, C):
    # NHWC -> NCHW and back with a handful of channels: per image a (H*W) x C matrix, too thin for LDS tiles
    xb = special_bits((N, H, W, C), 144)
    nchw = run_transpose_batched(lg, lgo, xb, (N, C, H, W), H * W, C, C, H * W, N, 1,
                                 (H * W * C, 0), (C * H * W, 0))
    assert np.array_equal(nchw, np.transpose(xb, (0, 3, 1, 2)))
    back = run_transpose_batched(lg, lgo, nchw, (N, H, W, C), C, H * W, H * W, C, N, 1,
                                 (C * H * W, 0), (H * W * C, 0))
    assert np.array_equal(back, xb)


def test_transpose_batched_3d_padded_and_empty(lg, lgo):
    # [b,i,j] -> [b,j,i] with padded rows on both sides: the padding keeps its fill pattern
    B, R, Cn, pi, po = 7, 50, 36, 3, 5
    xb = special_bits((B, R, Cn + pi), 143)
    got = run_transpose_batched(lg, lgo, xb, (B, Cn, R + po), R, Cn, Cn + pi, R + po, B, 1,
                                (R * (Cn + pi), 0), (Cn * (R + po), 0))
    assert np.array_equal(got[:, :, :R], np.transpose(xb[:, :, :Cn], (0, 2, 1)))
    assert np.all(got[:, :, R:] == 0x5EADBEEF)
    x = torch.zeros(16, device="cuda"); o = torch.zeros(16, device="cuda")
    lg.lg_transpose_batched(x, o, 4, 4, 4, 4, 0, 1, (0, 0), (0, 0)); sync()      # empty batch: no launch
    with pytest.raises(lg.LgError):
        lg.lg_transpose_batched(x, o, 2, 2, 1, 2, 1, 1, (0, 0), (0, 0))             # ld_in < Cn


def test_transpose_full_size(lg, lgo):
    x = si.uniform(1, 1, si.TRANSPOSE_SHAPE, 0, 1)
    od = torch.empty((x.shape[1], x.shape[0]), device="cuda")
    lg.lg_transpose(dev(x), od); sync()
    assert np.array_equal(bits(od.cpu().numpy()), bits(lgo.transpose(x)))


def test_mfma_probe_checksums(lg):
    """The matrix-pipe yardstick really does the MFMAs it is priced for: its per-lane checksums
    follow from the instruction's definition (D[i,j] += sum_k A[i,k] B[k,j], lane l holding A[l%32, l//32]
    and B[l//32, l%32]; a lane's 16 results are rows 8*(v//4) + 4*(l//32) + v%4 of column l%32)."""
    n = lg.lg_mfma_probe_out_elems()
    groups, threads, chains = 512, 256, 4
    assert n == groups * threads
    out = Guarded((n,))
    lg.lg_mfma_probe(out.t, 0); sync(); out.check()
    assert not out.host().any()
    iters = 48
    lg.lg_mfma_probe(out.t, iters); sync(); out.check()
    got = out.host().reshape(groups, threads // 64, 64).astype(np.float64)
    lane = np.arange(64)
    rows = np.array([[8 * (v // 4) + 4 * (l // 32) + v % 4 for v in range(16)] for l in lane])   # [lane, v]
    for g in (0, 1, 77, 511):
        for w in range(threads // 64):
            a = (((lane * 37 + g * 11) % 127) - 63) / 65536.0         # A[i = l%32, k = l//32]
            b = (((lane * 53 + w * 29) % 113) - 56) / 65536.0         # B[k = l//32, j = l%32]
            A = a.reshape(2, 32).T                                      # [i, k]
            B = b.reshape(2, 32)                                        # [k, j]
            D = A @ B                                                   # one MFMA's increment
            want = np.array([D[rows[l], l % 32].sum() for l in lane]) * iters * chains
            assert np.allclose(got[g, w], want, rtol=1e-5, atol=1e-9), (g, w)


# ------------------------------------------------------------------------------- misaligned base pointers

def shifted(a, fill=None):
    """A device copy of `a` (or a NaN-filled tensor of its shape) that starts 4 bytes into a 16-byte
    aligned allocation: every extent may be a multiple of 4 and still no access is 16-byte aligned."""
    n = int(np.prod(a.shape))
    buf = torch.full((n + 5,), float("nan") if fill is None else fill, device="cuda")
    view = buf[1:1 + n].view(*a.shape)
    if fill is None:
        view.copy_(dev(a))
    assert view.data_ptr() % 16 == 4
    return buf, view


@pytest.mark.parametrize("which", ["A", "B", "C"])
@pytest.mark.parametrize("M,N,K", [(256, 256, 256), (200, 192, 1024), (1024, 512, 64), (2048, 4, 2048)])
def test_matmul_misaligned_operand(lg, lgo, M, N, K, which):
    A, B = si.matmul_inputs(150, M, N, K)
    ref = lgo.matmul(A, B)
    keep = []
    Ad = shifted(A) if which == "A" else (None, dev(A))
    Bd = shifted(B) if which == "B" else (None, dev(B))
    Cd = shifted(np.empty((M, N), np.float32), fill=7.0) if which == "C" else (None, torch.empty((M, N), device="cuda"))
    keep += [Ad, Bd, Cd]
    lg.lg_matmul(Ad[1], Bd[1], Cd[1], workspace=workspace(lg.lg_matmul_workspace_bytes(M, N, K))); sync()
    assert_close(Cd[1].cpu().numpy(), ref, K, f"matmul with {which} 4 bytes off alignment")
    if which == "C":
        b = Cd[0].cpu().numpy()
        assert b[0] == 7.0 and np.all(b[1 + M * N:] == 7.0)       # nothing written outside the view
    for ta, tb in ((True, False), (False, True)):
        At = np.ascontiguousarray(A.T) if ta else A
        Bt = np.ascontiguousarray(B.T) if tb else B
        Ad2 = shifted(At) if which == "A" else (None, dev(At))
        Bd2 = shifted(Bt) if which == "B" else (None, dev(Bt))
        out = shifted(np.empty((M, N), np.float32), fill=7.0) if which == "C" else (None, torch.empty((M, N), device="cuda"))
        lg.lg_matmul_t(Ad2[1], Bd2[1], out[1], trans_a=ta, trans_b=tb,
                       workspace=workspace(lg.lg_matmul_workspace_bytes(M, N, K))); sync()
        assert_close(out[1].cpu().numpy(), ref, K, f"matmul_t {ta, tb} with {which} 4 bytes off alignment")


def test_other_ops_misaligned_operands(lg, lgo):
    I, Kf = si.conv2d_inputs(151, 2, 20, 20, 32, 64, 3, 3)
    ref = lgo.conv2d_nhwc_hwcf(I, Kf)
    for which in range(3):
        ops = [shifted(I) if which == 0 else (None, dev(I)), shifted(Kf) if which == 1 else (None, dev(Kf)),
               shifted(ref, fill=7.0) if which == 2 else (None, torch.empty(ref.shape, device="cuda"))]
        lg.lg_conv2d_nhwc_hwcf(ops[0][1], ops[1][1], ops[2][1],
                               workspace=workspace(lg.lg_conv2d_workspace_bytes(2, 20, 20, 32, 3, 3, 64))); sync()
        assert_close(ops[2][1].cpu().numpy(), ref, 288, f"conv2d operand {which} misaligned")
    Id, Kd = si.dwconv2d_inputs(152, 2, 30, 30, 64, 3, 3)
    refd = lgo.dwconv2d_nhwc_hwc(Id, Kd)
    I1, K1 = si.dwconv1d_inputs(153, 2, 300, 128, 3)
    ref1 = lgo.dwconv1d_nwc_wc(I1, K1)
    for which in range(3):
        ops = [shifted(Id) if which == 0 else (None, dev(Id)), shifted(Kd) if which == 1 else (None, dev(Kd)),
               shifted(refd, fill=7.0) if which == 2 else (None, torch.empty(refd.shape, device="cuda"))]
        lg.lg_dwconv2d_nhwc_hwc(ops[0][1], ops[1][1], ops[2][1]); sync()
        assert_close(ops[2][1].cpu().numpy(), refd, 9, f"dwconv2d operand {which} misaligned")
        ops = [shifted(I1) if which == 0 else (None, dev(I1)), shifted(K1) if which == 1 else (None, dev(K1)),
               shifted(ref1, fill=7.0) if which == 2 else (None, torch.empty(ref1.shape, device="cuda"))]
        lg.lg_dwconv1d_nwc_wc(ops[0][1], ops[1][1], ops[2][1]); sync()
        assert_close(ops[2][1].cpu().numpy(), ref1, 3, f"dwconv1d operand {which} misaligned")
    X = si.uniform(154, 0, (2052, 1024), 0, 1)
    for mis_in, mis_out in ((True, False), (False, True), (True, True)):
        xin = shifted(X) if mis_in else (None, dev(X))
        rows = shifted(np.empty(2052, np.float32), fill=7.0) if mis_out else (None, torch.empty(2052, device="cuda"))
        cols = shifted(np.empty(1024, np.float32), fill=7.0) if mis_out else (None, torch.empty(1024, device="cuda"))
        xt = shifted(np.empty((1024, 2052), np.float32), fill=7.0) if mis_out else (None, torch.empty((1024, 2052), device="cuda"))
        xc = shifted(np.empty((2052, 1024), np.float32), fill=7.0) if mis_out else (None, torch.empty((2052, 1024), device="cuda"))
        lg.lg_reduce_rows(xin[1], rows[1])
        lg.lg_reduce_cols(xin[1], cols[1], workspace=workspace(lg.lg_reduce_cols_workspace_bytes(2052, 1024)))
        lg.lg_transpose(xin[1], xt[1])
        lg.lg_copy2d(xin[1], xc[1]); sync()
        assert_close(rows[1].cpu().numpy(), lgo.reduce_rows(X), 1024, "reduce_rows misaligned")
        assert_close(cols[1].cpu().numpy(), lgo.reduce_cols(X), 2052, "reduce_cols misaligned")
        assert np.array_equal(bits(xt[1].cpu().numpy()), bits(lgo.transpose(X)))
        assert np.array_equal(bits(xc[1].cpu().numpy()), bits(X))
        if mis_out:
            for b, n in ((rows[0], 2052), (cols[0], 1024), (xt[0], 2052 * 1024), (xc[0], 2052 * 1024)):
                h = b.cpu().numpy()
                assert h[0] == 7.0 and np.all(h[1 + n:] == 7.0)


# ------------------------------------------------------------------------------- non-finite values

def assert_same_nonfinite(got, ref, K, what):
    """NaNs and infinities land exactly where the definition puts them (zero padding of ragged tiles
    must never meet an infinity); everything else meets the usual bar."""
    got, ref = np.asarray(got), np.asarray(ref)
    assert np.array_equal(np.isnan(got), np.isnan(ref)), f"{what}: NaN positions differ"
    inf = np.isinf(ref)
    assert np.array_equal(np.isinf(got), inf) and np.array_equal(got[inf], ref[inf]), f"{what}: infinities differ"
    fin = np.isfinite(ref)
    assert_close(np.where(fin, got, 0), np.where(fin, ref, 0), K, what)


@pytest.mark.parametrize("M,N,K", [(70, 50, 30), (300, 260, 1001), (130, 129, 64)])
def test_matmul_propagates_nonfinite_values(lg, lgo, M, N, K):
    A, B = si.matmul_inputs(160, M, N, K)
    A[3, K - 1] = np.inf            # last k of a ragged slice
    A[M - 1, 0] = np.nan            # last row of a ragged tile
    B[K - 1, N - 1] = -np.inf       # last column
    A[5, 2] = np.inf; A[5, 7] = -np.inf        # +inf and -inf in one row: NaN wherever both count
    ref = lgo.matmul(A, B)
    assert np.isnan(ref).any() and np.isinf(ref).any() and np.isfinite(ref).any()
    assert_same_nonfinite(run_matmul(lg, A, B), ref, K, "matmul")
    for v in range(lg.lg_gemm_variants()):
        out = Guarded((M, N))
        lg.lg_matmul_variant(dev(A), dev(B), out.t, v); sync(); out.check()
        assert_same_nonfinite(out.host(), ref, K, f"matmul variant {v}")


def test_other_ops_propagate_nonfinite_values(lg, lgo):
    I, Kf = si.conv2d_inputs(161, 2, 11, 13, 6, 10, 3, 3)
    I[1, 10, 12, 5] = np.inf; I[0, 0, 0, 0] = np.nan; Kf[2, 2, 5, 9] = -np.inf
    assert_same_nonfinite(run_conv(lg, I, Kf), lgo.conv2d_nhwc_hwcf(I, Kf), 54, "conv2d")
    Id, Kd = si.dwconv2d_inputs(162, 2, 9, 21, 68, 3, 3)
    Id[1, 8, 20, 67] = np.inf; Id[0, 4, 4, 1] = np.nan; Kd[0, 0, 3] = -np.inf
    out = Guarded((2, 7, 19, 68))
    lg.lg_dwconv2d_nhwc_hwc(dev(Id), dev(Kd), out.t); sync(); out.check()
    assert_same_nonfinite(out.host(), lgo.dwconv2d_nhwc_hwc(Id, Kd), 9, "dwconv2d")
    X = si.uniform(163, 0, (523, 1031), 0, 1)
    X[0, 1030] = np.inf; X[522, 0] = np.nan; X[7, 5] = -np.inf; X[9, 5] = np.inf
    rows, cols = Guarded((523,)), Guarded((1031,))
    lg.lg_reduce_rows(dev(X), rows.t)
    lg.lg_reduce_cols(dev(X), cols.t, workspace=workspace(lg.lg_reduce_cols_workspace_bytes(523, 1031))); sync()
    rows.check(); cols.check()
    assert_same_nonfinite(rows.host(), lgo.reduce_rows(X), 1031, "reduce_rows")
    assert_same_nonfinite(cols.host(), lgo.reduce_cols(X), 523, "reduce_cols")


# ------------------------------------------------------------------------------- calibration probes

@pytest.mark.parametrize("threads,unroll,hint", [(256, 1, 3), (256, 4, 0), (512, 2, 1), (1024, 8, 2), (1024, 1, 3)])
def test_stream_probe_moves_what_it_says(lg, threads, unroll, hint):
    n = 4 * (threads * unroll * 37 + 13)               # a ragged last workgroup
    x = si.uniform(140, 0, (n,), -1, 1)
    src = Guarded((n,), init=x)
    dst = Guarded((n,))
    lg.lg_stream_probe("copy", src.t, dst.t, threads=threads, unroll=unroll, hint=hint)
    sync(); dst.check(); src.check()
    assert np.array_equal(bits(dst.host()), bits(x))
    w = Guarded((n,))
    lg.lg_stream_probe("write", None, w.t, threads=threads, unroll=unroll, hint=hint)
    sync(); w.check()
    assert np.array_equal(w.host().reshape(-1, 4), np.tile(np.array([1, 2, 3, 4], np.float32), (n // 4, 1)))
    sink = Guarded((1024,), init=np.full(1024, 5.0, np.float32))
    lg.lg_stream_probe("read", src.t, sink.t, threads=threads, unroll=unroll, hint=hint)
    sync(); sink.check()
    assert np.all(sink.host() == 5.0)                   # finite input: the sink is never written
