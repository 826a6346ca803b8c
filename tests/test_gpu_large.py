"""Maximum-size cases on the GPU: tensors past 2^31 elements or 2^31 bytes, where 32-bit index or
offset arithmetic anywhere in a kernel would go wrong.  Inputs are built on the device (index
patterns for data movement, ones with a marker for the reductions, seeded torch randoms for the
contractions); the contractions are checked against the CPU oracle on sampled row blocks / images
copied back to the host, the rest against what the definition fixes exactly."""
import numpy as np
import pytest
import torch

from gpu_util import assert_close, workspace

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lg():
    import paper_2202_03293_amd as pkg
    pkg.lib()
    return pkg


def sync():
    torch.cuda.synchronize()


def test_copy_and_transpose_past_2_31_elements(lg):
    R, Cn = 46400, 46400                       # 2.15e9 elements, 8.6 GB per tensor; ragged 128x128 tiles
    assert R * Cn > 2 ** 31
    ri = torch.arange(R, dtype=torch.int32, device="cuda")
    cj = torch.arange(Cn, dtype=torch.int32, device="cuda")
    x = ri[:, None] * 48271 + cj[None, :]      # int32 pattern, wraps; distinct along rows and columns
    out = torch.empty((Cn, R), dtype=torch.int32, device="cuda")
    lg.lg_transpose(x.view(torch.float32), out.view(torch.float32)); sync()
    for j0 in range(0, Cn, 8192):              # compare in slabs: out[j, i] = x[i, j], bit for bit
        j1 = min(Cn, j0 + 8192)
        expect = cj[j0:j1, None] + ri[None, :] * 48271
        assert torch.equal(out[j0:j1], expect), f"transpose rows {j0}..{j1}"
    del expect
    out2 = out.view(-1)[: R * Cn].view(R, Cn)
    out2.fill_(-1)
    lg.lg_copy2d(x.view(torch.float32), out2.view(torch.float32)); sync()
    assert torch.equal(out2, x)


def test_reduce_rows_past_2_31_elements(lg):
    R, Cn = 70000, 32768                       # 2.29e9 elements, 9.2 GB: row offsets pass 2^31 elements
    assert R * Cn > 2 ** 31
    x = torch.ones((R, Cn), device="cuda")
    x[R - 1, Cn - 1] = 3.0
    x[R - 7, 5] = 9.0
    out = torch.full((R,), float("nan"), device="cuda")
    lg.lg_reduce_rows(x, out); sync()
    expect = np.full(R, float(Cn), np.float32)  # integer partial sums below 2^24: exact
    expect[R - 1] += 2
    expect[R - 7] += 8
    assert np.array_equal(out.cpu().numpy(), expect)


def test_reduce_cols_past_2_31_elements(lg):
    R, Cn = 2_100_000, 1028
    assert R * Cn > 2 ** 31
    x = torch.ones((R, Cn), device="cuda")     # 8.6 GB
    x[R - 1, Cn - 1] = 3.0
    out = torch.full((Cn,), float("nan"), device="cuda")
    lg.lg_reduce_cols(x, out, workspace=workspace(lg.lg_reduce_cols_workspace_bytes(R, Cn))); sync()
    expect = np.full(Cn, float(R), np.float32)
    expect[-1] += 2
    assert np.array_equal(out.cpu().numpy(), expect)


def test_matmul_operand_past_2_31_bytes(lg, lgo):
    M, N, K = 2 ** 23 + 64, 64, 64             # A and C are 2.1 GB each
    g = torch.Generator(device="cuda").manual_seed(7)
    A = torch.rand((M, K), device="cuda", generator=g) * 2 - 1
    B = torch.rand((K, N), device="cuda", generator=g) * 2 - 1
    C = torch.full((M, N), float("nan"), device="cuda")
    lg.lg_matmul(A, B, C, workspace=workspace(lg.lg_matmul_workspace_bytes(M, N, K))); sync()
    Bh = B.cpu().numpy()
    for m0 in (0, 2 ** 22 - 32, 2 ** 23 - 64, M - 128):      # around and past the 2^31-byte mark
        ref = lgo.matmul(np.ascontiguousarray(A[m0:m0 + 128].cpu().numpy()), Bh)
        assert_close(C[m0:m0 + 128].cpu().numpy(), ref, K, f"matmul rows {m0}..")
    assert bool(torch.isfinite(C).all())


# C = 128: every k-slice stays inside one filter tap (scalar tap walk); C = 24: slices straddle taps
# (per-lane walk).  F = 64 so that whole tiles exist and the global->LDS transfer path runs.
@pytest.mark.parametrize("N,H,W,C", [(66, 258, 258, 128), (66, 600, 600, 24)])
def test_conv_input_past_2_31_bytes(lg, lgo, N, H, W, C):
    F, KH, KW = 64, 3, 3
    assert N * H * W * C * 4 > 2 ** 31
    g = torch.Generator(device="cuda").manual_seed(8)
    I = torch.rand((N, H, W, C), device="cuda", generator=g) * 2 - 1
    Kf = torch.rand((KH, KW, C, F), device="cuda", generator=g) * 2 - 1
    O = torch.full((N, H - 2, W - 2, F), float("nan"), device="cuda")
    lg.lg_conv2d_nhwc_hwcf(I, Kf, O, workspace=workspace(lg.lg_conv2d_workspace_bytes(N, H, W, C, KH, KW, F))); sync()
    Kh = Kf.cpu().numpy()
    for n in (0, N - 1):                       # the last image lies wholly past the 2^31-byte mark
        ref = lgo.conv2d_nhwc_hwcf(np.ascontiguousarray(I[n:n + 1].cpu().numpy()), Kh)
        assert_close(O[n:n + 1].cpu().numpy(), ref, KH * KW * C, f"conv image {n}")
    assert bool(torch.isfinite(O).all())


def test_matmul_with_rows_256_mib_apart(lg, lgo):
    """A small problem whose A rows are 2^26 floats apart (a 12.9 GB allocation): the planner's pick for
    the extents is the register-direct kernel, whose 32-bit offsets do not reach that far, so the
    call must run on the tiled kernel's 64-bit path instead; forcing the direct kernel is refused."""
    M, N, K, lda = 48, 40, 72, 2 ** 26
    assert lg.lg_matmul_plan(M, N, K)[0] == 16
    g = torch.Generator(device="cuda").manual_seed(9)
    buf = torch.empty((M, lda), device="cuda")
    A = buf[:, :K]
    A.copy_(torch.rand((M, K), device="cuda", generator=g) * 2 - 1)
    B = torch.rand((K, N), device="cuda", generator=g) * 2 - 1
    C = torch.full((M, N), float("nan"), device="cuda")
    lg.lg_matmul(A, B, C); sync()
    ref = lgo.matmul(np.ascontiguousarray(A.cpu().numpy()), B.cpu().numpy())
    assert_close(C.cpu().numpy(), ref, K, "matmul with lda = 2^26")
    direct = next(v for v in range(lg.lg_gemm_variants()) if lg.lg_gemm_variant_info(v)[0] == 16)
    with pytest.raises(lg.LgError) as e:
        lg.lg_matmul_variant(A, B, C, direct)
    assert e.value.status == -2          # LG_ERR_UNSUPPORTED


def test_first_layer_conv_many_rounds_of_small_blocks(lg, lgo):
    """Three input channels, 3x3 filter: a contraction of 27, which the planner gives to the
    register-direct kernel on its one-float path -- here as 25 000 blocks, many rounds of the chip.
    The first and the last image are checked against the oracle element by element."""
    N, H, W, C, F = 8, 226, 226, 3, 32
    assert lg.lg_matmul_plan(N * 224 * 224, F, 27)[0] == 16
    g = torch.Generator(device="cuda").manual_seed(10)
    I = torch.rand((N, H, W, C), device="cuda", generator=g) * 2 - 1
    Kf = torch.rand((3, 3, C, F), device="cuda", generator=g) * 2 - 1
    O = torch.full((N, 224, 224, F), float("nan"), device="cuda")
    lg.lg_conv2d_nhwc_hwcf(I, Kf, O); sync()
    Kh = Kf.cpu().numpy()
    for n in (0, N - 1):
        ref = lgo.conv2d_nhwc_hwcf(np.ascontiguousarray(I[n:n + 1].cpu().numpy()), Kh)
        assert_close(O[n:n + 1].cpu().numpy(), ref, 27, f"conv image {n}")
    assert bool(torch.isfinite(O).all())
