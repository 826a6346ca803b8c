"""The library only enqueues work: no allocation, no synchronisation, no host-side state per call.
So a sequence of calls can be recorded into a HIP graph and replayed.  The test records one call of
every op family, replays the graph several times with fresh inputs written into the same buffers
(eager work and synchronisations between replays), and checks every replay against the eager result
bit for bit (each op is deterministic) and against the CPU oracle."""
import numpy as np
import pytest
import torch

import seeded_inputs as si
from gpu_util import assert_close, dev, workspace

pytestmark = pytest.mark.gpu


def test_graph_replay_matches_eager_and_oracle(lgo):
    import paper_2202_03293_amd as lg
    lg.lib()
    M, N, K = 300, 260, 1000                   # split-k plan or not, edge tiles and a k tail
    A, B = dev(si.uniform(70, 0, (M, K), -1, 1)), dev(si.uniform(70, 1, (K, N), -1, 1))
    C = torch.zeros((M, N), device="cuda")
    ws_mm = workspace(lg.lg_matmul_workspace_bytes(M, N, K))
    I, Kf = dev(si.uniform(70, 2, (2, 20, 20, 32), -1, 1)), dev(si.uniform(70, 3, (3, 3, 32, 64), -1, 1))
    O = torch.zeros((2, 18, 18, 64), device="cuda")
    ws_cv = workspace(lg.lg_conv2d_workspace_bytes(2, 20, 20, 32, 3, 3, 64))
    Kd = dev(si.uniform(70, 4, (3, 3, 32), -1, 1))
    Od = torch.zeros((2, 18, 18, 32), device="cuda")
    X = dev(si.uniform(70, 5, (2100, 520), 0, 1))
    rows, cols = torch.zeros(2100, device="cuda"), torch.zeros(520, device="cuda")
    ws_rc = workspace(lg.lg_reduce_cols_workspace_bytes(2100, 520))
    Xt = torch.zeros((520, 2100), device="cuda")
    # the other entry points and the other GEMM kernels: transposed operand, the register-direct kernel
    # (a small product), matrix times one vector, 1-D convolutions, copy, batched transpose, long rows
    # cut into pieces
    Ct = torch.zeros((K, N), device="cuda")                      # A^T (K x M) times C-shaped (M x N)
    As, Cs = dev(si.uniform(70, 6, (64, 64), -1, 1)), torch.zeros((64, 64), device="cuda")
    Av, xv = dev(si.uniform(70, 7, (2048, 2048), -1, 1)), dev(si.uniform(70, 8, (2048, 1), -1, 1))
    yv = torch.zeros((2048, 1), device="cuda")
    I1, K1 = dev(si.uniform(70, 9, (2, 40, 32), -1, 1)), dev(si.uniform(70, 10, (3, 32, 64), -1, 1))
    O1 = torch.zeros((2, 38, 64), device="cuda")
    ws_c1 = workspace(lg.lg_conv1d_workspace_bytes(2, 40, 32, 3, 64))
    Kd1, Od1 = dev(si.uniform(70, 11, (3, 32), -1, 1)), torch.zeros((2, 38, 32), device="cuda")
    Xc = torch.zeros((2100, 520), device="cuda")
    Xb = torch.zeros(2100 * 520, device="cuda")                  # 4 x 5 transposes of 105 x 104 blocks... as a batch
    Xl, long_rows = dev(si.uniform(70, 12, (3, 40000), 0, 1)), torch.zeros(3, device="cuda")
    ws_rr = workspace(lg.lg_reduce_rows_workspace_bytes(3, 40000))

    def run_all():
        lg.lg_matmul(A, B, C, workspace=ws_mm)
        lg.lg_conv2d_nhwc_hwcf(I, Kf, O, workspace=ws_cv)
        lg.lg_dwconv2d_nhwc_hwc(I, Kd, Od)
        lg.lg_reduce_rows(X, rows)
        lg.lg_reduce_cols(X, cols, workspace=ws_rc)
        lg.lg_transpose(X, Xt)
        lg.lg_matmul_t(A, C, Ct, trans_a=True, workspace=workspace(0))
        lg.lg_matmul(As, As, Cs)
        lg.lg_matmul(Av, xv, yv)
        lg.lg_conv1d_nwc_wcf(I1, K1, O1, workspace=ws_c1)
        lg.lg_dwconv1d_nwc_wc(I1, Kd1, Od1)
        lg.lg_copy2d(X, Xc)
        lg.lg_transpose_batched(X.view(-1), Xb, 105, 104, 520, 105, 20, 5, (105 * 520, 104), (5 * 104 * 105, 104 * 105))
        lg.lg_reduce_rows_ws(Xl, long_rows, workspace=ws_rr)

    outs = (C, O, Od, rows, cols, Xt, Ct, Cs, yv, O1, Od1, Xc, Xb, long_rows)
    run_all()                                  # first use of each kernel happens outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run_all()
    for rep in range(3):
        A.copy_(dev(si.uniform(71 + rep, 0, (M, K), -1, 1)))
        I.copy_(dev(si.uniform(71 + rep, 2, (2, 20, 20, 32), -1, 1)))
        X.copy_(dev(si.uniform(71 + rep, 5, (2100, 520), 0, 1)))
        run_all()
        torch.cuda.synchronize()
        eager = [o.clone() for o in outs]
        for o in outs:
            o.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip(outs, eager):
            assert torch.equal(got, want), f"replay {rep} differs from the eager run"
    assert_close(C.cpu().numpy(), lgo.matmul(A.cpu().numpy(), B.cpu().numpy()), K, "graph matmul")
    assert_close(O.cpu().numpy(), lgo.conv2d_nhwc_hwcf(I.cpu().numpy(), Kf.cpu().numpy()), 288, "graph conv")
    assert_close(rows.cpu().numpy(), lgo.reduce_rows(X.cpu().numpy()), 520, "graph reduce_rows")
    assert np.array_equal(Xt.cpu().numpy().view(np.uint32), lgo.transpose(X.cpu().numpy()).view(np.uint32))


def test_ops_run_on_the_stream_they_are_given(lgo):
    """Two side streams, each with several milliseconds of other work queued ahead of the library
    calls and the operands produced on that stream right before them, no synchronisation until the
    end.  A call that ran anywhere but on its stream (or that synchronised or kept state shared with
    the other stream's calls) would read operands that are not there yet."""
    import paper_2202_03293_amd as lg
    lg.lib()
    M, N, K = 784, 512, 4608                   # the planner splits k here: two kernels and a workspace
    assert lg.lg_matmul_plan(M, N, K)[2] > 1
    R, Cn = 4100, 1028                         # column reduction in chunks: two kernels and a workspace
    hA, hB = si.uniform(80, 0, (M, K), -1, 1), si.uniform(80, 1, (K, N), -1, 1)
    hX = si.uniform(80, 2, (R, Cn), 0, 1)
    srcA, srcB, srcX = dev(hA), dev(hB), dev(hX)
    big = torch.rand((6144, 6144), device="cuda")
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    results = []
    for s in streams:
        with torch.cuda.stream(s):
            busy = big @ big                   # keeps the stream busy while the calls below are enqueued
            A, B, X = torch.zeros_like(srcA), torch.zeros_like(srcB), torch.zeros_like(srcX)
            A.add_(srcA); B.add_(srcB); X.add_(srcX)
            C = torch.full((M, N), float("nan"), device="cuda")
            cols, rows = torch.full((Cn,), float("nan"), device="cuda"), torch.full((R,), float("nan"), device="cuda")
            Xt = torch.zeros((Cn, R), device="cuda")
            ws_mm = workspace(lg.lg_matmul_workspace_bytes(M, N, K))
            ws_rc = workspace(lg.lg_reduce_cols_workspace_bytes(R, Cn))
            lg.lg_matmul(A, B, C, workspace=ws_mm, stream=s)
            lg.lg_reduce_cols(X, cols, workspace=ws_rc, stream=s)
            lg.lg_reduce_rows(X, rows, stream=s)
            lg.lg_transpose(X, Xt, stream=s)
            results.append((busy, A, B, X, C, cols, rows, Xt, ws_mm, ws_rc))
    for s in streams:
        s.synchronize()
    refC, refcols, refrows = lgo.matmul(hA, hB), lgo.reduce_cols(hX), lgo.reduce_rows(hX)
    for _, _, _, _, C, cols, rows, Xt, _, _ in results:
        assert_close(C.cpu().numpy(), refC, K, "matmul on a side stream")
        assert_close(cols.cpu().numpy(), refcols, R, "reduce_cols on a side stream")
        assert_close(rows.cpu().numpy(), refrows, Cn, "reduce_rows on a side stream")
        assert np.array_equal(Xt.cpu().numpy().view(np.uint32), lgo.transpose(hX).view(np.uint32))


def test_first_use_of_a_kernel_inside_a_capture():
    """A caller may record a graph before it has ever launched anything: the one-time set-up a
    kernel needs on first use (its dynamic LDS limit) must work under stream capture too.  Runs in
    a fresh process, where no kernel of the library has been launched yet."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = r"""
import sys
sys.path.insert(0, %r)
import torch
import paper_2202_03293_amd as lg
A = torch.rand(512, 2048, device="cuda") - 0.5
B = torch.rand(2048, 1024, device="cuda") - 0.5
C = torch.zeros(512, 1024, device="cuda")
X = torch.rand(300, 520, device="cuda")
Xt = torch.zeros(520, 300, device="cuda")
cols = torch.zeros(520, device="cuda")
ws = torch.empty(max(lg.lg_matmul_workspace_bytes(512, 1024, 2048) // 4, 1), device="cuda")
wc = torch.empty(max(lg.lg_reduce_cols_workspace_bytes(300, 520) // 4, 1), device="cuda")
torch.cuda.synchronize()
g = torch.cuda.CUDAGraph()
with torch.cuda.graph(g):
    for v in range(lg.lg_gemm_variants()):          # every kernel of the menu, first use
        lg.lg_matmul_variant(A, B, C, v)
    lg.lg_matmul(A, B, C, workspace=ws)
    lg.lg_transpose(X, Xt)
    lg.lg_reduce_cols(X, cols, workspace=wc)
C.zero_(); Xt.zero_(); cols.zero_()
torch.cuda.synchronize()
g.replay()
torch.cuda.synchronize()
ref = (A.double() @ B.double()).float()
assert (C - ref).abs().max().item() < 1e-4 * 2048 ** 0.5, (C - ref).abs().max().item()
assert torch.equal(Xt, X.t().contiguous())
assert (cols - X.double().sum(0).float()).abs().max().item() < 1e-4 * 300 ** 0.5
print("capture-first ok")
""" % root
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=110)
    assert r.returncode == 0 and "capture-first ok" in r.stdout, r.stdout[-2000:] + r.stderr[-2000:]


def test_tile_loop_in_a_graph(lgo):
    """The GEMM's tile loop (several output tiles per workgroup, the planner's choice for a short contraction
    with a large output) recorded once and replayed with fresh operands: every replay equals the eager call
    bit for bit, and sampled rows equal the oracle."""
    import paper_2202_03293_amd as lg
    lg.lib()
    M, N, K = 3072, 3072, 64
    assert lg.lg_matmul_plan_tile_loop(M, N, K)
    A, B = torch.zeros((M, K), device="cuda"), torch.zeros((K, N), device="cuda")
    C, Ce = torch.zeros((M, N), device="cuda"), torch.zeros((M, N), device="cuda")
    g = torch.cuda.CUDAGraph()
    lg.lg_matmul(A, B, C)                       # first use outside the capture
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        lg.lg_matmul(A, B, C)
    rows = np.r_[0:8, 127:130, 1530:1540, M - 5:M]
    for rep in range(3):
        hA, hB = si.matmul_inputs(80 + rep, M, N, K, case=rep)
        A.copy_(dev(hA)); B.copy_(dev(hB))
        C.fill_(float("nan")); Ce.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        lg.lg_matmul(A, B, Ce)                  # eager, behind the replay on the same stream
        torch.cuda.synchronize()
        assert torch.equal(C, Ce), f"replay {rep} differs from the eager call"
        ref = lgo.matmul(hA[rows], hB)
        assert_close(C[torch.as_tensor(rows, device="cuda")].cpu().numpy(), ref, K, f"tile loop in a graph, replay {rep}")
