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

    def run_all():
        lg.lg_matmul(A, B, C, workspace=ws_mm)
        lg.lg_conv2d_nhwc_hwcf(I, Kf, O, workspace=ws_cv)
        lg.lg_dwconv2d_nhwc_hwc(I, Kd, Od)
        lg.lg_reduce_rows(X, rows)
        lg.lg_reduce_cols(X, cols, workspace=ws_rc)
        lg.lg_transpose(X, Xt)

    outs = (C, O, Od, rows, cols, Xt)
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
