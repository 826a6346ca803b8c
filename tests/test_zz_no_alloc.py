"""The column reduction for callers that cannot allocate (lg_reduce_cols_static): through the C ABI,
its output must equal lg_reduce_cols' (same kernels, so bit for bit; and both within the fp32 bar of
the oracle) on two calls in a row, the second on a smaller input that leaves stale partial sums of
the first call in the library's device array."""
import numpy as np
import pytest
import torch

import seeded_inputs as si
from gpu_util import Guarded, assert_close, dev, workspace

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lg():
    import paper_2202_03293_amd as m
    m.lib()
    return m


def _both(lg, x, accumulate):
    R, Cn = x.shape
    xd = dev(x)
    init = si.uniform(9, 7, (Cn,), -1, 1) if accumulate else None
    a = Guarded((Cn,), init=init)
    b = Guarded((Cn,), init=init)
    lg.lg_reduce_cols(xd, a.t, accumulate=accumulate, workspace=workspace(lg.lg_reduce_cols_workspace_bytes(R, Cn)))
    lg.lg_reduce_cols_static(xd, b.t, accumulate=accumulate)
    torch.cuda.synchronize()
    a.check()
    b.check()
    return a.host(), b.host(), init


def test_static_matches_workspace_variant_on_two_calls_in_a_row(lg, lgo):
    # 4096 x 16384: 8 row chunks, 0.5 MiB of partial sums; then 1500 x 1000 (unaligned, fewer and
    # shorter partial rows: the array still holds the first call's sums beside and behind them)
    for case, (shape, accumulate) in enumerate((((4096, 16384), False), ((1500, 1000), True))):
        x = si.uniform(9, case, shape, 0, 1)
        assert lg.lg_reduce_cols_workspace_bytes(*shape) > 0, "the case must use the scratch array"
        ws_out, st_out, init = _both(lg, x, accumulate)
        assert np.array_equal(ws_out.view(np.uint32), st_out.view(np.uint32)), f"{shape}: outputs differ"
        ref = lgo.reduce_cols(x).astype(np.float64)
        if accumulate:
            ref = ref + init.astype(np.float64)
        assert_close(st_out, ref, shape[0], f"reduce_cols_static {shape}")


def test_static_single_launch_and_empty_cases(lg, lgo):
    x = si.uniform(9, 3, (100, 4098), 0, 1)                 # one launch, no partial sums
    ws_out, st_out, _ = _both(lg, x, False)
    assert np.array_equal(ws_out.view(np.uint32), st_out.view(np.uint32))
    assert_close(st_out, lgo.reduce_cols(x), 100, "reduce_cols_static 100x4098")
    out = Guarded((64,))
    lg.lg_reduce_cols_static(torch.empty((0, 64), device="cuda"), out.t)     # zero rows: the neutral element
    torch.cuda.synchronize()
    out.check()
    assert np.all(out.host() == 0.0)


def test_static_rejects_what_exceeds_its_array(lg):
    # 1024 row chunks x 1280 columns of partial sums = 5 MiB > 4 MiB: refused on the host before
    # anything is launched or dereferenced, so placeholder addresses will do
    import ctypes
    R, Cn = 1 << 20, 1280
    assert lg.lg_reduce_cols_workspace_bytes(R, Cn) > 4 << 20
    rc = lg.lib().lg_reduce_cols_static(ctypes.c_void_p(1 << 40), ctypes.c_void_p(1 << 20), R, Cn, Cn, 0, None)
    assert rc == -2


def test_static_recorded_into_a_graph_and_replayed(lg, lgo):
    """The callers it is for: recorded into a HIP graph (no allocation may happen there) and replayed with
    fresh inputs, eager work and synchronisations in between; every replay against the eager result bit for
    bit, the last one against the oracle."""
    R, Cn = 3000, 1000
    assert lg.lg_reduce_cols_workspace_bytes(R, Cn) > 0
    X = dev(si.uniform(9, 20, (R, Cn), 0, 1))
    out = torch.zeros(Cn, device="cuda")
    lg.lg_reduce_cols_static(X, out)              # first use on this device happens outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lg.lg_reduce_cols_static(X, out)
    for rep in range(3):
        x = si.uniform(9, 21 + rep, (R, Cn), 0, 1)
        X.copy_(dev(x))
        lg.lg_reduce_cols_static(X, out)
        torch.cuda.synchronize()
        eager = out.clone()
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {rep} differs from the eager run"
    assert_close(out.cpu().numpy(), lgo.reduce_cols(x), R, "reduce_cols_static replayed")


def test_static_first_use_inside_a_capture():
    """First call on the device while the stream is being captured (fresh process): the look-up of the
    device array's address is no stream operation and must not disturb the capture."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = r"""
import sys
sys.path.insert(0, %r)
import torch
import paper_2202_03293_amd as lg
X = torch.rand(3000, 1000, device="cuda")
out = torch.zeros(1000, device="cuda")
I = torch.rand(2, 26, 50, 64, device="cuda") - 0.5
K = torch.rand(3, 3, 64, device="cuda") - 0.5
O = torch.zeros(2, 24, 48, 64, device="cuda")
torch.cuda.synchronize()
g = torch.cuda.CUDAGraph()
with torch.cuda.graph(g):
    lg.lg_reduce_cols_static(X, out)
    lg.lg_dwconv2d_nhwc_hwc(I, K, O)                # the LDS-tile kernel, first use as well
out.zero_(); O.zero_()
torch.cuda.synchronize()
for _ in range(2):
    g.replay()
    torch.cuda.synchronize()
assert (out - X.double().sum(0).float()).abs().max().item() < 1e-4 * 3000 ** 0.5
ref = torch.nn.functional.conv2d(I.permute(0, 3, 1, 2).double(), K.permute(2, 0, 1).unsqueeze(1).double(), groups=64)
assert (O - ref.permute(0, 2, 3, 1).float()).abs().max().item() < 3e-4
print("capture-first ok")
""" % root
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=110)
    assert r.returncode == 0 and "capture-first ok" in r.stdout, r.stdout[-2000:] + r.stderr[-2000:]
