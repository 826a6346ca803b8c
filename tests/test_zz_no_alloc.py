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
