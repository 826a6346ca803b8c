"""Host-side checks of the C ABI that need no GPU: the library loads, exports what the header
declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "lg.h")


@pytest.fixture(scope="module")
def L():
    from paper_2202_03293_amd import ops
    if not os.path.exists(ops.LIB_PATH):
        from paper_2202_03293_amd import build
        build.build()
    return ops.lib()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lg_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported_and_bound(L):
    from paper_2202_03293_amd import ops
    names = declared_symbols()
    assert "lg_matmul" in names and "lg_transpose" in names and len(names) >= 14
    for n in names:
        assert hasattr(L, n), f"{n} declared in lg.h but not exported"
    assert sorted(ops.exported_symbols()) == names
    import paper_2202_03293_amd as pkg
    for n in names:
        assert hasattr(pkg, n), f"python binding lacks {n}"


def test_version_status_and_extent(L):
    assert L.lg_version() == 100
    assert L.lg_status_string(0) == b"LG_OK"
    assert L.lg_status_string(-1) == b"LG_ERR_INVALID_ARG"
    assert L.lg_status_string(-3) == b"LG_ERR_WORKSPACE"
    assert L.lg_conv_out_extent(58, 3, 1, 1) == 56
    assert L.lg_conv_out_extent(56, 1, 2, 1) == 28
    assert L.lg_conv_out_extent(4, 3, 1, 2) == 0


def test_argument_validation_without_device(L):
    P = ctypes.c_void_p(4096)      # never dereferenced: every call below fails validation first
    Q = ctypes.c_void_p(1 << 30)
    assert L.lg_matmul(P, P, Q, -1, 4, 4, 4, 4, 4, 0, None, 0, None) == -1
    assert L.lg_matmul(P, P, Q, 4, 4, 4, 3, 4, 4, 0, None, 0, None) == -1      # lda < K
    assert L.lg_matmul(P, P, Q, 4, 4, 4, 4, 4, 3, 0, None, 0, None) == -1      # ldc < N
    assert L.lg_matmul(None, P, Q, 4, 4, 4, 4, 4, 4, 0, None, 0, None) == -1
    assert L.lg_matmul(P, P, P, 4, 4, 4, 4, 4, 4, 0, None, 0, None) == -1      # A aliases C
    assert L.lg_matmul(P, P, Q, 0, 4, 4, 4, 4, 4, 0, None, 0, None) == 0       # empty output
    assert L.lg_matmul_t(P, P, Q, 4, 4, 8, 3, 4, 4, 1, 0, 0, None, 0, None) == -1   # A stored K x M: lda < M
    assert L.lg_matmul_t(P, P, Q, 4, 4, 8, 4, 4, 4, 0, 1, 0, None, 0, None) == -1   # B stored N x K: ldb < K
    assert L.lg_matmul_t(P, P, Q, 4, 4, 8, 4, 8, 4, 1, 1, 0, None, 0, None) == -2   # both transposed
    assert L.lg_conv2d_nhwc_hwcf(P, P, Q, 1, 2, 2, 4, 3, 3, 4, 1, 1, 1, 1, 0, None, 0, None) == -1  # window too big
    assert L.lg_conv2d_nhwc_hwcf(P, P, Q, 1, 8, 8, 4, 3, 3, 4, 0, 1, 1, 1, 0, None, 0, None) == -1  # stride 0
    assert L.lg_dwconv1d_nwc_wc(P, P, Q, 1, 8, 4, 3, 1, 0, 0, None) == -1                           # dilation 0
    assert L.lg_dwconv2d_nhwc_hwc(P, P, Q, 1, 2, 8, 4, 3, 3, 1, 1, 1, 1, 0, None) == -1
    assert L.lg_reduce_rows(P, Q, 4, 8, 7, 0, None) == -1
    assert L.lg_reduce_cols(P, Q, 4, 8, 7, 0, None, 0, None) == -1
    assert L.lg_reduce_cols(P, Q, 4096, 64, 64, 0, None, 0, None) == -3        # needs a workspace
    assert L.lg_reduce_cols_static(P, Q, 4, 8, 7, 0, None) == -1
    assert L.lg_reduce_cols_static(ctypes.c_void_p(1 << 40), Q, 1 << 20, 1280, 1280, 0, None) == -2   # 5 MiB of partial sums
    assert L.lg_transpose(P, Q, 4, 8, 8, 3, None) == -1                        # ld_out < R
    assert L.lg_transpose(P, P, 4, 4, 4, 4, None) == -1                        # in place
    assert L.lg_copy2d(P, Q, 4, 8, 7, 8, None) == -1
    assert L.lg_transpose(P, Q, 0, 8, 8, 8, None) == 0
    n = L.lg_mfma_probe_out_elems()
    assert n == 512 * 256
    assert L.lg_mfma_probe(None, n, 10, None) == -1                            # no buffer
    assert L.lg_mfma_probe(P, n - 1, 10, None) == -1                           # short buffer
    assert L.lg_mfma_probe(P, n, -1, None) == -1
    assert L.lg_mfma_probe(P, n, (1 << 22) + 1, None) == -1
    assert L.lg_mfma_probe_flops(1) == 512 * 4 * 4 * 4096.0                    # groups x waves x chains x flops per MFMA
    assert L.lg_mfma_probe_flops(-5) == 0.0
    assert L.lg_stream_probe(3, P, Q, 1024, 256, 1, 3, None) == -1                 # unknown mode
    assert L.lg_stream_probe(2, P, Q, 1022, 256, 1, 3, None) == -1                 # not whole 128-bit words
    assert L.lg_stream_probe(2, P, Q, 1024, 128, 1, 3, None) == -1                 # workgroup size not on the menu
    assert L.lg_stream_probe(2, P, Q, 1024, 256, 3, 3, None) == -1                 # unroll not on the menu
    assert L.lg_stream_probe(2, P, P, 1024, 256, 1, 3, None) == -1                 # copy onto itself
    assert L.lg_stream_probe(0, None, Q, 1024, 256, 1, 3, None) == -1
    assert L.lg_stream_probe(2, P, Q, 0, 256, 1, 3, None) == 0
    assert L.lg_conv1d_nwc_wcf(P, P, Q, 1, 4, 4, 3, 4, 1, 2, 0, None, 0, None) == -1   # dilated window too big
    assert L.lg_conv1d_nwc_wcf(P, P, Q, 1, 8, 4, 3, 4, 0, 1, 0, None, 0, None) == -1   # stride 0
    assert L.lg_conv1d_nwc_wcf(P, P, Q, 0, 8, 4, 3, 4, 1, 1, 0, None, 0, None) == 0    # empty batch
    assert L.lg_transpose_batched(P, Q, 4, 8, 8, 3, 2, 2, 32, 64, 32, 64, None) == -1  # ld_out < R
    assert L.lg_transpose_batched(P, Q, 4, 8, 8, 4, 2, 2, -1, 64, 32, 64, None) == -1  # negative stride
    assert L.lg_transpose_batched(P, P, 4, 4, 4, 4, 2, 1, 16, 0, 16, 0, None) == -1    # in place
    assert L.lg_transpose_batched(P, Q, 4, 4, 4, 4, 0, 1, 16, 0, 16, 0, None) == 0     # empty batch


def test_workspace_queries(L):
    assert L.lg_matmul_workspace_bytes(8192, 8192, 8192) == 0
    assert L.lg_matmul_workspace_bytes(0, 8, 8) == 0
    assert L.lg_reduce_cols_workspace_bytes(4096, 16384) > 0
    assert L.lg_reduce_cols_workspace_bytes(4096, 16384) <= 4096 * 16384 * 4 // 32   # << input
    assert L.lg_reduce_cols_workspace_bytes(64, 16384) == 0
    assert L.lg_conv1d_workspace_bytes(4, 100, 32, 3, 64, 2, 2) == \
        L.lg_conv2d_workspace_bytes(4, 1, 100, 32, 1, 3, 64, 1, 2, 1, 2)
    ws = L.lg_conv2d_workspace_bytes(8, 16, 16, 256, 3, 3, 256, 1, 1, 1, 1)
    assert ws % (8 * 14 * 14 * 256 * 4) == 0


def test_binding_fails_loudly_without_library(monkeypatch):
    from paper_2202_03293_amd import ops
    monkeypatch.setattr(ops, "_lib", None)
    monkeypatch.setattr(ops, "LIB_PATH", "/nonexistent/liblg.so")
    with pytest.raises(ImportError):
        ops.lib()


def test_bench_refuses_more_than_one_gpu():
    """The benchmark is a one-GPU program: asked for more it says so and exits before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
