"""Helpers for the GPU parity tests: device buffers with guard bands, error metrics."""
import math

import numpy as np
import torch

CANARY = 0x7FA5A5A5          # a NaN pattern: any stray write or read of the guard band shows


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


class Guarded:
    """A device tensor of `shape` surrounded by canary words; check() proves nothing leaked."""

    def __init__(self, shape, init=None, pad=1024):
        n = int(np.prod(shape))
        self.pad, self.n = pad, n
        self.buf = torch.full((n + 2 * pad,), CANARY, dtype=torch.int32, device="cuda")
        self.t = self.buf[pad:pad + n].view(torch.float32).view(*shape)
        if init is not None:
            self.t.copy_(dev(init))

    def host(self):
        return self.t.cpu().numpy()

    def check(self):
        b = self.buf.cpu().numpy()
        assert np.all(b[:self.pad] == CANARY) and np.all(b[self.pad + self.n:] == CANARY), \
            "write outside the output buffer"


def workspace(nbytes):
    if nbytes == 0:
        return None
    return torch.empty((nbytes + 3) // 4, dtype=torch.float32, device="cuda")


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


def assert_close(got, ref, K, what=""):
    """The parity bar for fp32 ops: max |err| <= 1e-4*sqrt(K) and relative Frobenius <= 1e-5."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, f"{what}: shape {got.shape} vs {ref.shape}"
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    err = np.abs(got - ref)
    max_err = float(err.max()) if err.size else 0.0
    bound = 1e-4 * math.sqrt(max(K, 1))
    assert max_err <= bound, f"{what}: max abs err {max_err:.3e} > {bound:.3e}"
    den = float(np.linalg.norm(ref.ravel()))
    if den > 0:
        rel = float(np.linalg.norm((got - ref).ravel())) / den
        assert rel <= 1e-5, f"{what}: relative Frobenius err {rel:.3e} > 1e-5"
