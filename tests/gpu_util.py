"""Helpers for the GPU parity tests: guarded device buffers and the tolerance rule."""
import numpy as np
import torch

DEV = "cuda:0"
GUARD = 64          # floats of canary on each side of every output buffer
CANARY = -7.25e37


def have_gpu():
    return torch.cuda.is_available()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


class Guarded:
    """Output buffer with canaries on both sides; `check()` fails on any out-of-range write."""

    def __init__(self, n):
        self.full = torch.full((n + 2 * GUARD,), CANARY, dtype=torch.float32, device=DEV)
        self.t = self.full[GUARD:GUARD + n]
        self.n = n

    def check(self):
        torch.cuda.synchronize()
        f = self.full.cpu().numpy()
        assert (f[:GUARD] == np.float32(CANARY)).all() and (f[GUARD + self.n:] == np.float32(CANARY)).all(), \
            "kernel wrote outside its output buffer"
        return f[GUARD:GUARD + self.n].copy()


def tol(ref, K):
    """spec tolerance for fp32 FMA reductions of length K."""
    return 1e-4 * (np.sqrt(K) * float(np.abs(ref).max()) + 1.0)


def assert_close(got, ref, K, what=""):
    assert got.shape == ref.shape, (got.shape, ref.shape)
    err = float(np.abs(got.astype(np.float64) - ref.astype(np.float64)).max())
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    assert err <= tol(ref, K), f"{what}: max |gpu-ref| = {err:.3e} > tol {tol(ref, K):.3e}"
    return err


def assert_bits(got, ref, what=""):
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), f"{what}: not bit-exact"


def dev8(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).to(DEV)


class Guarded8:
    """uint8 output buffer (16-byte aligned start) with canaries on both sides and a canary fill inside,
    so both stray writes and bytes never written show."""

    def __init__(self, n):
        self.full = torch.full((n + 2 * GUARD,), 0xA5, dtype=torch.uint8, device=DEV)
        self.t = self.full[GUARD:GUARD + n]
        self.n = n

    def check(self):
        torch.cuda.synchronize()
        f = self.full.cpu().numpy()
        assert (f[:GUARD] == 0xA5).all() and (f[GUARD + self.n:] == 0xA5).all(), "kernel wrote outside its output buffer"
        return f[GUARD:GUARD + self.n].copy()
