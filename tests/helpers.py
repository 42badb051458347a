"""Shared plumbing of the GPU parity tests: moving bitsets between numpy and torch, comparing
sign vectors up to near ties.  No arithmetic of the method lives here."""
import numpy as np
import torch

TIE_TOL = 1e-6     # a sign may differ only where |value| < TIE_TOL * max|value| (f32 path)
C_RTOL = 1e-5      # coefficient tolerance
ID_RTOL = 1e-6     # Frobenius identity tolerance
CURVE_RTOL = 1e-3  # ||R_w||_F / ||A||_F curve tolerance


def to_dev_bits(bits: np.ndarray, device="cuda") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits, dtype=np.uint64).view(np.int64)).to(device)


def to_np_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy().view(np.uint64)


def dense(bits, n):
    b = np.asarray(bits, dtype=np.uint64).reshape(-1)
    idx = np.arange(n)
    return 1.0 - 2.0 * ((b[idx // 64] >> (idx % 64).astype(np.uint64)) & np.uint64(1)).astype(np.float64)


def sign_mismatch(bits_a, bits_b, n):
    """Indices at which two bitsets of length n differ."""
    return np.nonzero(dense(bits_a, n) != dense(bits_b, n))[0]


def assert_signs_match(bits_gpu, bits_ref, values_ref, n, what, tol=TIE_TOL):
    """Signs must be identical except where the reference value is within tol of a tie."""
    bad = sign_mismatch(bits_gpu, bits_ref, n)
    if bad.size:
        v = np.abs(np.asarray(values_ref, dtype=np.float64))
        lim = tol * v.max()
        worst = v[bad].max()
        assert worst < lim, f"{what}: {bad.size} sign(s) differ, largest |value| {worst:.3e} >= tie limit {lim:.3e}"
    # padding bits clear
    nw = (n + 63) // 64
    g = np.asarray(bits_gpu, dtype=np.uint64).reshape(-1)[:nw]
    if n % 64:
        assert int(g[-1]) >> (n % 64) == 0, f"{what}: padding bits set"
    return bad.size
