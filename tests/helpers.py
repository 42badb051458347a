"""Shared plumbing of the GPU parity tests: moving bitsets between numpy and torch, comparing
sign vectors up to near ties.  No arithmetic of the method lives here."""
import numpy as np
import torch

TIE_TOL = 1e-6     # a sign may differ only where |value| < TIE_TOL * max|value| (f32 path)
STOP_TOL = 1e-7    # the stop test c_j <= c_{j-1} may go the other way only where |c_j - c_{j-1}| <= STOP_TOL |c_j|
TIE_TOL_F64, STOP_TOL_F64 = 1e-12, 1e-13   # the same for f64 inputs (f64 sums in another order)
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


def tie_tolerances(f32):
    return (TIE_TOL, STOP_TOL) if f32 else (TIE_TOL_F64, STOP_TOL_F64)


def adoption_bound(decisions, f32):
    """Most terms that may differ from the literal run of Algorithm 4.  An f32 sum of a row carries about
    1e-7 max|value| of rounding error, and the entries of a decision vector have density about 3.2 near zero
    (relative to their maximum, Gaussian-like sums): 3.2e-7 expected deviations per sign decision."""
    return 3 + 3 * 3.2e-7 * decisions if f32 else 1


def match_matrix_term(oracle, R, t0, s_gpu, t_gpu, iters_gpu, f32, what):
    """The GPU's term must be an outcome of Algorithm 4 from (R, t_0): the literal one, or one reached by
    taking only near-tie decisions the other way (signs within TIE_TOL of a tie, stop tests within STOP_TOL).
    Returns (number of such decisions on the way, the literal run)."""
    g = oracle.greedy_signed_cut(R, t0)
    if np.array_equal(g["s"], s_gpu) and np.array_equal(g["t"], t_gpu) and int(iters_gpu) == g["iters"]:
        return 0, g
    tol, tol_c = tie_tolerances(f32)
    r = oracle.greedy_signed_cut_near_ties(
        R, t0, tol, tol_c, max_runs=96,
        accept=lambda o: o["iters"] == int(iters_gpu) and np.array_equal(o["s"], s_gpu) and np.array_equal(o["t"], t_gpu))
    assert r["accepted"] is not None, (
        f"{what}: the GPU's term ({int(iters_gpu)} alternations) is none of the {len(r['outcomes'])} outcomes of "
        f"Algorithm 4 within the tie tolerance (oracle: {g['iters']} alternations, margins {g['margin']}, "
        f"search truncated: {r['truncated']})")
    return r["outcomes"][r["accepted"]]["flips"], g


def match_tensor_term(oracle, r, start, signs_gpu, iters_gpu, f32, what, modes=None):
    """The same for Algorithm 12; `modes`: how many leading modes' sign vectors the GPU reports (default all)."""
    modes = len(start) if modes is None else modes
    same = lambda sg: all(np.array_equal(sg[i], signs_gpu[i]) for i in range(modes))
    g = oracle.axial_greedy_cut(r, start)
    if same(g["signs"]) and int(iters_gpu) == g["iters"]:
        return 0, g
    tol, tol_c = tie_tolerances(f32)
    res = oracle.axial_greedy_cut_near_ties(r, start, tol, tol_c, max_runs=96,
                                            accept=lambda o: o["iters"] == int(iters_gpu) and same(o["signs"]))
    assert res["accepted"] is not None, (
        f"{what}: the GPU's term ({int(iters_gpu)} sweeps) is none of the {len(res['outcomes'])} outcomes of "
        f"Algorithm 12 within the tie tolerance (oracle: {g['iters']} sweeps, margins {g['margin']}, "
        f"search truncated: {res['truncated']})")
    return res["outcomes"][res["accepted"]]["flips"], g
