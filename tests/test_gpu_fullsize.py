"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (default
workgroup count, register-tiled row pass): the first terms of each headline shape are checked
against the oracle term by term, later outputs by properties that hold at any size."""
import math

import numpy as np
import pytest
import torch

from helpers import C_RTOL, CURVE_RTOL, ID_RTOL, TIE_TOL, dense, to_np_bits
from test_gpu_parity import lockstep_check

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def scd():
    from paper_2410_01799_amd import scd as mod

    mod.lib()
    return mod


def run_case(scd, oracle, A, seed, w_check, w_total):
    m, n = A.shape
    A64 = A.astype(np.float64)
    Ad = torch.from_numpy(A).cuda()
    res = scd.scd_decompose(Ad, w_total, seed)
    S, T = to_np_bits(res["signs"][0]), to_np_bits(res["signs"][1])
    c = res["c"].cpu().numpy().astype(np.float64)
    trace = res["trace"].cpu().numpy()
    iters = res["iters"].cpu().numpy()
    assert res["status"] == 0
    # identity of Section 3.2 on every term of the whole run
    np.testing.assert_allclose(trace[1:] ** 2, trace[:-1] ** 2 - m * n * c ** 2, rtol=ID_RTOL)
    assert np.all(c > 0) and np.all(iters >= 2)
    # oracle in lockstep on the first terms
    curve, adopted = lockstep_check(oracle, A64, seed, S[:w_check], T[:w_check], c[:w_check], trace, iters,
                                    A.dtype == np.float32)
    np.testing.assert_allclose(trace[: w_check + 1] / trace[0], curve / curve[0], rtol=CURVE_RTOL)
    np.testing.assert_allclose(trace[: w_check + 1], curve, rtol=2e-5 if A.dtype == np.float32 else 1e-11)
    # the definition on the whole run: ||A - expand|| is the last trace value (f64 on the GPU)
    E = scd.scd_expand(res["signs"], res["c"], (m, n))
    resid = float((Ad.double() - E.double()).norm())
    assert resid == pytest.approx(trace[-1], rel=1e-4 if A.dtype == np.float32 else 1e-10)
    # sampled entries of the expansion, computed one by one
    rs = np.random.default_rng(0)
    Eh = E.cpu().numpy()
    for i, l in zip(rs.integers(0, m, 16).tolist(), rs.integers(0, n, 16).tolist()):
        acc = 0.0
        for j in range(w_total):
            sj = -1.0 if (int(S[j, i // 64]) >> (i % 64)) & 1 else 1.0
            tj = -1.0 if (int(T[j, l // 64]) >> (l % 64)) & 1 else 1.0
            acc += float(res["c"][j].item()) * sj * tj
        assert Eh[i, l] == np.asarray(acc, dtype=A.dtype)
    return res, adopted


def test_config2_f32_prefix(scd, oracle):
    from paper_2410_01799_amd import workloads

    A = workloads.gaussian_matrix(4096, 4096, 2, np.float32)
    res, _ = run_case(scd, oracle, A, seed=2, w_check=6, w_total=40)
    trace = res["trace"].cpu().numpy()
    # Figure 7 slope: ln r_k ~ -2.38e-4 k on 4096^2 N(0,1)
    slope = math.log(trace[-1] / trace[0]) / 40
    assert slope == pytest.approx(-2.3845e-4, rel=0.04)


def test_config2_f64_prefix(scd, oracle):
    from paper_2410_01799_amd import workloads

    A = workloads.gaussian_matrix(4096, 4096, 2, np.float64)
    run_case(scd, oracle, A, seed=2, w_check=4, w_total=12)


@pytest.mark.parametrize("m,n", [(1024, 4096), (4096, 14336), (14336, 4096)])
def test_layer_shapes_prefix(scd, oracle, m, n):
    from paper_2410_01799_amd import workloads

    A = workloads.weight_like_matrix(m, n, 300)
    run_case(scd, oracle, A, seed=300, w_check=2, w_total=40)


def test_image_tensor_full_size_first_term(scd, oracle):
    """Workload 4 at its real shape (4000 x 3000 x 3): the first term against Algorithm 12 of the oracle, the
    following ones by the identity and the expansion."""
    from paper_2410_01799_amd import workloads

    a = workloads.image_like_tensor(blobs=24)
    N = a.size
    ad = torch.from_numpy(a).cuda()
    res = scd.scd_decompose(ad, 5, 4)
    c = res["c"].cpu().numpy().astype(np.float64)
    tr = res["trace"].cpu().numpy()
    # the first term removes 98 % of the energy (the mean level): the identity is a difference of large
    # numbers there, and its tolerance is relative to ||R_k||^2, the minuend (c is stored in f32)
    assert np.all(np.abs(tr[1:] ** 2 - (tr[:-1] ** 2 - N * c ** 2)) <= ID_RTOL * tr[:-1] ** 2)
    s0 = [oracle.rng_signs(4, 0, i, d) for i, d in enumerate(a.shape)]
    g = oracle.axial_greedy_cut(a.astype(np.float64), s0)
    if g["margin"].min() >= 10 * TIE_TOL:
        for i in range(3):
            assert np.array_equal(to_np_bits(res["signs"][i])[0], g["signs"][i])
        assert c[0] == pytest.approx(g["c"] / N, rel=C_RTOL)
        assert int(res["iters"][0]) == g["iters"]
    E = scd.scd_expand(res["signs"], res["c"], a.shape)
    assert float((ad.double() - E.double()).norm()) == pytest.approx(tr[-1], rel=1e-4)


def test_profile_and_traffic_counters(scd):
    A = torch.randn(1024, 4096, device="cuda")
    with scd.ScdContext(A, 64, 1) as ctx:
        ctx.run(4)
        t0 = ctx.traffic()
        a, b = ctx.profile_sweeps(64)
        t1 = ctx.traffic()
        k = ctx.width
        res = ctx.results()
    assert 0 < a < 1e-3 and 0 < b < 1e-3
    # 64 sampled passes, plus one start pass when the register-resident engine ran the first terms and
    # the launch-stream state had to be rebuilt for the sampling
    assert t1["passes"] - t0["passes"] in (64, 65)
    it = res["iters"].cpu().numpy()
    # passes so far = alternations of the finished terms + those of the term in progress
    assert it.sum() <= t1["passes"] <= it.sum() + 4096
    tr = res["trace"].cpu().numpy()
    c = res["c"].cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(tr[1:] ** 2, tr[:-1] ** 2 - 1024 * 4096 * c ** 2, rtol=ID_RTOL)
    sec = scd.scd_probe_stream(A, None, 256, 5)
    assert 0 < sec < 1e-2
