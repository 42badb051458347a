"""The register-resident engine (whole remainder in the register files, one persistent launch) against
the oracle and against the launch-stream path, on every shape it is built for."""
import numpy as np
import pytest
import torch

from helpers import C_RTOL, CURVE_RTOL, ID_RTOL, to_np_bits
from test_gpu_parity import lockstep_check

pytestmark = pytest.mark.gpu

SHAPES = [(1024, 4096), (2048, 2048), (4096, 4096), (256, 256), (512, 512), (1024, 1024)]
# shapes the grid overhangs (zero rows and columns in the registers), or with an oblong thread tile
RAGGED = [(4096, 1024), (2048, 4096), (1000, 4096), (2052, 516), (100, 76), (8, 8), (5, 4096), (300, 260), (1, 4),
          (1030, 520), (4000, 4092), (64, 4096), (3000, 2000)]


@pytest.fixture(scope="module")
def scd():
    from paper_2410_01799_amd import scd as mod

    mod.lib()
    return mod


RESIDENT = {"resident": 1}
STREAM = {"resident": 0, "sparse": 0, "persistent_stream": 0}


def gauss(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape).astype(np.float32)


@pytest.mark.parametrize("m,n", SHAPES + RAGGED)
def test_resident_matches_oracle_in_lockstep(scd, oracle, m, n):
    w, seed = min(10, m * n), 17
    A = gauss((m, n), m + n)
    with scd.ScdContext(torch.from_numpy(A).cuda(), w, seed, options=RESIDENT) as ctx:
        assert ctx.engine()["engine"] == 1
        ctx.run(w)
        res = ctx.results()
        R = ctx.remainder()
    S, T = to_np_bits(res["signs"][0]), to_np_bits(res["signs"][1])
    c = res["c"].cpu().numpy().astype(np.float64)
    trace = res["trace"].cpu().numpy()
    iters = res["iters"].cpu().numpy()
    # (a 1 x 4 matrix is exhausted after three terms: the identity then compares rounding noise)
    np.testing.assert_allclose(trace[1:] ** 2, trace[:-1] ** 2 - m * n * c ** 2, rtol=ID_RTOL, atol=1e-12 * trace[0] ** 2)
    curve, _ = lockstep_check(oracle, A.astype(np.float64), seed, S, T, c, trace, iters, True)
    np.testing.assert_allclose(trace, curve, rtol=2e-5, atol=1e-6 * trace[0])
    np.testing.assert_allclose(trace / trace[0], curve / curve[0], rtol=CURVE_RTOL, atol=1e-6)
    E = scd.scd_expand(res["signs"], res["c"], (m, n)).double()
    resid = float((torch.from_numpy(A).cuda().double() - E).norm())
    assert resid == pytest.approx(trace[-1], rel=1e-4, abs=1e-6 * trace[0])
    # padding bits of the sign vectors are clear, and the remainder in memory is A - expand(S, T, c)
    if m % 64:
        assert np.all(S[:, -1] >> np.uint64(m % 64) == 0)
    if n % 64:
        assert np.all(T[:, -1] >> np.uint64(n % 64) == 0)
    assert float((torch.from_numpy(A).cuda() - E.float() - R).abs().max()) <= 2e-6 * float(np.abs(A).max())


@pytest.mark.parametrize("m,n", SHAPES[:2] + SHAPES[3:])
def test_resident_and_stream_paths_agree(scd, m, n):
    A = torch.from_numpy(gauss((m, n), 5)).cuda()
    a = scd.scd_decompose(A, 8, 3, options=RESIDENT)
    b = scd.scd_decompose(A, 8, 3, options=STREAM)
    ta, tb = a["trace"].cpu().numpy(), b["trace"].cpu().numpy()
    np.testing.assert_allclose(ta / ta[0], tb / tb[0], rtol=CURVE_RTOL)
    # same signs unless a near tie split the two summation orders: then the curves still agree (above)
    if torch.equal(a["signs"][0], b["signs"][0]) and torch.equal(a["signs"][1], b["signs"][1]):
        np.testing.assert_allclose(a["c"].cpu().numpy(), b["c"].cpu().numpy(), rtol=C_RTOL)
        assert torch.equal(a["iters"], b["iters"])
        np.testing.assert_allclose(ta, tb, rtol=1e-6)


def test_resident_chunking_determinism_and_handover(scd):
    m, n = 1024, 4096
    A = torch.from_numpy(gauss((m, n), 9)).cuda()
    one = scd.scd_decompose(A, 9, 4)
    two = scd.scd_decompose(A, 9, 4)
    for k in ("c", "trace", "iters"):
        assert torch.equal(one[k], two[k])
    with scd.ScdContext(A, 12, 4) as ctx:
        ctx.step()
        ctx.run(5)
        ctx.step()
        ctx.run(2)
        assert ctx.width == 9
        res = ctx.results()
        R = ctx.remainder()
        # hand-over to the launch-stream path: profiling sweeps continue the same decomposition
        ctx.profile_sweeps(40)
        k2 = ctx.width
        res2 = ctx.results()
    assert torch.equal(one["signs"][0], res["signs"][0]) and torch.equal(one["signs"][1], res["signs"][1])
    assert torch.equal(one["c"], res["c"]) and torch.equal(one["trace"], res["trace"])
    E = scd.scd_expand(res["signs"], res["c"], (m, n))
    assert float((A - E - R).abs().max()) <= 2e-6 * float(A.abs().max())
    assert k2 >= 9
    tr = res2["trace"].cpu().numpy()
    c2 = res2["c"].cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(tr[1:] ** 2, tr[:-1] ** 2 - m * n * c2 ** 2, rtol=ID_RTOL)


def test_resident_iteration_cap(scd):
    A = torch.from_numpy(gauss((2048, 2048), 2)).cuda()
    with scd.ScdContext(A, 3, 1) as ctx:
        assert ctx.engine()["engine"] == 1
        ctx.set_max_iters(2)
        assert ctx.run(3) == scd.WMAXITER
        r = ctx.results()
    assert r["iters"].cpu().tolist() == [2, 2, 2]
    tr = r["trace"].cpu().numpy()
    c = r["c"].cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(tr[1:] ** 2, tr[:-1] ** 2 - 2048 * 2048 * c ** 2, rtol=ID_RTOL)


def test_exchange_probe_runs(scd):
    t = scd.scd_probe_exchange(0, 256, 16, 200)
    assert 0 < t < 1e-3


def test_a_context_that_loses_its_share_continues_on_the_launch_stream(scd):
    m = n = 1024
    A = torch.from_numpy(gauss((m, n), 21)).cuda()
    with scd.ScdContext(A, 8, 6, options={"sparse": 0, "persistent_stream": 0}) as ctx:
        assert ctx.engine()["engine"] == 1
        ctx.run(4)
        ctx.set_workgroups(16)            # the 8 x 8 grid no longer fits, the other persistent engines are switched off
        assert ctx.engine()["engine"] == 0
        ctx.run(4)
        mixed = ctx.results()
        R = ctx.remainder()
    whole = scd.scd_decompose(A, 8, 6)
    tr = mixed["trace"].cpu().numpy()
    c = mixed["c"].cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(tr[1:] ** 2, tr[:-1] ** 2 - m * n * c ** 2, rtol=ID_RTOL)
    tw = whole["trace"].cpu().numpy()
    np.testing.assert_allclose(tr / tr[0], tw / tw[0], rtol=CURVE_RTOL)
    assert torch.equal(mixed["c"][:4], whole["c"][:4])
    E = scd.scd_expand(mixed["signs"], mixed["c"], (m, n))
    assert float((A - E - R).abs().max()) <= 2e-6 * float(A.abs().max())
