"""The persistent streaming engine (one launch that streams the remainder once per alternation, the first rows
of every workgroup's block kept in LDS) against the oracle in lockstep and against the other engines: f32 and
f64, square, ragged, more rows than fit in LDS, a share of the device."""
import numpy as np
import pytest
import torch

from helpers import C_RTOL, CURVE_RTOL, ID_RTOL, dense, match_tensor_term, to_np_bits
from test_gpu_parity import lockstep_check

pytestmark = pytest.mark.gpu

OPTS = {"resident": 0, "sparse": 0}


@pytest.fixture(scope="module")
def scd():
    from paper_2410_01799_amd import scd as mod

    mod.lib()
    return mod


def gauss(shape, seed, dtype=np.float32):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape).astype(dtype)


def run_and_check(scd, oracle, A, w, seed, share=0, chunks=None):
    m, n = A.shape
    Ad = torch.from_numpy(A).cuda()
    with scd.ScdContext(Ad, w, seed, options=OPTS) as ctx:
        if share:
            ctx.set_workgroups(share)
        assert ctx.engine()["engine"] == 3
        for part in (chunks or [w]):
            ctx.run(part)
        res = ctx.results()
        R = ctx.remainder()
    S, T = to_np_bits(res["signs"][0]), to_np_bits(res["signs"][1])
    c = res["c"].cpu().numpy().astype(np.float64)
    trace = res["trace"].cpu().numpy()
    iters = res["iters"].cpu().numpy()
    f32 = A.dtype == np.float32
    np.testing.assert_allclose(trace[1:] ** 2, trace[:-1] ** 2 - m * n * c ** 2, rtol=ID_RTOL)
    curve, _ = lockstep_check(oracle, A.astype(np.float64), seed, S, T, c, trace, iters, f32)
    np.testing.assert_allclose(trace, curve, rtol=2e-5 if f32 else 1e-11)
    np.testing.assert_allclose(trace / trace[0], curve / curve[0], rtol=CURVE_RTOL)
    # padding bits clear
    if m % 64:
        assert np.all(S[:, -1] >> np.uint64(m % 64) == 0)
    if n % 64:
        assert np.all(T[:, -1] >> np.uint64(n % 64) == 0)
    # the remainder in memory is A - expand(S, T, c), and its norm is the last trace value
    E = scd.scd_expand(res["signs"], res["c"], (m, n))
    tol = 2e-6 if f32 else 1e-13
    assert float((Ad - E - R).abs().max()) <= tol * float(Ad.abs().max())
    assert float(R.double().norm()) == pytest.approx(trace[-1], rel=1e-6 if f32 else 1e-12)
    return res


@pytest.mark.parametrize("m,n,w", [(256, 256, 32), (100, 76, 20), (8, 8, 6), (77, 1024, 16), (1000, 4096, 12),
                                   (2052, 516, 12), (1030, 520, 16), (130, 8200, 8), (16, 64, 4), (8, 4, 2),
                                   (4096, 4096, 8), (700, 16384, 4)])
def test_stream_matches_oracle_f32(scd, oracle, m, n, w):
    run_and_check(scd, oracle, gauss((m, n), m * 3 + n), w, 11)


@pytest.mark.parametrize("m,n,w", [(256, 256, 24), (130, 1026, 12), (65, 130, 10), (2048, 2048, 6), (300, 8192, 4)])
def test_stream_matches_oracle_f64(scd, oracle, m, n, w):
    run_and_check(scd, oracle, gauss((m, n), m + 7 * n, np.float64), w, 5)


def test_stream_large_layer_shape(scd, oracle):
    # 14336 x 4096: 56 rows per workgroup of which 9 stay in LDS
    from paper_2410_01799_amd import workloads

    run_and_check(scd, oracle, workloads.weight_like_matrix(14336, 4096, 300), 3, 300)


@pytest.mark.parametrize("m,n,w,share", [(1000, 4096, 8, 64), (256, 256, 12, 16), (2052, 516, 8, 85)])
def test_stream_on_a_share_of_the_device(scd, oracle, m, n, w, share):
    run_and_check(scd, oracle, gauss((m, n), m + n + share), w, 13, share)


def test_stream_chunking_determinism_and_handover(scd):
    m, n = 640, 896
    A = torch.from_numpy(gauss((m, n), 9)).cuda()
    one = scd.scd_decompose(A, 10, 4, options=OPTS)
    two = scd.scd_decompose(A, 10, 4, options=OPTS)
    for k in ("c", "trace", "iters"):
        assert torch.equal(one[k], two[k])
    assert torch.equal(one["signs"][0], two["signs"][0]) and torch.equal(one["signs"][1], two["signs"][1])
    with scd.ScdContext(A, 14, 4, options=OPTS) as ctx:
        ctx.step()
        ctx.run(6)
        ctx.step()
        ctx.run(2)
        res = ctx.results()
        # the launch-stream kernels take over for a while, then the persistent launch again
        ctx.profile_sweeps(30)
        k2 = ctx.width
        if k2 < 14:
            ctx.run(14 - k2)
        res2 = ctx.results()
        R = ctx.remainder()
    # a launch boundary changes nothing: every launch starts from the remainder in memory and the keyed start
    assert torch.equal(one["signs"][0], res["signs"][0]) and torch.equal(one["signs"][1], res["signs"][1])
    assert torch.equal(one["c"], res["c"]) and torch.equal(one["trace"], res["trace"])
    tr = res2["trace"].cpu().numpy()
    c2 = res2["c"].cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(tr[1:] ** 2, tr[:-1] ** 2 - m * n * c2 ** 2, rtol=ID_RTOL)
    E = scd.scd_expand(res2["signs"], res2["c"], (m, n))
    assert float((A - E - R).abs().max()) <= 4e-6 * float(A.abs().max())


def test_stream_iteration_cap_and_set_remainder(scd):
    A = torch.from_numpy(gauss((512, 512), 2)).cuda()
    with scd.ScdContext(A, 6, 1, options=OPTS) as ctx:
        assert ctx.engine()["engine"] == 3
        ctx.set_max_iters(1)
        assert ctx.run(2) == scd.WMAXITER
        assert ctx.results()["iters"].cpu().tolist() == [1, 1]
        ctx.set_max_iters(4096)
        R2 = ctx.remainder()
        ctx.set_remainder(R2)
        ctx.run(2)
        r = ctx.results()
    tr = r["trace"].cpu().numpy()
    c = r["c"].cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(tr[1:] ** 2, tr[:-1] ** 2 - 512 * 512 * c ** 2, rtol=ID_RTOL)


def test_stream_and_launch_stream_engines_agree(scd):
    A = torch.from_numpy(gauss((768, 1280), 5)).cuda()
    a = scd.scd_decompose(A, 16, 3, options=OPTS)
    b = scd.scd_decompose(A, 16, 3, options={**OPTS, "persistent_stream": 0})
    ta, tb = a["trace"].cpu().numpy(), b["trace"].cpu().numpy()
    np.testing.assert_allclose(ta / ta[0], tb / tb[0], rtol=CURVE_RTOL)
    if torch.equal(a["signs"][0], b["signs"][0]) and torch.equal(a["signs"][1], b["signs"][1]):
        np.testing.assert_allclose(a["c"].cpu().numpy(), b["c"].cpu().numpy(), rtol=C_RTOL)
        assert torch.equal(a["iters"], b["iters"])


# ---- order-3 tensors (Algorithms 12 and 13) on the same engine


def kron_dense(sign_rows, shape):
    out = np.array([1.0])
    for b, d in zip(sign_rows, shape):
        out = np.multiply.outer(out, dense(b, d))
    return out.reshape(shape)


@pytest.mark.parametrize("shape,w,dtype", [((64, 40, 3), 16, np.float32), ((40, 30, 3), 16, np.float64),
                                           ((130, 64, 4), 12, np.float32), ((300, 200, 3), 8, np.float32),
                                           ((50, 44, 2), 10, np.float32), ((33, 16, 1), 8, np.float32),
                                           ((700, 1000, 3), 5, np.float32), ((90, 130, 3), 8, np.float64)])
def test_stream_tensor_matches_oracle(scd, oracle, shape, w, dtype):
    seed = 4
    a = gauss(shape, int(np.prod(shape)), dtype)
    a64 = a.astype(np.float64)
    N = a.size
    ad = torch.from_numpy(a).cuda()
    with scd.ScdContext(ad, w, seed, options=OPTS) as ctx:
        assert ctx.engine()["engine"] == 3
        ctx.run(w // 2)
        ctx.run(w - w // 2)
        res = ctx.results()
        R = ctx.remainder()
    signs = [to_np_bits(s) for s in res["signs"]]
    c = res["c"].cpu().numpy().astype(np.float64)
    trace = res["trace"].cpu().numpy()
    iters = res["iters"].cpu().numpy()
    f32 = dtype == np.float32
    np.testing.assert_allclose(trace[1:] ** 2, trace[:-1] ** 2 - N * c ** 2, rtol=ID_RTOL)
    r = a64.copy()
    for k in range(w):
        s0 = [oracle.rng_signs(seed, k, i, d) for i, d in enumerate(shape)]
        mine = [sg[k] for sg in signs]
        flips, g = match_tensor_term(oracle, r, s0, mine, iters[k], f32, f"term {k}")
        if flips == 0:
            assert c[k] == pytest.approx(g["c"] / N, rel=C_RTOL)
        ck = (r * kron_dense(mine, shape)).sum() / N
        assert c[k] == pytest.approx(ck, rel=C_RTOL)
        oracle.tensor_update(r, ck, mine)
        assert trace[k + 1] == pytest.approx(np.linalg.norm(r), rel=2e-5 if f32 else 1e-11)
        for i, d in enumerate(shape):
            if d % 64:
                assert int(mine[i][-1]) >> (d % 64) == 0, "padding bits"
    E = scd.scd_expand(res["signs"], res["c"], shape)
    assert float((ad - E - R).abs().max()) <= (2e-6 if f32 else 1e-13) * float(ad.abs().max())
    assert float(R.double().norm()) == pytest.approx(trace[-1], rel=1e-6 if f32 else 1e-12)
    # the launch-per-sweep engine on the same input: the same curve, the same terms unless a near tie split them
    other = scd.scd_decompose(ad, w, seed, options={**OPTS, "persistent_stream": 0})
    to = other["trace"].cpu().numpy()
    np.testing.assert_allclose(trace / trace[0], to / to[0], rtol=CURVE_RTOL)
