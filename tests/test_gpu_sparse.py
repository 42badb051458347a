"""The sparse engine (cached products updated from the flipped signs only, Section 3.1) against the
oracle in lockstep and against the launch-stream engine, f32 and f64, square, ragged and large."""
import numpy as np
import pytest
import torch

from helpers import C_RTOL, CURVE_RTOL, ID_RTOL, to_np_bits
from test_gpu_parity import lockstep_check

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def scd():
    from paper_2410_01799_amd import scd as mod

    mod.lib()
    return mod


OPTS = {}


@pytest.fixture(autouse=True, params=["immediate", "delayed"])
def engines(request):
    """Options for every context of a test: the sparse engine also for the register-resident engine's shapes
    and for matrices below the size from which it pays off; updates subtracted at once, or kept in a list of
    pending terms (Section 3.2)."""
    OPTS.clear()
    OPTS.update({"resident": 0, "sparse_min_mib": 0, "sparse_delay_width": 8 if request.param == "delayed" else 0})
    yield request.param
    OPTS.clear()


def context(scd, A, w, seed, **extra):
    return scd.ScdContext(A, w, seed, options={**OPTS, **extra})


def decompose(scd, A, w, seed, **extra):
    return scd.scd_decompose(A, w, seed, options={**OPTS, **extra})


def gauss(shape, seed, dtype=np.float32):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape).astype(dtype)


def run_and_check(scd, oracle, A, w, seed, share=0, **extra):
    m, n = A.shape
    Ad = torch.from_numpy(A).cuda()
    with context(scd, Ad, w, seed, **extra) as ctx:
        if share:
            ctx.set_workgroups(share)
        assert ctx.engine()["engine"] == 2
        ctx.run(w)
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
    # the remainder in memory is A - expand(S, T, c), and its norm is the last trace value
    E = scd.scd_expand(res["signs"], res["c"], (m, n))
    tol = 2e-6 if f32 else 1e-13
    assert float((Ad - E - R).abs().max()) <= tol * float(Ad.abs().max())
    assert float(R.double().norm()) == pytest.approx(trace[-1], rel=1e-6 if f32 else 1e-12)
    return res


@pytest.mark.parametrize("m,n,w", [(256, 256, 32), (100, 76, 20), (8, 8, 6), (1000, 4096, 12), (2052, 516, 12),
                                   (4096, 4096, 8)])
def test_sparse_matches_oracle_f32(scd, oracle, m, n, w):
    run_and_check(scd, oracle, gauss((m, n), m * 3 + n), w, 11)


@pytest.mark.parametrize("m,n,w", [(256, 256, 24), (130, 1026, 12), (4096, 4096, 4)])
def test_sparse_matches_oracle_f64(scd, oracle, m, n, w):
    run_and_check(scd, oracle, gauss((m, n), m + 7 * n, np.float64), w, 5)


@pytest.mark.parametrize("m,n,w,dtype", [(256, 256, 70, np.float32), (100, 76, 45, np.float64), (1000, 520, 36, np.float32)])
def test_sparse_more_terms_than_the_pending_list_holds(scd, oracle, m, n, w, dtype):
    run_and_check(scd, oracle, gauss((m, n), m + n + w, dtype), w, 19)


def test_sparse_pending_list_of_the_papers_length(scd, oracle, engines):
    # the default list holds 8 terms; Section 3.2's 32 (and the shortest, 4) go through the same code
    for width in (32, 4):
        run_and_check(scd, oracle, gauss((300, 260), 31 + width), 70, 23, sparse_delay_width=width)


def test_sparse_large_layer_shape(scd, oracle):
    from paper_2410_01799_amd import workloads

    run_and_check(scd, oracle, workloads.weight_like_matrix(14336, 4096, 300), 3, 300)


def test_sparse_embedding_shape(scd, oracle):
    # 32000 x 4096 (500 MiB), the largest matrix of the model and the shape for which delayed updates are the
    # default: slices of 128 rows and 16 columns per workgroup
    from paper_2410_01799_amd import workloads

    run_and_check(scd, oracle, workloads.gaussian_matrix(32000, 4096, 5, np.float32) * np.float32(0.02), 2, 29)


def test_sparse_and_stream_engines_agree(scd):
    A = torch.from_numpy(gauss((768, 1280), 5)).cuda()
    a = decompose(scd, A, 16, 3)
    b = decompose(scd, A, 16, 3, sparse=0)
    ta, tb = a["trace"].cpu().numpy(), b["trace"].cpu().numpy()
    np.testing.assert_allclose(ta / ta[0], tb / tb[0], rtol=CURVE_RTOL)
    if torch.equal(a["signs"][0], b["signs"][0]) and torch.equal(a["signs"][1], b["signs"][1]):
        np.testing.assert_allclose(a["c"].cpu().numpy(), b["c"].cpu().numpy(), rtol=C_RTOL)
        assert torch.equal(a["iters"], b["iters"])


def test_sparse_chunking_determinism_and_handover(scd, engines):
    m, n = 640, 896
    A = torch.from_numpy(gauss((m, n), 9)).cuda()
    one = decompose(scd, A, 10, 4)
    two = decompose(scd, A, 10, 4)
    for k in ("c", "trace", "iters"):
        assert torch.equal(one[k], two[k])
    with context(scd, A, 14, 4) as ctx:
        ctx.step()
        ctx.run(6)
        ctx.step()
        ctx.run(2)
        res = ctx.results()
        # launch-stream kernels take over (the transpose goes stale), then the sparse engine again
        ctx.profile_sweeps(30)
        k2 = ctx.width
        if k2 < 14:
            ctx.run(14 - k2)
        res2 = ctx.results()
        R = ctx.remainder()
    if engines == "immediate":
        assert torch.equal(one["signs"][0], res["signs"][0]) and torch.equal(one["signs"][1], res["signs"][1])
        assert torch.equal(one["c"], res["c"]) and torch.equal(one["trace"], res["trace"])
    else:
        # a launch boundary flushes the pending terms: the copies are bit-identical afterwards, but the sums of the
        # following terms are formed from other operands (R' plus corrections), and the norm is measured at other
        # terms: same curve, not necessarily the same bits
        np.testing.assert_allclose(one["trace"].cpu().numpy(), res["trace"].cpu().numpy(), rtol=1e-5)
    tr = res2["trace"].cpu().numpy()
    c2 = res2["c"].cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(tr[1:] ** 2, tr[:-1] ** 2 - m * n * c2 ** 2, rtol=ID_RTOL)
    E = scd.scd_expand(res2["signs"], res2["c"], (m, n))
    assert float((A - E - R).abs().max()) <= 4e-6 * float(A.abs().max())


def test_sparse_iteration_cap_and_set_remainder(scd):
    A = torch.from_numpy(gauss((512, 512), 2)).cuda()
    with context(scd, A, 6, 1) as ctx:
        assert ctx.engine()["engine"] == 2
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


# ---- a share of the device per context (several decompositions side by side)

@pytest.mark.parametrize("m,n,w,share", [(1000, 4096, 10, 64), (2052, 516, 10, 128), (256, 256, 16, 16),
                                         (4096, 4096, 6, 32), (100, 76, 12, 100), (2052, 516, 10, 85), (1000, 4096, 10, 51)])
def test_share_matches_oracle(scd, oracle, m, n, w, share):
    run_and_check(scd, oracle, gauss((m, n), m + n + share), w, 13, share)


def test_share_f64_and_large(scd, oracle):
    from paper_2410_01799_amd import workloads

    run_and_check(scd, oracle, gauss((1026, 770), 3, np.float64), 8, 2, 64)
    run_and_check(scd, oracle, workloads.weight_like_matrix(14336, 4096, 301), 3, 301, 64)


def test_share_limits_and_engine_choice(scd):
    A = torch.from_numpy(gauss((4096, 4096), 1)).cuda()
    with scd.ScdContext(A, 4, 1) as ctx:
        assert ctx.engine()["engine"] == 1            # the whole device: register-resident
        ctx.run(2)
        ctx.set_workgroups(64)                        # its 256 workgroups do not fit a share of 64
        assert ctx.engine()["engine"] == 2
        ctx.run(2)
        res = ctx.results()
        with pytest.raises(scd.ScdError):
            ctx.set_workgroups(8)
        with pytest.raises(scd.ScdError):
            ctx.set_workgroups(-1)
        ctx.set_workgroups(0)
        assert ctx.engine()["engine"] == 1
    tr = res["trace"].cpu().numpy()
    c = res["c"].cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(tr[1:] ** 2, tr[:-1] ** 2 - 4096 * 4096 * c ** 2, rtol=ID_RTOL)
    B = torch.from_numpy(gauss((256, 256), 2)).cuda()
    with scd.ScdContext(B, 4, 1) as ctx:
        ctx.set_workgroups(64)
        assert ctx.engine()["engine"] == 1            # 4 x 4 workgroups fit
    # a tensor has no persistent engine: the share is accepted and changes nothing
    Tn = torch.from_numpy(gauss((20, 30, 3), 3)).cuda()
    with scd.ScdContext(Tn, 4, 1) as ctx:
        ctx.set_workgroups(64)
        assert ctx.engine()["engine"] == 0
        ctx.run(4)


def test_contexts_side_by_side_reproduce_their_solo_runs(scd):
    import threading

    shapes = [(2048, 1024), (1024, 4096), (1536, 1536), (4096, 1024)]
    mats = [torch.from_numpy(gauss(sh, 40 + i)).cuda() for i, sh in enumerate(shapes)]
    w = 24

    def one(i, out):
        torch.cuda.set_device(0)
        st = torch.cuda.Stream()
        with torch.cuda.stream(st):
            with context(scd, mats[i], w, 100 + i) as ctx:
                ctx.set_workgroups(64)
                assert ctx.engine()["engine"] == 2
                for _ in range(3):
                    ctx.run(w // 3)
                out[i] = ctx.results()
            st.synchronize()

    solo = [None] * len(mats)
    for i in range(len(mats)):
        one(i, solo)
    together = [None] * len(mats)
    errors = []

    def guarded(i):
        try:
            one(i, together)
        except Exception as e:  # noqa: BLE001 - reported below, in the main thread
            errors.append((i, repr(e)))

    threads = [threading.Thread(target=guarded, args=(i,)) for i in range(len(mats))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for a, b in zip(solo, together):
        assert torch.equal(a["signs"][0], b["signs"][0]) and torch.equal(a["signs"][1], b["signs"][1])
        assert torch.equal(a["c"], b["c"]) and torch.equal(a["trace"], b["trace"]) and torch.equal(a["iters"], b["iters"])


def test_sparse_flip_counts(scd):
    A = torch.from_numpy(gauss((512, 1024), 77)).cuda()
    with context(scd, A, 6, 3) as ctx:
        assert ctx.engine()["engine"] == 2
        assert ctx.sparse_flips() == dict(rows=0, cols=0)
        ctx.run(6)
        fl = ctx.sparse_flips()
        alts = int(ctx.results()["iters"].sum())
    # every alternation after a term's first changes at least one sign of each kind (else it would have stopped
    # one earlier, or be the last), and never more than all of them
    assert 0 < fl["rows"] <= 512 * alts and 0 < fl["cols"] <= 1024 * alts
    with context(scd, A, 2, 3, sparse=0) as ctx:
        ctx.run(2)
        assert ctx.sparse_flips() == dict(rows=0, cols=0)
