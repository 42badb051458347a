"""The real-last-mode variant ("RGB scalars", Section 5) on the GPU against the oracle, in lockstep: for every
term the oracle repeats the axial greedy cut on its own f64 remainder and refits the per-slice coefficients."""
import numpy as np
import pytest
import torch

from helpers import C_RTOL, CURVE_RTOL, dense, match_tensor_term, to_np_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def scd():
    from paper_2410_01799_amd import scd as mod

    mod.lib()
    return mod


def gauss(shape, seed, dtype=np.float32):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape).astype(dtype)


def lead_product(signs, j, shape):
    t = np.ones(())
    for i, d in enumerate(shape[:-1]):
        t = np.multiply.outer(t, dense(signs[i][j], d))
    return t


def run_and_check(scd, oracle, a, w, seed):
    shape = a.shape
    f32 = a.dtype == np.float32
    a64 = a.astype(np.float64)
    res = scd.scd_decompose_scalars(torch.from_numpy(a).cuda(), w, seed)
    assert res["status"] == 0
    sg = [to_np_bits(s) for s in res["signs"]]
    c = res["c"].cpu().numpy().astype(np.float64)
    trace = res["trace"].cpu().numpy()
    iters = res["iters"].cpu().numpy()
    P = int(np.prod(shape[:-1]))
    r = a64.copy()
    curve = [np.linalg.norm(r)]
    for k in range(w):
        start = [oracle.rng_signs(seed, k, i, d) for i, d in enumerate(shape)]
        match_tensor_term(oracle, r, start, [s[k] for s in sg], iters[k], f32, f"term {k}", modes=len(shape) - 1)
        lead = lead_product(sg, k, shape)                      # the GPU's sign vectors (adopted where they differ)
        ck = np.tensordot(lead, r, axes=len(shape) - 1) / P
        np.testing.assert_allclose(c[k], ck, rtol=C_RTOL, atol=C_RTOL * np.abs(ck).max())
        r = r - np.multiply.outer(lead, c[k])                  # what the GPU subtracted: its stored coefficients
        curve.append(np.linalg.norm(r))
        for i, d in enumerate(shape[:-1]):
            if d % 64:
                assert int(sg[i][k][-1]) >> (d % 64) == 0
    curve = np.array(curve)
    np.testing.assert_allclose(trace, curve, rtol=2e-5 if f32 else 1e-11)
    np.testing.assert_allclose(trace / trace[0], curve / curve[0], rtol=CURVE_RTOL)
    assert np.all(np.diff(trace) < 0)
    return res


@pytest.mark.parametrize("shape,w,dtype", [((40, 30, 3), 12, np.float32), ((40, 30, 3), 10, np.float64), ((9, 70, 5, 2), 8, np.float32),
                                           ((130, 1, 3), 6, np.float64), ((66, 9, 1), 7, np.float32), ((50, 64), 8, np.float32),
                                           ((300, 200, 3), 10, np.float32),
                                           # order 3 with rows of whole 16-byte pieces: the persistent streaming engine
                                           ((257, 64, 4), 8, np.float32), ((100, 50, 2), 8, np.float32), ((513, 33, 4), 6, np.float64),
                                           ((1000, 750, 3), 6, np.float32)])
def test_scalars_match_oracle_in_lockstep(scd, oracle, shape, w, dtype):
    run_and_check(scd, oracle, gauss(shape, sum(shape) + w, dtype), w, 7)


def test_scalars_beat_signs_on_an_image_like_tensor(scd):
    # Section 5: "this approach converges noticeably faster"
    from paper_2410_01799_amd import workloads

    a = torch.from_numpy(workloads.image_like_tensor(240, 180, 3, blobs=40, seed=400)).cuda()
    w = 32
    sc = scd.scd_decompose_scalars(a, w, 3)
    sg = scd.scd_decompose(a, w, 3)
    assert float(sc["trace"][w]) < float(sg["trace"][w])
    # the definition, rebuilt with torch from the bitsets and the real vectors
    S = 1.0 - 2.0 * torch.from_numpy(np.stack([dense(r_, 240) for r_ in to_np_bits(sc["signs"][0])]) < 0).double().cuda()
    T = 1.0 - 2.0 * torch.from_numpy(np.stack([dense(r_, 180) for r_ in to_np_bits(sc["signs"][1])]) < 0).double().cuda()
    E = torch.einsum("ji,jl,jc->ilc", S, T, sc["c"].double())
    assert float((a.double() - E).norm()) == pytest.approx(float(sc["trace"][w]), rel=1e-4)


def test_scalars_image_tensor_full_size(scd, oracle):
    """Workload 4 at its real shape with a real last mode: the first term in lockstep with the oracle (the sweeps are
    Algorithm 12's, the coefficients the slice-wise least squares ones), the following terms by the definition
    rebuilt with torch and by the norm identity ||r_{j+1}||^2 = ||r_j||^2 - mn sum_c c_j[c]^2."""
    from paper_2410_01799_amd import workloads

    a = workloads.image_like_tensor(blobs=24)
    m, n, q = a.shape
    ad = torch.from_numpy(a).cuda()
    w = 4
    res = scd.scd_decompose_scalars(ad, w, 4)
    c = res["c"].double()
    tr = res["trace"].cpu().numpy()
    cc = c.cpu().numpy()
    # (the first term removes most of the energy: the tolerance is relative to the minuend; c is stored in f32)
    assert np.all(np.abs(tr[1:] ** 2 - (tr[:-1] ** 2 - m * n * (cc ** 2).sum(axis=1))) <= 1e-6 * tr[:-1] ** 2)
    s0 = [oracle.rng_signs(4, 0, i, d) for i, d in enumerate(a.shape)]
    match_tensor_term(oracle, a.astype(np.float64), s0, [to_np_bits(res["signs"][i])[0] for i in range(2)],
                      int(res["iters"][0]), True, "first term of the image tensor, real last mode", modes=2)
    S = 1.0 - 2.0 * torch.from_numpy(np.stack([dense(r_, m) for r_ in to_np_bits(res["signs"][0])]) < 0).double().cuda()
    T = 1.0 - 2.0 * torch.from_numpy(np.stack([dense(r_, n) for r_ in to_np_bits(res["signs"][1])]) < 0).double().cuda()
    lead0 = torch.outer(S[0], T[0])
    want0 = torch.tensordot(lead0, ad.double(), dims=2) / (m * n)   # slice-wise least squares coefficients of term 0
    assert torch.allclose(c[0], want0, rtol=1e-5, atol=0)
    E = torch.einsum("ji,jl,jc->ilc", S, T, c)
    assert float((ad.double() - E).norm()) == pytest.approx(float(tr[w]), rel=1e-4)


def test_scalars_edges_and_errors(scd):
    a = torch.from_numpy(gauss((20, 30, 3), 1)).cuda()
    r0 = scd.scd_decompose_scalars(a, 0, 1)
    assert r0["c"].shape == (0, 3) and float(r0["trace"][0]) == pytest.approx(float(a.double().norm()), rel=1e-12)
    bad = a.clone()
    bad[1, 2, 0] = float("inf")
    with pytest.raises(scd.ScdError) as e:
        scd.scd_decompose_scalars(bad, 2, 1)
    assert e.value.code == -5
    capped = scd.scd_decompose_scalars(a, 3, 1, max_iters=1)
    assert capped["status"] == 1 and torch.all(capped["iters"] == 1)
    one = scd.scd_decompose_scalars(a, 4, 1)
    two = scd.scd_decompose_scalars(a, 4, 1)
    assert torch.equal(one["c"], two["c"]) and torch.equal(one["trace"], two["trace"])
