"""Edge cases of the GPU path: degenerate and ragged shapes, extreme values, high order, exhausted
remainders -- each against the oracle or against properties that hold for any input."""
import numpy as np
import pytest
import torch

from helpers import C_RTOL, ID_RTOL, dense, match_matrix_term, match_tensor_term, to_dev_bits, to_np_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def scd():
    from paper_2410_01799_amd import scd as mod

    mod.lib()
    return mod


def gauss(shape, seed, dtype=np.float32):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape).astype(dtype)


def check_against_oracle(scd, oracle, A, w, seed):
    """Lockstep: every term must be an outcome of Algorithm 4 / 12 on the oracle's own remainder (the literal
    one unless a decision was a near tie); then the free-running oracle's curve is compared as well."""
    A64 = A.astype(np.float64)
    f32 = A.dtype == np.float32
    res = scd.scd_decompose(torch.from_numpy(np.ascontiguousarray(A)).cuda(), w, seed)
    c = res["c"].cpu().numpy().astype(np.float64)
    trace = res["trace"].cpu().numpy()
    iters = res["iters"].cpu().numpy()
    signs = [to_np_bits(s) for s in res["signs"]]
    N = A.size
    np.testing.assert_allclose(trace[1:] ** 2, trace[:-1] ** 2 - N * c ** 2, rtol=ID_RTOL, atol=1e-12 * trace[0] ** 2)
    r = A64.copy()
    literal = True
    for k in range(w):
        start = [oracle.rng_signs(seed, k, i, d) for i, d in enumerate(A.shape)]
        mine = [sg[k] for sg in signs]
        if A.ndim == 2:
            flips, g = match_matrix_term(oracle, r, start[1], mine[0], mine[1], iters[k], f32, f"term {k}")
        else:
            flips, g = match_tensor_term(oracle, r, start, mine, iters[k], f32, f"term {k}")
        literal = literal and flips == 0
        if flips == 0 and g["c"] != 0.0:
            assert c[k] == pytest.approx(g["c"] / N, rel=C_RTOL), f"term {k}"
        prod = np.ones(())
        for b, d in zip(mine, A.shape):
            prod = np.multiply.outer(prod, dense(b, d))
        ck = float((r * prod).sum()) / N
        assert c[k] == pytest.approx(ck, rel=C_RTOL, abs=1e-7 * np.abs(A64).max()), f"term {k}: c vs <s, r>/N"
        r = r - ck * prod
        assert trace[k + 1] == pytest.approx(np.linalg.norm(r), rel=2e-5, abs=1e-6 * trace[0])
    ref = oracle.decompose(A64, w, seed) if A.ndim == 2 else oracle.tensor_decompose(A64, w, seed)
    if literal:
        signs_ref = [ref["S"], ref["T"]] if A.ndim == 2 else ref["signs"]
        for got, want in zip(signs, signs_ref):
            assert np.array_equal(got, want)
        assert np.array_equal(iters, ref["iters"])
    np.testing.assert_allclose(trace, ref["trace"], rtol=1e-3, atol=1e-6 * trace[0])
    return res


@pytest.mark.parametrize("m,n", [(1, 1), (1, 9), (9, 1), (2, 3), (3, 2), (65, 2), (2, 65), (5, 4096), (4096, 5),
                                 (300, 6), (63, 129)])
def test_degenerate_matrix_shapes(scd, oracle, m, n):
    check_against_oracle(scd, oracle, gauss((m, n), 7 * m + n), min(6, m * n), 3)


@pytest.mark.parametrize("shape", [(2, 2, 2), (3, 1, 4), (1, 5, 1), (2, 2, 2, 2, 2, 2, 2, 2), (17, 3, 5, 2), (130, 2, 70)])
def test_degenerate_tensor_shapes(scd, oracle, shape):
    check_against_oracle(scd, oracle, gauss(shape, sum(shape)), 5, 9)


def test_extreme_magnitudes(scd, oracle):
    # squares of 1e25 overflow f32: the norm must be carried in f64
    A = gauss((64, 96), 1) * np.float32(1e25)
    res = check_against_oracle(scd, oracle, A, 6, 2)
    assert np.all(np.isfinite(res["trace"].cpu().numpy()))
    B = gauss((64, 96), 2) * np.float32(1e-25)
    check_against_oracle(scd, oracle, B, 6, 2)


def test_exhausted_remainder_and_zero_matrix(scd):
    # rank-one input: after the first term the remainder is exactly zero; further terms have c = 0
    s = np.sign(gauss(33, 1)); t = np.sign(gauss(65, 2))
    A = torch.from_numpy((2.5 * np.outer(s, t)).astype(np.float32)).cuda()
    res = scd.scd_decompose(A, 4, 1)
    c = res["c"].cpu().numpy()
    tr = res["trace"].cpu().numpy()
    assert c[0] == pytest.approx(2.5, rel=1e-6) and np.all(np.abs(c[1:]) <= 1e-12)
    assert np.all(tr[1:] <= 1e-6 * tr[0])
    Z = torch.zeros(40, 50, device="cuda")
    rz = scd.scd_decompose(Z, 3, 0)
    assert float(rz["c"].abs().max()) == 0.0 and float(rz["trace"].abs().max()) == 0.0
    assert rz["iters"].cpu().tolist() == [2, 2, 2]


def test_signed_zero_and_padding(scd, oracle):
    # -0.0 entries and sums that are exactly zero give sign +1 (bit 0); padding bits stay clear
    R = np.zeros((70, 66), dtype=np.float32)
    R[:, 0] = -0.0
    R[3, 5] = 1.0
    R[3, 6] = -1.0
    t = oracle.pack(np.ones(66))
    u, sb = scd.scd_row_signed_sum(torch.from_numpy(R).cuda(), to_dev_bits(t))
    assert float(u.abs().max()) == 0.0
    assert np.array_equal(to_np_bits(sb), np.zeros(2, dtype=np.uint64))
    s = oracle.pack(-np.ones(70))
    v, tb, c = scd.scd_col_signed_sum(torch.from_numpy(R).cuda(), to_dev_bits(s))
    bits = dense(to_np_bits(tb), 66)
    assert bits[5] == -1.0 and bits[6] == 1.0 and float(c) == 2.0
    assert int(to_np_bits(tb)[1]) >> 2 == 0


def test_capacity_and_argument_errors(scd):
    A = torch.randn(32, 48, device="cuda")
    with scd.ScdContext(A, 1, 0) as ctx:
        assert ctx.run(0) == 0
        ctx.step()
        with pytest.raises(scd.ScdError) as e:
            ctx.run(1)
        assert e.value.code == scd.EFULL
        with pytest.raises(ValueError):
            ctx.set_remainder(torch.randn(32, 47, device="cuda"))
    with pytest.raises(TypeError):
        scd.scd_decompose(A.half(), 1, 0)
    with pytest.raises(ValueError):
        scd.scd_decompose(A.cpu(), 1, 0)
