"""The product of a decomposition with a vector from the packed factors (Section 6.1, Question A):
the HIP path through the C ABI against the f64 oracle, entry by entry."""
import ctypes as C

import numpy as np
import pytest
import torch


pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def scd():
    from paper_2410_01799_amd import scd as mod

    mod.lib()
    return mod


def random_factors(m, n, w, seed, dtype):
    rs = np.random.Generator(np.random.PCG64(seed))
    mw, nw = (m + 63) // 64, (n + 63) // 64
    S = rs.integers(0, 2 ** 63, (w, mw), dtype=np.uint64) * np.uint64(2) + rs.integers(0, 2, (w, mw), dtype=np.uint64)
    T = rs.integers(0, 2 ** 63, (w, nw), dtype=np.uint64) * np.uint64(2) + rs.integers(0, 2, (w, nw), dtype=np.uint64)
    if m % 64 and w:
        S[:, -1] &= np.uint64((1 << (m % 64)) - 1)     # padding bits are zero, as the library writes them
    if n % 64 and w:
        T[:, -1] &= np.uint64((1 << (n % 64)) - 1)
    c = (rs.standard_normal(w) * 10.0 ** rs.uniform(-3, 0, w)).astype(dtype)
    return S, T, c


def fixed_point_tol(c64, x64, nin, w):
    """Bound on what the two block fixed points of the f32 path may cost (independent roundings: of the order
    of the square root of their number; 4 times that is far above it and far below a lost digit)."""
    zmax = float(np.abs(c64).max(initial=0.0) * np.abs(x64).sum())
    return (4.0 * np.sqrt(nin) * float(np.abs(x64).max(initial=0.0)) * 2.0 ** -30 * float(np.abs(c64).sum())
            + 4.0 * np.sqrt(max(w, 1)) * zmax * 2.0 ** -30)


def dev_bits(a):
    return torch.from_numpy(a.view(np.int64).copy()).cuda()


def check(scd, oracle, m, n, w, seed, dtype, transpose, nvec=1):
    S, T, c = random_factors(m, n, w, seed, dtype)
    rs = np.random.Generator(np.random.PCG64(seed + 1))
    nin, nout = (m, n) if transpose else (n, m)
    x = rs.standard_normal((nvec, nin)).astype(dtype)
    y = scd.scd_apply(dev_bits(S), dev_bits(T), torch.from_numpy(c).cuda(), m, n, torch.from_numpy(x).cuda(),
                      transpose=transpose)
    assert y.shape == (nvec, nout) and y.dtype == torch.from_numpy(c).dtype
    y = y.cpu().numpy().astype(np.float64)
    for v in range(nvec):
        ref = oracle.apply(S, T, c.astype(np.float64), m, n, x[v].astype(np.float64), transpose=transpose)
        # f64 path: both sides add the same exactly representable terms in f64, in different orders.
        # f32 path: <t_j, x> is formed in fixed point on the matrix cores: x is rounded to 30 bits below the
        # largest entry of its chunk of 4096 (at most max|x| 2^-30 per entry, exact sums afterwards), the rest
        # is f64; the result is rounded once to f32.  The roundings are independent, so their sum over a row is
        # of the order sqrt(n) of them; 4 sqrt(n) is far above that and far below what a lost digit would cost.
        # The sum over the terms is formed the same way: z_j = c_j <t_j, x> is rounded to 30 bits below the
        # largest |z| of its split of the terms (|z_j| <= |c_j| sum|x|), exact sums afterwards.
        c64, x64 = c.astype(np.float64), x[v].astype(np.float64)
        zabs = float(np.abs(c64).sum() * np.abs(x64).sum())
        tol = 1e-13 * zabs
        if dtype == np.float32:
            tol = tol + fixed_point_tol(c64, x64, nin, w) + 2.0 ** -23 * np.abs(ref)
        assert np.all(np.abs(y[v] - ref) <= tol + 1e-300), (m, n, w, transpose, float(np.abs(y[v] - ref).max()))


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("m,n,w", [(256, 256, 64), (100, 76, 33), (8, 8, 5), (1, 1, 3), (4096, 4100, 70), (65, 8200, 9),
                                   (5000, 130, 300), (64, 64, 1)])
def test_apply_matches_oracle(scd, oracle, m, n, w, dtype):
    check(scd, oracle, m, n, w, m + 3 * n + w, dtype, False)
    check(scd, oracle, m, n, w, m + 3 * n + w + 7, dtype, True)


def test_apply_scales_of_x(scd, oracle):
    # the fixed point follows the scale of x: tiny, huge and mixed-magnitude vectors
    m, n, w = 200, 4100, 50
    S, T, c = random_factors(m, n, w, 21, np.float32)
    rs = np.random.Generator(np.random.PCG64(22))
    for scale in (1e-30, 1e30):
        x = (rs.standard_normal(n) * scale).astype(np.float32)
        y = scd.scd_apply(dev_bits(S), dev_bits(T), torch.from_numpy(c).cuda(), m, n, torch.from_numpy(x).cuda())
        ref = oracle.apply(S, T, c.astype(np.float64), m, n, x.astype(np.float64))
        tol = fixed_point_tol(c.astype(np.float64), x.astype(np.float64), n, w) + 2.0 ** -23 * np.abs(ref)
        assert np.all(np.abs(y.cpu().numpy().astype(np.float64) - ref) <= tol)
    x = (rs.standard_normal(n) * 10.0 ** rs.uniform(-6, 0, n)).astype(np.float32)
    y = scd.scd_apply(dev_bits(S), dev_bits(T), torch.from_numpy(c).cuda(), m, n, torch.from_numpy(x).cuda())
    ref = oracle.apply(S, T, c.astype(np.float64), m, n, x.astype(np.float64))
    tol = fixed_point_tol(c.astype(np.float64), x.astype(np.float64), n, w) + 2.0 ** -23 * np.abs(ref)
    assert np.all(np.abs(y.cpu().numpy().astype(np.float64) - ref) <= tol)


def test_apply_several_vectors_and_empty_sum(scd, oracle):
    check(scd, oracle, 300, 200, 40, 5, np.float32, False, nvec=3)
    check(scd, oracle, 300, 200, 40, 6, np.float64, True, nvec=2)
    check(scd, oracle, 130, 70, 0, 7, np.float32, False)           # w = 0: y = 0
    check(scd, oracle, 130, 70, 0, 8, np.float64, True)


def test_apply_full_size_layer_width(scd, oracle):
    # 4096 x 4096 at the 50 % width of Table 2 (16320 terms): several chunks of terms per wave, 64 splits
    check(scd, oracle, 4096, 4096, 16320, 11, np.float32, False)
    check(scd, oracle, 1024, 4096, 6512, 12, np.float32, True)


def test_apply_reproduces_a_minus_remainder(scd):
    # (A - R_w) x from the factors the decomposition itself returned (definition, Section 1)
    g = torch.Generator(device="cuda")
    g.manual_seed(3)
    A = torch.randn(1000, 520, generator=g, device="cuda")
    with scd.ScdContext(A, 40, 4) as ctx:
        ctx.run(40)
        res = ctx.results()
        R = ctx.remainder()
    x = torch.randn(520, generator=g, device="cuda")
    y = scd.scd_apply(res["signs"][0], res["signs"][1], res["c"], 1000, 520, x)
    ref = (A.double() - R.double()) @ x.double()
    assert float((y.double() - ref).abs().max()) <= 2e-5 * float(ref.abs().max())
    xt = torch.randn(1000, generator=g, device="cuda")
    yt = scd.scd_apply(res["signs"][0], res["signs"][1], res["c"], 1000, 520, xt, transpose=True)
    reft = (A.double() - R.double()).T @ xt.double()
    assert float((yt.double() - reft).abs().max()) <= 2e-5 * float(reft.abs().max())


def test_apply_rejects_bad_arguments(scd):
    L = scd.lib()
    S, T, c = random_factors(128, 128, 4, 1, np.float32)
    Sd, Td, cd = dev_bits(S), dev_bits(T), torch.from_numpy(c).cuda()
    x = torch.zeros(128, device="cuda")
    y = torch.zeros(128, device="cuda")
    need = L.scd_apply_workspace_bytes(128, 128, 4)
    assert need > 0
    ws = torch.empty(need // 8 + 1, dtype=torch.float64, device="cuda")
    p = lambda t: C.c_void_p(t.data_ptr())  # noqa: E731
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert L.scd_apply(p(Sd), p(Td), p(cd), 0, 128, 128, 4, 0, p(x), 1, p(y), p(ws), need - 8, st) == -1   # too small
    assert L.scd_apply(p(Sd), p(Td), p(cd), 0, 128, 128, 4, 0, p(x), 1, p(y), None, need, st) == -1
    assert L.scd_apply(None, p(Td), p(cd), 0, 128, 128, 4, 0, p(x), 1, p(y), p(ws), need, st) == -1
    assert L.scd_apply(p(Sd), p(Td), p(cd), 0, -1, 128, 4, 0, p(x), 1, p(y), p(ws), need, st) == -1
    assert L.scd_apply(p(Sd), p(Td), p(cd), 7, 128, 128, 4, 0, p(x), 1, p(y), p(ws), need, st) == -1
    assert L.scd_apply(p(Sd), p(Td), p(cd), 0, 128, 128, 4, 0, p(x), 1, p(y), p(ws), need, st) == 0
    with pytest.raises(ValueError):
        scd.scd_apply(Sd, Td, cd, 128, 128, torch.zeros(100, device="cuda"))


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_apply_non_finite_input_gives_nan(scd, dtype):
    S, T, c = random_factors(130, 200, 9, 3, dtype)
    x = np.ones(200, dtype=dtype)
    x[77] = np.inf
    y = scd.scd_apply(dev_bits(S), dev_bits(T), torch.from_numpy(c).cuda(), 130, 200, torch.from_numpy(x).cuda())
    assert bool(torch.isnan(y).all())
    # zeros and a tiny vector pass through the fixed point unharmed
    z = scd.scd_apply(dev_bits(S), dev_bits(T), torch.from_numpy(c).cuda(), 130, 200,
                      torch.zeros(200, dtype=torch.from_numpy(c).dtype, device="cuda"))
    assert float(z.abs().max()) == 0.0
