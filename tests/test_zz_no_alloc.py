"""The column half step that allocates nothing (scd_col_signed_sum_noalloc) against the allocating entry
point it is a variant of: same kernels and geometry, so every output must be identical bit for bit.  Two
calls in a row share the library's fixed work space, the second with a smaller input: stale contents of the
first must not leak into it."""
import numpy as np
import pytest
import torch

from helpers import to_dev_bits, to_np_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def scd():
    from paper_2410_01799_amd import scd as mod

    mod.lib()
    assert torch.cuda.is_available()
    return mod


def gauss(shape, seed, dtype):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape).astype(dtype)


def both(scd, oracle, m, n, dtype, seed):
    R = torch.from_numpy(gauss((m, n), seed, dtype)).cuda()
    s = to_dev_bits(oracle.rng_signs(seed, 0, 0, m))
    v0, t0, c0 = scd.scd_col_signed_sum(R, s)
    v1 = torch.full((n,), float("nan"), dtype=torch.float64, device="cuda")
    t1 = torch.full(((n + 63) // 64,), -1, dtype=torch.int64, device="cuda")
    c1 = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda")
    scd.scd_col_signed_sum_noalloc(R, s, v1, t1, c1)
    torch.cuda.current_stream().synchronize()
    return (v0, t0, c0), (v1, t1, c1), R, s


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_noalloc_matches_allocating_entry_point_twice(scd, oracle, dtype):
    # first call: several tiles and a ragged tail; second call: smaller, on the same work space
    for (m, n, seed) in [(1500, 2070, 11), (300, 517, 12)]:
        (v0, t0, c0), (v1, t1, c1), R, s = both(scd, oracle, m, n, dtype, seed)
        assert torch.equal(v0, v1), (m, n)
        assert torch.equal(t0, t1), (m, n)
        assert torch.equal(c0, c1), (m, n)
        # and against the oracle, to the bar of the other half-step tests
        v_ref = oracle.col_signed_sum(R.cpu().numpy().astype(np.float64), to_np_bits(s))
        tol = 2e-6 if dtype == np.float32 else 1e-13
        np.testing.assert_allclose(v1.cpu().numpy(), v_ref, rtol=0, atol=tol * np.abs(v_ref).max())
        assert float(c1) == pytest.approx(np.abs(v_ref).sum(), rel=1e-5)


def test_noalloc_optional_outputs_and_limit(scd, oracle):
    (v0, t0, c0), _, R, s = both(scd, oracle, 640, 1000, np.float32, 13)
    t1 = torch.zeros_like(t0)
    scd.scd_col_signed_sum_noalloc(R, s, None, t1, None)
    torch.cuda.current_stream().synchronize()
    assert torch.equal(t0, t1)
    # the headline shape fits the fixed work space (1024 workgroups x 4096 columns x 4 bytes = 16 MiB)
    A = torch.randn(4096, 4096, device="cuda")
    sb = to_dev_bits(oracle.rng_signs(1, 0, 0, 4096))
    vb = torch.empty(4096, dtype=torch.float64, device="cuda")
    tb = torch.zeros(64, dtype=torch.int64, device="cuda")
    cb = torch.zeros(1, dtype=torch.float64, device="cuda")
    scd.scd_col_signed_sum_noalloc(A, sb, vb, tb, cb)
    torch.cuda.current_stream().synchronize()
    va, ta, ca = scd.scd_col_signed_sum(A, sb)
    assert torch.equal(va, vb) and torch.equal(ta, tb) and torch.equal(ca, cb)
    # its f64 copy does not: refused before anything is enqueued
    with pytest.raises(scd.ScdError) as e:
        scd.scd_col_signed_sum_noalloc(A.double(), sb, vb, tb, cb)
    assert e.value.code == scd.ETOOBIG
