"""The give-up path of the persistent engines, forced from the host: with a spin limit of zero every bounded
wait in the kernel expires at its first stale read, every workgroup leaves normally, the call reports
SCD_ETIMEOUT, the context keeps the terms it had and refuses further steps until it is given a remainder
again; after that it continues exactly like a context that never failed."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def scd():
    from paper_2410_01799_amd import scd as mod

    mod.lib()
    return mod


def gauss(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape).astype(np.float32)


@pytest.mark.parametrize("name,opts,engine", [("resident", {"resident": 1}, 1),
                                              ("sparse", {"resident": 0, "sparse_min_mib": 0}, 2),
                                              ("sparse-immediate", {"resident": 0, "sparse_min_mib": 0, "sparse_delay_width": 0}, 2),
                                              ("persistent-stream", {"resident": 0, "sparse": 0}, 3)])
def test_a_wait_that_runs_out_is_reported_and_the_context_recovers(scd, name, opts, engine):
    A = torch.from_numpy(gauss((1024, 1024), 31)).cuda()
    seed, w = 8, 6
    # the reference: a context that runs the same two launches (2 terms, then 4) and never fails
    with scd.ScdContext(A, w, seed, options=opts) as good:
        assert good.engine()["engine"] == engine
        good.run(2)
        good.run(4)
        want = good.results()
    with scd.ScdContext(A, w, seed, options=opts) as ctx:
        ctx.run(2)
        R2 = ctx.remainder()
        before = ctx.results()
        ctx.set_option("max_spin", 0)
        ctx.set_option("poll_delay", 0)
        with pytest.raises(scd.ScdError) as e:
            ctx.run(4)
        assert e.value.code == scd.ETIMEOUT
        # nothing of the failed launch is reported; the terms before it are intact
        assert ctx.width == 2
        after = ctx.results()
        for k in ("c", "trace", "iters"):
            assert torch.equal(before[k], after[k])
        assert torch.equal(before["signs"][0], after["signs"][0]) and torch.equal(before["signs"][1], after["signs"][1])
        # the context refuses to go on, with the same code, until it gets a remainder
        for call in (lambda: ctx.run(1), ctx.step, ctx.remainder):
            with pytest.raises(scd.ScdError) as e:
                call()
            assert e.value.code == scd.ETIMEOUT
        ctx.set_option("max_spin", 1 << 22)
        ctx.set_option("poll_delay", 16)
        ctx.set_remainder(R2)
        assert ctx.engine()["engine"] == engine
        ctx.run(4)
        got = ctx.results()
    assert torch.equal(want["signs"][0], got["signs"][0]) and torch.equal(want["signs"][1], got["signs"][1])
    assert torch.equal(want["c"], got["c"]) and torch.equal(want["iters"], got["iters"])
    # trace[2] was measured again by a pass of another kind after scd_set_remainder
    np.testing.assert_allclose(want["trace"].cpu().numpy(), got["trace"].cpu().numpy(), rtol=1e-8)


def test_option_values_are_checked(scd):
    A = torch.from_numpy(gauss((64, 64), 1)).cuda()
    with scd.ScdContext(A, 2, 0) as ctx:
        assert ctx.get_option("sparse_delay_width") == 8 and ctx.get_option("resident") == 1
        for name, bad in (("resident", 2), ("sparse_delay_width", 3), ("sparse_delay_width", 33), ("poll_delay", -1),
                          ("sweep_batch", 0), ("max_spin", -5)):
            with pytest.raises(scd.ScdError) as e:
                ctx.set_option(name, bad)
            assert e.value.code == scd.EINVAL
        assert scd.lib().scd_set_option(ctx._h, 99, 1) == scd.EINVAL
        ctx.set_option("sparse_delay_width", 32)
        assert ctx.get_option("sparse_delay_width") == 32
