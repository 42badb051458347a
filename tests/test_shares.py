"""Host logic that shares the device out among decompositions in flight (no GPU)."""
from paper_2410_01799_amd.shares import ShareBoard, min_share, solve_shares

LAYER = [(4096, 4096, 16320), (1024, 4096, 6512), (1024, 4096, 6512), (4096, 4096, 16320), (14336, 4096, 25442),
         (14336, 4096, 25442), (4096, 14336, 25442)]


def info(i):
    m, n, w = LAYER[i]
    return dict(m=m, n=n, left=w, alt=40.0)


def test_min_share_follows_the_slice_limit():
    assert min_share(1024, 4096) == 16 and min_share(4096, 4096) == 16
    assert min_share(14336, 4096) == 32 and min_share(4096, 14336) == 32 and min_share(32000, 4096) == 64


def test_first_shares_fit_the_device_and_favour_the_job_that_ends_last():
    sh = solve_shares({i: info(i) for i in range(7)})
    assert sum(sh.values()) <= 256 and all(g >= min_share(*LAYER[i][:2]) for i, g in sh.items())
    assert all(g & (g - 1) == 0 for g in sh.values())            # powers of two
    assert sh[4] >= sh[0] >= sh[1]                               # the large matrices get the most
    assert solve_shares({3: info(3)}) == {3: 256}


def test_shares_only_grow_and_only_into_free_room():
    b = ShareBoard()
    b.register({i: info(i) for i in range(7)})
    before = dict(b.shares)
    for left in (6000, 3000, 100):                               # progress alone never moves a share
        for i in range(7):
            b.progress(i, left, 38.0)
        assert b.shares == before
    for gone in (2, 1, 0, 3):
        prev = dict(b.shares)
        b.finish(gone)
        assert gone not in b.shares and sum(b.shares.values()) <= 256
        assert all(b.shares[k] >= prev[k] for k in b.shares)     # nobody shrinks: no launch ever waits for room
    b.finish(4)
    b.finish(5)
    assert b.share(6) == 0                                       # the last job has the whole device
    b.finish(6)
    assert b.shares == {}


def test_a_waiting_job_is_admitted_into_free_room_only():
    b = ShareBoard()
    b.register({i: info(i) for i in (4, 5, 6, 0)})
    assert not b.admit(3, info(3)) or sum(b.shares.values()) <= 256
    b.jobs.pop(0), b.shares.pop(0)
    assert b.admit(3, info(3)) and sum(b.shares.values()) <= 256


def test_a_stream_of_waiting_jobs_fills_the_device_with_small_shares():
    # the model run: jobs admitted one by one with a target share while others wait behind them
    b = ShareBoard()
    order = [0, 1, 2, 3, 4, 5, 6, 0, 1, 2]
    started = []
    for j, i in enumerate(order):
        if len(started) < 8 and b.admit(100 + j, info(i), 32):
            started.append(100 + j)
    b.grow()
    assert len(started) == 8 and sum(b.shares.values()) <= 256
    assert all(g == 32 for g in b.shares.values())               # eight times 32: nothing left to grow into
    b.release(started[1])                                        # a finished job leaves room for exactly one more
    assert sum(b.shares.values()) == 224
    assert b.admit(200, info(4), 32) and b.shares[200] == 32
    b.release(started[0])
    b.release(started[2])
    assert b.admit(201, dict(m=32000, n=4096, left=29023, alt=30.0), 32) and b.shares[201] == 64   # its shape needs 64
    b.grow()
    assert sum(b.shares.values()) <= 256
