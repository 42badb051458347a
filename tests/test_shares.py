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


def test_a_stream_of_jobs_runs_all_of_them_within_the_device_and_the_limit():
    # the scheduler of the model run with a stand-in for the decomposition: every job runs exactly once, never more
    # than `concurrency` at a time, the shares in flight never exceed the device, streams are handed on
    import threading
    import time

    from paper_2410_01799_amd.shares import run_stream_of_jobs

    jobs = [dict(id=100 + j, m=LAYER[j % 7][0], n=LAYER[j % 7][1], left=LAYER[j % 7][2], alt=40.0) for j in range(23)]
    jobs.append(dict(id=999, m=32000, n=4096, left=29023, alt=30.0))
    board = ShareBoard()
    lock = threading.Lock()
    in_flight, seen, worst = set(), [], [0, 0]
    streams = [object() for _ in range(8)]

    def run_one(job, share_fn, progress_fn, stream):
        with lock:
            assert stream not in in_flight
            in_flight.add(stream)
            seen.append(job["id"])
            worst[0] = max(worst[0], len(in_flight))
        for step in range(3):
            g = share_fn() or 256
            assert g >= min_share(job["m"], job["n"])
            with board.lock:
                worst[1] = max(worst[1], sum(board.shares.values()))
            time.sleep(0.002 * (1 + job["id"] % 3))
            progress_fn(job["left"] * (2 - step) // 3, 38.0)
        with lock:
            in_flight.discard(stream)
        return dict(id=job["id"], share=g)

    res = run_stream_of_jobs(jobs, 8, 32, run_one, streams, board=board)
    assert sorted(seen) == sorted(j["id"] for j in jobs) and len(res["rows"]) == len(jobs)
    assert not res["failures"] and not res["not_started"]
    assert worst[0] <= 8 and res["most_in_flight"] <= 8 and worst[1] <= 256
    assert board.shares == {} and board.jobs == {}
    # a failing job is reported, nothing new is started after it, and the call still returns
    def boom(job, share_fn, progress_fn, stream):
        if job["id"] == 103:
            raise RuntimeError("no")
        time.sleep(0.001)
        return dict(id=job["id"])

    res = run_stream_of_jobs(jobs, 4, 32, boom, streams[:4])
    assert [f[0] for f in res["failures"]] == [103] and res["not_started"]
    # a budget that is already spent starts nothing
    res = run_stream_of_jobs(jobs, 4, 32, boom, streams[:4], budget_seconds=-1.0)
    assert len(res["not_started"]) == len(jobs) and not res["rows"]
