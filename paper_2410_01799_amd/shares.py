"""Shares of the device for decompositions that run side by side (the matrices of a layer or a model are
independent, Section 4.2, and one greedy decomposition is bound by the latency of its alternations).

Host-side scheduling only: no arithmetic of the method.  An alternation of the sparse engine on `g` workgroups
costs about ``L + W / g`` microseconds (measured alone on the device, 14336 x 4096 f32: 31.6 us on 32 workgroups,
21.0 on 64, 16.0 on 128, 14.5 on 256: L = 10 us, W = 680 us x workgroups; 4096 x 4096: 12.7 / 10.8 / 10.2 / 10.5,
W = 120; 1024 x 4096: 14.3 / 11.7 / 11.0, W = 170), so small shares do more work per compute unit and as many
matrices as possible should be in flight.  Shares are powers of two (slices of whole multiples of 8 rows make
the cost a step function of the share, with its steps there).  Given what every matrix in flight has left
(terms x alternations per term), the board starts every job at the smallest share its shape allows and keeps
doubling the share of the job that would finish last, while the device has room.
"""
from __future__ import annotations

import threading
import time
from typing import Callable, Dict, List, Optional

LATENCY_US = 10.0
DEVICE = 256


def work_us(m: int, n: int) -> float:
    """W of the cost model for an m x n f32 matrix (microseconds x workgroups per alternation)."""
    return {(14336, 4096): 680.0, (4096, 14336): 700.0, (4096, 4096): 120.0, (1024, 4096): 170.0}.get((m, n), 0.035 * (m + n))


def min_share(m: int, n: int) -> int:
    """Smallest share the sparse engine runs an m x n matrix on: slices of at most 512 rows and columns."""
    g = 16
    while g < DEVICE and max(m, n) > 512 * g:
        g *= 2
    return g


class ShareBoard:
    """Shares that only ever grow, and only into room that a finished job has left: a launch then never has to
    wait for room on the device (a persistent launch needs all its workgroups resident at once, so the library
    holds back a launch that does not fit beside the others), whatever the moment at which each job reaches its
    next launch boundary.  All jobs of a batch are registered before the first launch."""

    def __init__(self, device: int = DEVICE):
        self.device = device
        self.lock = threading.Lock()
        self.jobs: Dict[int, dict] = {}
        self.shares: Dict[int, int] = {}

    def register(self, jobs: Dict[int, dict]) -> None:
        """jobs: {id: dict(m, n, left, alt)}: the first shares, for all of them at once."""
        with self.lock:
            self.jobs = {k: dict(v) for k, v in jobs.items()}
            self.shares = solve_shares(self.jobs, self.device)

    def admit(self, job: int, info: dict, target: int = 0) -> bool:
        """A further job, if the room that is free now holds the smallest share its shape allows.  It gets the
        largest power of two that fits the room, or at most `target` (if given and its shape allows so little):
        a stream of waiting jobs then fills the device with many small shares, which do the most work per
        compute unit."""
        with self.lock:
            room = self.device - sum(self.shares.values())
            g = min_share(info["m"], info["n"])
            if g > room:
                return False
            while 2 * g <= room and (target <= 0 or 2 * g <= target):
                g *= 2
            self.jobs[job] = dict(info)
            self.shares[job] = g
            return True

    def release(self, job: int) -> None:
        """A finished job leaves; its room stays free until admit() or grow() hands it out."""
        with self.lock:
            self.jobs.pop(job, None)
            self.shares.pop(job, None)

    def grow(self) -> None:
        with self.lock:
            self._grow()

    def progress(self, job: int, terms_left: int, alternations_per_term: float) -> None:
        with self.lock:
            j = self.jobs[job]
            j["left"], j["alt"] = terms_left, max(2.0, alternations_per_term)

    def finish(self, job: int) -> None:
        with self.lock:
            self.jobs.pop(job, None)
            self.shares.pop(job, None)
            self._grow()

    def share(self, job: int) -> int:
        """Workgroups for the next launch of this job (0 = the whole device)."""
        with self.lock:
            g = self.shares.get(job, 0)
        return 0 if g >= self.device else g

    def _grow(self) -> None:
        def seconds(k):
            j = self.jobs[k]
            return j["left"] * j["alt"] * alternation_us(j["m"], j["n"], self.shares[k]) * 1e-6

        while True:
            room = self.device - sum(self.shares.values())
            grown = False
            for k in sorted(self.shares, key=lambda k: -seconds(k)):
                if self.shares[k] <= room and 2 * self.shares[k] <= self.device:
                    self.shares[k] *= 2
                    grown = True
                    break
            if not grown:
                return


def solve_shares(jobs: Dict[int, dict], device: int = DEVICE) -> Dict[int, int]:
    """Shares for jobs {id: dict(m, n, left (terms), alt (alternations per term))}: every job starts at the smallest
    share its shape allows; the share of the job that would finish last is doubled while the device has room."""
    act = {k: dict(w=work_us(v["m"], v["n"]), lo=min_share(v["m"], v["n"]), left=v["left"], alt=v["alt"])
           for k, v in jobs.items() if v["left"] > 0}
    if len(act) <= 1:
        return {k: device for k in act}

    def seconds(j, g):
        return j["left"] * j["alt"] * (LATENCY_US + j["w"] / g) * 1e-6

    new = {k: v["lo"] for k, v in act.items()}
    while True:
        room = device - sum(new.values())
        grown = False
        for k in sorted(act, key=lambda k: -seconds(act[k], new[k])):
            if new[k] <= room and 2 * new[k] <= device:
                new[k] *= 2
                grown = True
                break
        if not grown:
            return new


def alternation_us(m: int, n: int, g: int) -> float:
    """Cost model: microseconds per alternation of an m x n matrix on g workgroups."""
    return LATENCY_US + work_us(m, n) / g


def run_stream_of_jobs(jobs: List[dict], concurrency: int, target_share: int, run_one: Callable, streams: List,
                       budget_seconds: float = float("inf"), guess_seconds: Optional[Callable] = None,
                       on_done: Optional[Callable] = None, board: Optional[ShareBoard] = None) -> dict:
    """Run `jobs` (dicts with id, m, n, left, alt; in this order) with at most `concurrency` in flight, each on a
    share of the device: a waiting job starts as soon as room that is free holds its share (`target_share`, or what
    its shape needs; the last waiting job takes all the room there is), and room no waiting job can use goes to the
    job that would finish last.  `run_one(job, share_fn, progress_fn, stream)` does the work on one of `streams`
    (one per job in flight, handed from a finished job to the next: on the GPU a stream made later would share a
    hardware queue with a busy one) and returns a row; `share_fn()` gives the share for the next launch (0 = the
    whole device), `progress_fn(terms left, alternations per term)` feeds the board.  No job is started once
    `guess_seconds(job)` more would overrun `budget_seconds`.  Returns dict(rows, not_started, failures, wall_seconds,
    most_in_flight)."""
    assert len(streams) >= concurrency >= 1
    board = board or ShareBoard()
    cv = threading.Condition()
    todo = list(jobs)
    free = list(streams)
    running: Dict[int, threading.Thread] = {}
    rows, failures = [], []
    t_begin = time.perf_counter()
    most = [0]

    def worker(job, stream):
        jid = job["id"]
        try:
            row = run_one(job, lambda: board.share(jid), lambda left, alt: board.progress(jid, left, alt), stream)
        except Exception as err:  # noqa: BLE001 - handed to the caller
            row = None
            with cv:
                failures.append((jid, repr(err)))
        with cv:
            if row is not None:
                rows.append(row)
                if on_done:
                    on_done(row)
            board.release(jid)  # the room stays free until the loop below has tried the waiting jobs
            free.append(stream)
            running.pop(jid, None)
            cv.notify_all()

    with cv:
        while True:
            while todo and not failures and len(running) < concurrency:
                job = todo[0]
                ahead = guess_seconds(job) if guess_seconds else 0.0
                if time.perf_counter() - t_begin + ahead > budget_seconds:
                    break
                info = dict(m=job["m"], n=job["n"], left=job["left"], alt=job.get("alt", 40.0))
                if not board.admit(job["id"], info, target_share if len(todo) > 1 else 0):
                    break
                todo.pop(0)
                t = threading.Thread(target=worker, args=(job, free.pop()))
                running[job["id"]] = t
                most[0] = max(most[0], len(running))
                t.start()
            board.grow()
            if not running:
                break
            cv.wait()
    return dict(rows=rows, not_started=todo, failures=failures, wall_seconds=time.perf_counter() - t_begin,
                most_in_flight=most[0])
