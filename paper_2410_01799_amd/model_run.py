"""Decompose the synthetic Mistral-7B-shaped weight set (workload 5: 226 matrices) matrix by matrix.

Resumable: ``python -m paper_2410_01799_amd.model_run --start 0 --stop 80 --out gpurun_out/model/part0.jsonl``
writes one JSON line per matrix; several invocations cover the manifest.  Each matrix is decomposed once, to
the width of 50 % of its bf16 footprint; the errors at 25 % and 37.5 % are read off the same run at the
narrower widths (a greedy run contains every narrower run as a prefix).  Matrices are generated on the GPU
from a seeded torch generator with the recipe of ``workloads.weight_like_matrix`` (the numpy recipe is used
where a CPU oracle has to see the same values; nothing here is compared with the oracle).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from pathlib import Path

# matrices side by side need a hardware queue each (HIP's default is four per process); read when HIP starts,
# so the command line is looked at before torch is imported
_queues = 8
if "--hw-queues" in sys.argv[:-1]:
    _queues = max(4, min(32, int(sys.argv[sys.argv.index("--hw-queues") + 1])))
if int(os.environ.get("GPU_MAX_HW_QUEUES", "0") or 0) < _queues:
    os.environ["GPU_MAX_HW_QUEUES"] = str(_queues)

import torch  # noqa: E402

from . import scd, workloads
from .shares import run_stream_of_jobs


def device_weight_like(m: int, n: int, seed: int, kind: str) -> torch.Tensor:
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    G = torch.randn(m, n, generator=g, device="cuda", dtype=torch.float32) * 0.02
    if kind == "weight":
        U = torch.randn(m, 16, generator=g, device="cuda", dtype=torch.float32)
        V = torch.randn(n, 16, generator=g, device="cuda", dtype=torch.float32)
        L = U @ V.T
        a = torch.sqrt(0.1 / 0.9 * G.double().square().sum() / L.double().square().sum()).float()
        G += a * L
        del L
        cols = torch.randperm(n, generator=g, device="cuda")[: n // 100]
        G[:, cols] *= 8.0
    return G.bfloat16().float().contiguous()   # bf16-representable values, stored as f32


def decompose_one(e: dict, share_fn, chunk: int, progress_fn=None) -> dict:
    """One matrix of the manifest on the current stream; returns its result row.  share_fn() says, before every
    launch, how many compute units this matrix may take (0 = all); progress_fn(terms left, alternations per term)
    is told after every launch."""
    m, n = e["m"], e["n"]
    A = device_weight_like(m, n, e["seed"], e["kind"])
    w = e["widths"]["1/2"]
    torch.cuda.current_stream().synchronize()
    t0 = time.perf_counter()
    with scd.ScdContext(A, w, e["seed"]) as ctx:
        share_now, shares_used = 0, [256]
        # launches of bounded length, so that the split of the device can follow the matrices in flight
        for k in range(0, w, chunk):
            want = share_fn()
            if want != share_now:
                ctx.set_workgroups(want)
                share_now = want
                shares_used.append(want or 256)
            done = min(chunk, w - k)
            ctx.run(done)
            if progress_fn is not None:
                progress_fn(w - k - done, ctx.traffic()["passes"] / (k + done))
        if len(shares_used) > 1:
            shares_used = shares_used[1:]
        res = ctx.results()
        eng = ctx.engine()["engine"]
        torch.cuda.current_stream().synchronize()
        dt = time.perf_counter() - t0
    tr = res["trace"].double()
    c = res["c"].double()
    ident = ((tr[1:] ** 2 - (tr[:-1] ** 2 - m * n * c ** 2)).abs() / tr[:-1] ** 2).max().item()
    rel = {p: float(tr[e["widths"][p]] / tr[0]) for p in ("1/4", "3/8", "1/2")}
    return dict(index=e["index"], name=e["name"], m=m, n=n, seed=e["seed"], width=w, seconds=round(dt, 3),
                terms_per_s=round(w / dt, 1), alternations_per_term=round(float(res["iters"].float().mean()), 2),
                rel_err=rel, identity_max_violation=ident, engine_at_the_end=eng, workgroups=shares_used)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--start", type=int, default=0)
    ap.add_argument("--stop", type=int, default=226)
    ap.add_argument("--out", type=str, required=True)
    ap.add_argument("--budget-seconds", type=float, default=1e9, help="take no new matrix that would overrun")
    ap.add_argument("--concurrency", type=int, default=1, choices=list(range(1, 17)),
                    help="most matrices decomposed side by side (the matrices of a model are independent, and one "
                         "decomposition is latency-bound); every one gets a share of the compute units")
    ap.add_argument("--share", type=int, default=32,
                    help="workgroups a newly started matrix gets when others wait behind it (more if its shape needs "
                         "more); room that no waiting matrix can use goes to the matrix that would finish last")
    ap.add_argument("--chunk", type=int, default=512, help="terms per launch when matrices run side by side")
    ap.add_argument("--hw-queues", type=int, default=8, help="hardware queues of the process (one per matrix in flight)")
    args = ap.parse_args()
    man = workloads.config5_manifest()
    for i, e in enumerate(man):
        e["index"] = i
    todo = list(range(args.start, min(args.stop, len(man))))
    out = Path(args.out)
    out.parent.mkdir(parents=True, exist_ok=True)
    K = args.concurrency
    chunk = 1 << 30 if K == 1 else args.chunk
    t_begin = time.perf_counter()
    cost: dict = {}      # (m, n) -> seconds the last matrix of that shape took
    scd.lib()
    torch.cuda.set_device(0)
    jobs = [dict(id=i, m=man[i]["m"], n=man[i]["n"], left=man[i]["widths"]["1/2"], alt=40.0) for i in todo]

    with out.open("a") as fh:
        def report(row):
            cost[(row["m"], row["n"])] = row["seconds"]
            fh.write(json.dumps(row) + "\n")
            fh.flush()
            rel = row["rel_err"]
            print(f"[{row['index']}] {row['name']} {row['m']}x{row['n']} w={row['width']}: "
                  f"{row['seconds']:.1f} s, {row['terms_per_s']:.0f} terms/s on {row['workgroups']} workgroups, "
                  f"rel err 1/4 {rel['1/4']:.4f} 3/8 {rel['3/8']:.4f} 1/2 {rel['1/2']:.4f}", flush=True)

        def guess(job):
            return 1.2 * cost.get((job["m"], job["n"]), 0.0)

        failures = []
        if K == 1:
            while jobs:
                if time.perf_counter() - t_begin + guess(jobs[0]) > args.budget_seconds:
                    break
                report(decompose_one(man[jobs.pop(0)["id"]], lambda: 0, chunk))
            left = jobs
        else:
            def run_one(job, share_fn, progress_fn, stream):
                torch.cuda.set_device(0)
                with torch.cuda.stream(stream):
                    return decompose_one(man[job["id"]], share_fn, chunk, progress_fn)

            # one stream per matrix in flight, made once and handed from a finished matrix to the next: streams made
            # later would share a hardware queue with one that is busy, and every launch of theirs would wait for a
            # whole launch of the other matrix
            res = run_stream_of_jobs(jobs, K, args.share, run_one, [torch.cuda.Stream() for _ in range(K)],
                                     budget_seconds=args.budget_seconds, guess_seconds=guess, on_done=report)
            left, failures = res["not_started"], res["failures"]
        torch.cuda.synchronize()
        wall = time.perf_counter() - t_begin
        nxt = left[0]["id"] if left else None
        fh.write(json.dumps(dict(summary=True, start=args.start, next_index=nxt, concurrency=K,
                                 wall_seconds=round(wall, 2))) + "\n")
    print(f"wall {wall:.1f} s, next index {nxt}", flush=True)
    if failures:
        print(f"failed: {failures}", file=sys.stderr)
        return 1
    return 0


if __name__ == "__main__":
    sys.exit(main())
