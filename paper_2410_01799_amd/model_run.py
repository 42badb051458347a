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
import sys
import time
from pathlib import Path

import torch

from . import scd, workloads


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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--start", type=int, default=0)
    ap.add_argument("--stop", type=int, default=226)
    ap.add_argument("--out", type=str, required=True)
    ap.add_argument("--budget-seconds", type=float, default=1e9, help="stop before a matrix that would overrun")
    args = ap.parse_args()
    man = workloads.config5_manifest()
    out = Path(args.out)
    out.parent.mkdir(parents=True, exist_ok=True)
    t_begin = time.perf_counter()
    last = 0.0
    with out.open("a") as fh:
        for idx in range(args.start, min(args.stop, len(man))):
            if time.perf_counter() - t_begin + 1.2 * last > args.budget_seconds:
                break
            e = man[idx]
            m, n = e["m"], e["n"]
            A = device_weight_like(m, n, e["seed"], e["kind"])
            w = e["widths"]["1/2"]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            with scd.ScdContext(A, w, e["seed"]) as ctx:
                ctx.run(w)
                res = ctx.results()
                eng = ctx.engine()["engine"]
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            last = dt
            tr = res["trace"].double()
            c = res["c"].double()
            ident = ((tr[1:] ** 2 - (tr[:-1] ** 2 - m * n * c ** 2)).abs() / tr[:-1] ** 2).max().item()
            rel = {p: float(tr[e["widths"][p]] / tr[0]) for p in ("1/4", "3/8", "1/2")}
            row = dict(index=idx, name=e["name"], m=m, n=n, seed=e["seed"], width=w, seconds=round(dt, 3),
                       terms_per_s=round(w / dt, 1), alternations_per_term=round(float(res["iters"].float().mean()), 2),
                       rel_err=rel, identity_max_violation=ident, engine=eng)
            fh.write(json.dumps(row) + "\n")
            fh.flush()
            print(f"[{idx}] {e['name']} {m}x{n} w={w}: {dt:.1f} s, {w / dt:.0f} terms/s, rel err 1/4 {rel['1/4']:.4f} "
                  f"3/8 {rel['3/8']:.4f} 1/2 {rel['1/2']:.4f}", flush=True)
            del A, res
    return 0


if __name__ == "__main__":
    sys.exit(main())
