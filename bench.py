#!/usr/bin/env python3
"""Benchmark of the signed cut decomposition hot path on one MI355X.

A step is one whole greedy decomposition (every hot-path stage: start, row passes, reductions,
termination, fused updates, appends) of the headline workload: a 4096x4096 f32 matrix with i.i.d.
N(0,1) entries taken to width 8192.  The input is resident in HBM before the timed region.
Prints ONE JSON line: terms/s, plus the roofline of the dominant kernel (the persistent register-resident
kernel, or the row pass of the launch-stream engine with --engine stream) and the CPU oracle timed on a
bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from pathlib import Path

# The layer figure runs up to seven decompositions side by side, each a persistent launch on its own stream.
# Streams that share a hardware queue run one after the other, and HIP's default is four queues per process:
# ask for eight before the runtime starts (read once, when the first HIP call initialises it).
if int(os.environ.get("GPU_MAX_HW_QUEUES", "0") or 0) < 8:
    os.environ["GPU_MAX_HW_QUEUES"] = "8"

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E bandwidth
FP32_VECTOR_PEAK_TFLOPS = 157.3  # MI355X published fp32 vector rate: 256 CUs x 128 lanes x 2 flop (FMA) x 2.4 GHz
# What add-only work without packed FP32 can issue: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-operations/s
# (one 64-lane instruction per SIMD every 4 cycles); packed FP32 is switched off on the test machines, and an add is
# one flop where the published rate counts two per FMA.
UNPACKED_LANE_OPS_PER_S = 256 * 64 * 2.4e9
TRAFFIC_FILE = ROOT / "profiles" / "memory_traffic_pmc.txt"
ENGINES = ["launch-stream", "register-resident", "sparse", "persistent-stream"]


def measured_traffic() -> dict:
    """HBM/fabric bytes from the committed rocprofv3 --pmc summary (FETCH_SIZE and WRITE_SIZE, each scaled by the
    plain copy kernel of known size): lines `TRAFFIC <key> <bytes> <per what>`.  Not measured by this run."""
    out = {}
    if TRAFFIC_FILE.exists():
        for line in TRAFFIC_FILE.read_text().splitlines():
            f = line.split()
            if len(f) >= 3 and f[0] == "TRAFFIC":
                out[f[1]] = float(f[2])
    return out


def cpu_baseline(A64, seed: int, budget_s: float):
    """The f64 oracle, as it stands, on the first terms of the same matrix; about `budget_s` seconds."""
    from oracle import scd_oracle as oracle

    oracle.build()
    threads = oracle.get_threads()
    t0 = time.perf_counter()
    oracle.decompose(A64, 1, seed)
    one = time.perf_counter() - t0
    terms = max(2, min(64, int(budget_s / max(one, 1e-3))))
    t0 = time.perf_counter()
    res = oracle.decompose(A64, terms, seed)
    dt = time.perf_counter() - t0
    return dict(value=terms / dt, unit="terms/s", cores=threads, kind="oracle",
                sample=f"first {terms} terms of the same 4096x4096 matrix in f64 ({dt:.1f} s, "
                       f"{float(res['iters'].mean()):.1f} alternations/term)")


def layer_mode(args, scd, workloads, torch, np) -> dict:
    """Seconds per decoder layer at 50 % of the bf16 size (workload 3): every matrix decomposed to its
    Table 2 width, all inputs resident in HBM before the timer starts.  With --concurrency K up to K of the
    seven matrices are in flight (largest first), each decomposition on its own stream and host thread, in
    launches of 512 terms; the compute units are shared out at the start so that the matrices in flight would
    finish together, and what a finished matrix leaves goes to the one that would finish last (shares.py).
    The figure is the wall time of the whole layer."""
    import threading

    from paper_2410_01799_amd.shares import ShareBoard

    K = args.concurrency
    jobs = []
    for name, M, wfull, seed in workloads.config3():
        jobs.append(dict(name=name, A=torch.from_numpy(M).cuda(), shape=list(M.shape), wfull=wfull, seed=seed,
                         w=max(1, int(round(wfull * args.layer_fraction)))))
    order = sorted(range(len(jobs)), key=lambda i: -jobs[i]["wfull"] * jobs[i]["shape"][0] * jobs[i]["shape"][1])
    rows, lock, errors = [None] * len(jobs), threading.Lock(), []
    board = ShareBoard()
    info = lambda i: dict(m=jobs[i]["shape"][0], n=jobs[i]["shape"][1], left=jobs[i]["w"], alt=40.0)
    first, waiting = order[:K], order[K:]
    board.register({i: info(i) for i in first})
    t_begin = [0.0]

    def worker(i):
        torch.cuda.set_device(0)
        stream = torch.cuda.Stream() if K > 1 else torch.cuda.current_stream()
        with torch.cuda.stream(stream):
            while i is not None:
                j = jobs[i]
                try:
                    t0 = time.perf_counter()
                    with scd.ScdContext(j["A"], j["w"], j["seed"]) as ctx:
                        step = j["w"] if K == 1 else 512
                        share_now, shares_used, busy_s = None, [], 0.0
                        for k in range(0, j["w"], step):
                            if K > 1:
                                want = board.share(i)
                                if want != share_now:
                                    ctx.set_workgroups(want)
                                    share_now = want
                                    shares_used.append(want or 256)
                            done = min(step, j["w"] - k)
                            ctx.run(done)
                            busy_s += ctx.engine()["last_launch_seconds"]
                            if K > 1:
                                board.progress(i, j["w"] - k - done, ctx.traffic()["passes"] / (k + done))
                        res = ctx.results()
                        eng = ctx.engine()["engine"]
                        stream.synchronize()
                        dt = time.perf_counter() - t0
                except Exception as err:  # noqa: BLE001 - reported by the main thread
                    with lock:
                        errors.append((j["name"], repr(err)))
                    board.finish(i)
                    return
                tr = res["trace"].cpu().numpy()
                it = res["iters"].cpu().numpy()
                rows[i] = {"matrix": j["name"], "shape": j["shape"], "width": j["wfull"], "terms_run": j["w"],
                           "started_at": round(t0 - t_begin[0], 3), "seconds": round(dt, 3),
                           "ended_at": round(t0 - t_begin[0] + dt, 3),
                           "terms_per_s": round(j["w"] / dt, 1),
                           "alternations_per_term": round(float(it.mean()), 2),
                           "relative_error": round(float(tr[-1] / tr[0]), 5),
                           "workgroups": shares_used if K > 1 else [256],
                           "seconds_inside_launches": round(busy_s, 3),
                           "engine_at_the_end": ENGINES[eng]}
                with lock:
                    # the next waiting matrix takes this one's place, before the room is given to the others
                    nxt = waiting.pop(0) if waiting and not errors else None
                    if nxt is not None:
                        board.jobs.pop(i, None)
                        board.shares.pop(i, None)
                        if not board.admit(nxt, info(nxt)):
                            waiting.insert(0, nxt)
                            nxt = None
                    board.finish(i)
                i = nxt

    torch.cuda.synchronize()
    t_begin[0] = time.perf_counter()
    if K == 1:
        for i in order:
            worker(i)
    else:
        threads = [threading.Thread(target=worker, args=(i,)) for i in first]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_begin[0]
    if errors or waiting:
        raise RuntimeError(f"layer run failed: {errors} (not started: {waiting})")
    total_terms = sum(j["wfull"] for j in jobs)
    total_s = wall / args.layer_fraction
    return {"metric": "seconds per Mistral-7B-shaped decoder layer at 50% of bf16 size", "value": round(total_s, 2),
            "unit": "s/layer", "n_gpus": 1, "higher_is_better": False, "dtype": "f32", "data": "synthetic",
            "extrapolated": args.layer_fraction < 1.0, "terms": total_terms, "concurrency": K,
            "compute_units_per_matrix": "shared out so that the matrices in flight finish together",
            "terms_per_s": round(total_terms / total_s, 1), "matrices": rows}


def apply_mode(args, scd, torch) -> int:
    """Microseconds per product of a decomposition with a vector, straight from the packed factors
    (Section 6.1), on random factors of the layer shapes at their 50 % widths; a plain f32 matrix-vector
    product of the same shape (torch) is timed beside it.  Wall-clock per product includes the host's three
    launches; the kernels' own durations are in profiles/."""
    rows = []
    L = scd.lib()
    for (m, n, w) in [(4096, 4096, 16320), (1024, 4096, 6512), (14336, 4096, 25442)]:
        g = torch.Generator(device="cuda")
        g.manual_seed(m + n)
        S = torch.randint(-2 ** 62, 2 ** 62, (w, (m + 63) // 64), device="cuda", generator=g)
        T = torch.randint(-2 ** 62, 2 ** 62, (w, (n + 63) // 64), device="cuda", generator=g)
        c = torch.randn(w, device="cuda", generator=g)
        reps = 20
        X = torch.randn(reps, n, device="cuda", generator=g)
        ws = torch.empty(L.scd_apply_workspace_bytes(m, n, w) // 8 + 1, dtype=torch.float64, device="cuda")
        scd.scd_apply(S, T, c, m, n, X, workspace=ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        scd.scd_apply(S, T, c, m, n, X, workspace=ws)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / reps
        A = torch.randn(m, n, device="cuda", generator=g)
        A @ X[0]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for r in range(reps):
            A @ X[r]
        torch.cuda.synchronize()
        dg = (time.perf_counter() - t0) / reps
        bits = w * ((m + 63) // 64 + (n + 63) // 64) * 8
        rows.append({"shape": [m, n], "width": w, "us_per_product": round(dt * 1e6, 1), "sign_bit_bytes": bits,
                     "sign_bits_gbs": round(bits / dt / 1e9, 1), "dense_f32_matvec_us": round(dg * 1e6, 1)})
    print(json.dumps({"metric": "microseconds per packed product y = (sum_j c_j s_j t_j^T) x", "unit": "us", "n_gpus": 1,
                      "dtype": "f32 in/out, int8 fixed-point sums joined in f64", "data": "synthetic", "products": rows}))
    return 0


def lsq_mode(args, scd, workloads, torch, np) -> int:
    """Terms/s of the least squares decomposition (Algorithm 6) beside the greedy one (Algorithm 5) from the
    same random starts, with the relative error each reaches."""
    rows = []
    for (m, n, w) in [(256, 256, 64), (1024, 1024, 512)]:
        A = torch.from_numpy(workloads.gaussian_matrix(m, n, 1, np.float32)).cuda()
        scd.scd_lsq_decompose(A, 4, 1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ls = scd.scd_lsq_decompose(A, w, 1)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        gr = scd.scd_decompose(A, w, 1)
        alts = int(ls["iters"].sum())
        rows.append({"shape": [m, n], "width": w, "seconds": round(dt, 3), "terms_per_s": round(w / dt, 1),
                     "us_per_alternation": round(dt / alts * 1e6, 1),
                     "relative_error_least_squares": round(float(ls["trace"][-1] / ls["trace"][0]), 6),
                     "relative_error_greedy": round(float(gr["trace"][-1] / gr["trace"][0]), 6)})
    print(json.dumps({"metric": "least squares decomposition (Algorithm 6) terms/s", "unit": "terms/s", "n_gpus": 1,
                      "dtype": "f32 input, f64 arithmetic", "data": "synthetic", "runs": rows}))
    return 0


def image_mode(args, scd, workloads, torch, np) -> int:
    """Workload 4: the 4000x3000x3 image-like tensor.  "RGB signs" (Algorithms 12/13, w = 129), "RGB scalars"
    (real last mode, w = 128) and, on a 1000x750x3 reduction, the least squares variant (Algorithm 14): seconds
    and the error at the logged widths in both normalisations of Section 5."""
    a_np, w_signs, seed = workloads.config4()
    a = torch.from_numpy(a_np).cuda()
    m, n, q = a_np.shape
    norm_a = float(np.linalg.norm(a_np.astype(np.float64)))
    norm_255 = 255.0 * (3.0 * m * n) ** 0.5

    def timed(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        r = fn()
        torch.cuda.synchronize()
        return r, time.perf_counter() - t0

    def curve(res, widths):
        tr = res["trace"].cpu().numpy()
        return {str(k): {"rel": round(float(tr[k] / norm_a), 5), "per_255": round(float(tr[k] / norm_255), 5)} for k in widths}

    rows = []
    scd.scd_decompose(a, 2, seed)
    res, dt = timed(lambda: scd.scd_decompose(a, w_signs, seed))
    rows.append({"variant": "RGB signs (Alg 12/13)", "width": w_signs, "packed_bytes": w_signs * (m + n + q + 32) // 8,
                 "seconds": round(dt, 3), "terms_per_s": round(w_signs / dt, 1),
                 "sweeps_per_term": round(float(res["iters"].float().mean()), 1), "error": curve(res, (8, 16, 32, 64, 129))})
    scd.scd_decompose_scalars(a, 2, seed)
    res, dt = timed(lambda: scd.scd_decompose_scalars(a, 128, seed))
    rows.append({"variant": "RGB scalars (real last mode)", "width": 128, "packed_bytes": 128 * (m + n + 96) // 8,
                 "seconds": round(dt, 3), "terms_per_s": round(128 / dt, 1),
                 "sweeps_per_term": round(float(res["iters"].float().mean()), 1), "error": curve(res, (8, 16, 32, 64, 128))})
    small = torch.from_numpy(workloads.image_like_tensor(1000, 750, 3, blobs=100, seed=400)).cuda()
    norm_s = float(small.double().norm())
    scd.scd_lsq_decompose(small, 2, seed)
    ls, dt = timed(lambda: scd.scd_lsq_decompose(small, 64, seed))
    gr = scd.scd_decompose(small, 64, seed)
    rows.append({"variant": "RGB signs + least squares (Alg 14) on 1000x750x3", "width": 64, "seconds": round(dt, 3),
                 "terms_per_s": round(64 / dt, 1), "rel_error_least_squares": round(float(ls["trace"][64]) / norm_s, 5),
                 "rel_error_greedy": round(float(gr["trace"][64]) / norm_s, 5)})
    print(json.dumps({"metric": "image-like tensor 4000x3000x3 f32 (workload 4)", "n_gpus": 1, "dtype": "f32", "data": "synthetic",
                      "runs": rows}))
    return 0


def oracle_mode(args, workloads, np) -> int:
    """The CPU oracle (plain f64, as it stands) timed on fixed prefixes of the workloads, with one thread and
    with all host cores: terms/s to quote beside the GPU figures.  No GPU work."""
    from oracle import scd_oracle as oracle

    oracle.build()
    all_cores = oracle.get_threads()
    cases = [("config 1: 256x256 N(0,1)", workloads.gaussian_matrix(256, 256, 1, np.float64), 64, 64, 1),
             ("config 2: 4096x4096 N(0,1)", workloads.gaussian_matrix(4096, 4096, 2, np.float64), 2, 32, 2),
             ("config 3: 14336x4096 weight-like", workloads.weight_like_matrix(14336, 4096, 300).astype(np.float64), 1, 8, 300)]
    rows = []
    for name, A, terms_one, terms_all, seed in cases:
        row = {"workload": name}
        for label, threads, terms in (("one_thread", 1, terms_one), ("all_cores", all_cores, terms_all)):
            oracle.set_threads(threads)
            t0 = time.perf_counter()
            res = oracle.decompose(A, terms, seed)
            dt = time.perf_counter() - t0
            row[label] = {"threads": threads, "terms": terms, "seconds": round(dt, 2), "terms_per_s": round(terms / dt, 3),
                          "alternations_per_term": round(float(res["iters"].mean()), 1)}
        rows.append(row)
    oracle.set_threads(all_cores)
    print(json.dumps({"metric": "CPU oracle terms/s (f64, first terms of each workload)", "unit": "terms/s", "kind": "oracle",
                      "host_cores": all_cores, "runs": rows}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--size", type=int, default=4096, help="matrix side (headline: 4096)")
    ap.add_argument("--rows", type=int, default=0, help="rows, when they differ from --size (profiling runs)")
    ap.add_argument("--f64", action="store_true",
                    help="instead of the headline: only the f64 copy of the matrix, to --width (profiling runs)")
    ap.add_argument("--width", type=int, default=8192, help="terms per decomposition (headline: 8192)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget of the CPU oracle leg (0 = skip)")
    ap.add_argument("--engine", choices=["auto", "stream", "launch"], default="auto",
                    help="auto: register-resident engine when the shape fits; stream: the persistent streaming engine; "
                         "launch: one kernel launch per alternation (the engine of last resort)")
    ap.add_argument("--layer", action="store_true",
                    help="instead of the headline: decompose one synthetic Mistral-7B-shaped decoder layer (7 "
                         "matrices, each to 50 %% of its bf16 footprint) and print seconds per layer")
    ap.add_argument("--no-layer", action="store_true",
                    help="headline only: skip the decoder-layer figure that the default run appends")
    ap.add_argument("--no-extra", action="store_true",
                    help="headline only: skip the f64 run, the error curves and the secondary rooflines")
    ap.add_argument("--layer-fraction", type=float, default=1.0,
                    help="with --layer: run only this fraction of every matrix's width (the rest is extrapolated "
                         "and the line says so)")
    ap.add_argument("--concurrency", type=int, default=7, choices=list(range(1, 9)),
                    help="with --layer: most matrices decomposed side by side (the compute units are shared out among them)")
    ap.add_argument("--apply", action="store_true",
                    help="instead of the headline: time the product of a decomposition with a vector from the "
                         "packed factors (scd_apply) on the layer shapes")
    ap.add_argument("--image", action="store_true",
                    help="instead of the headline: workload 4 (4000x3000x3 image-like tensor): RGB signs, RGB scalars, "
                         "least squares")
    ap.add_argument("--lsq", action="store_true",
                    help="instead of the headline: time the least squares decomposition (Algorithm 6)")
    ap.add_argument("--oracle-timing", action="store_true",
                    help="only time the CPU oracle (one thread, all cores) on prefixes of workloads 1-3")
    ap.add_argument("--calibrate", action="store_true",
                    help="only run the plain copy kernel (64 MiB, 20+1 launches): the known-size reference "
                         "for scaling the profiler's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import numpy as np

    if args.oracle_timing:
        from paper_2410_01799_amd import workloads as wl

        return oracle_mode(args, wl, np)
    import torch

    from paper_2410_01799_amd import scd, workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    scd.lib()
    torch.cuda.set_device(0)
    if args.calibrate:
        src = torch.randn(16 * 1024 * 1024, device="cuda")
        dst = torch.empty_like(src)
        sec = scd.scd_probe_stream(src, dst, 2048, 20)
        print(json.dumps({"calibrate": "stream_copy_kernel", "bytes_read_per_launch": src.numel() * 4,
                          "bytes_written_per_launch": src.numel() * 4, "launches": 21,
                          "us_per_launch": round(sec * 1e6, 2)}))
        return 0
    if args.layer:
        print(json.dumps(layer_mode(args, scd, workloads, torch, np)))
        return 0
    if args.apply:
        return apply_mode(args, scd, torch)
    if args.lsq:
        return lsq_mode(args, scd, workloads, torch, np)
    if args.image:
        return image_mode(args, scd, workloads, torch, np)
    n = args.size
    m = args.rows or n
    w, seed = args.width, 2
    if args.f64:
        A64d = torch.from_numpy(workloads.gaussian_matrix(m, n, seed, np.float64)).cuda()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        with scd.ScdContext(A64d, w, seed) as ctx:
            ctx.run(w)
            e = ctx.engine()
            tr = ctx.results()["trace"].cpu().numpy()
        dt = time.perf_counter() - t0
        print(json.dumps({"metric": f"signed-cut terms/s on {m}x{n} f64 (w={w})", "value": round(w / dt, 2), "unit": "terms/s",
                          "engine": ENGINES[e["engine"]], "launch_us": round(e["last_launch_seconds"] * 1e6, 1),
                          "final_relative_error": round(float(tr[-1] / tr[0]), 6)}))
        return 0
    A64 = workloads.gaussian_matrix(m, n, seed, np.float64)
    A = torch.from_numpy(A64.astype(np.float32)).cuda()
    torch.cuda.synchronize()
    esize = A.element_size()
    headline = (m, n, w) == (4096, 4096, 8192)
    traffic = measured_traffic()
    engine_opts = {"auto": {}, "stream": {"resident": 0, "sparse": 0},
                   "launch": {"resident": 0, "sparse": 0, "persistent_stream": 0}}[args.engine]

    def one_step():
        # one whole decomposition through the stateful calls (what scd_decompose does internally),
        # so that the engine's own launch timing can be read before the context goes away
        with scd.ScdContext(A, w, seed, options=engine_opts) as ctx:
            ctx.run(w)
            res = ctx.results()
            eng = ctx.engine()
        return res, eng

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    launch_s, launch_bytes = [], []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        res, eng = one_step()
        launch_s.append(eng["last_launch_seconds"])
        launch_bytes.append(eng["last_launch_bytes"])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    iters = res["iters"].cpu().numpy().astype(np.int64)
    trace = res["trace"].cpu().numpy()
    iters_total = int(iters.sum())
    final_rel = float(trace[-1] / trace[0])
    terms_per_s = args.steps * w / elapsed
    # algorithmic bytes of one decomposition by a streaming implementation: every alternation reads R once,
    # every term's update writes it once (fused into the first alternation of the next term)
    algo_bytes = (iters_total + w) * m * n * esize
    stream_s = scd.scd_probe_stream(A, None, 256, 50)
    stream_gbs = m * n * esize / stream_s / 1e9

    def stream_roofline(M, terms, label):
        """The persistent streaming kernel (one launch = `terms` terms; every pass reads the remainder once, the pass
        that ends a term also writes it): algorithmic bytes of the launch over its duration by HIP events on the
        library's stream.  The matrix is of the engine's own choosing only when the other engines are switched off."""
        mm, nn = M.shape
        with scd.ScdContext(M, terms, seed, options={"resident": 0, "sparse": 0}) as ctx:
            ctx.run(min(8, terms))
        with scd.ScdContext(M, terms, seed, options={"resident": 0, "sparse": 0}) as ctx:
            ctx.run(terms)
            e = ctx.engine()
            its = int(ctx.results()["iters"].sum())
        if e["engine"] != 3:
            return None
        gbs = e["last_launch_bytes"] / e["last_launch_seconds"] / 1e9
        passes = e["last_launch_bytes"] / (mm * nn * M.element_size()) - terms
        key = f"pstream_kernel_{mm}x{nn}_f32_per_pass"
        return {"bound": "hbm", "kernel": "pstream_kernel (one persistent launch)", "workload": label,
                "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4),
                "traffic": round(traffic[key] * passes) if key in traffic else None,
                "traffic_source": str(TRAFFIC_FILE.relative_to(ROOT)),
                "bytes_per_launch": round(e["last_launch_bytes"]), "launch_us": round(e["last_launch_seconds"] * 1e6, 1),
                "us_per_pass": round(e["last_launch_seconds"] * 1e6 / passes, 3), "terms": terms,
                "terms_per_s": round(terms / e["last_launch_seconds"], 1), "alternations_per_term": round(its / terms, 2),
                "measured_stream_read_gbs": round(stream_gbs, 1),
                "note": "rows of a workgroup's block that fit in LDS are read from memory once per launch, so traffic is "
                        "below the algorithmic bytes; the rest of a pass is the latency of two exchanges among all "
                        "workgroups"}

    extra = {}
    if eng["engine"] == 1:
        # Register-resident engine: the dominant kernel is the one persistent launch per decomposition; its
        # duration comes from HIP events recorded around it on the library's stream, inside the timed region.
        # The remainder never leaves the registers, so neither HBM nor the matrix cores bound it: its work is
        # one add per element and half step (Section 3.4), priced against the chip's fp32 vector rate; what
        # actually limits it is the latency of the two exchanges per alternation (latency_floor).
        sec = sum(launch_s) / len(launch_s)
        phases = sum(launch_bytes) / len(launch_bytes) / (m * n * esize)     # row phases + updates of one launch
        alternations = phases - w                                           # launch_bytes counts one write per update
        real_alternations = iters_total                                     # the dropped row phase per term is not work
        flops = 2.0 * m * n * real_alternations + 3.0 * m * n * w           # adds of both half steps; update: sub, square, add
        achieved = flops / sec / 1e12
        us_alt = sec * 1e6 / alternations
        lane_ops = 2.0 * m * n * alternations + 3.0 * m * n * w             # executed, dropped phases included
        xchg_s = scd.scd_probe_exchange(0, 256, 16, 2000)
        roof = {"bound": "alu", "kernel": "resident_kernel (one persistent launch per decomposition)",
                "achieved": round(achieved, 3), "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / FP32_VECTOR_PEAK_TFLOPS, 4),
                "traffic": round(traffic["resident_kernel_4096x4096_f32_per_alternation"] * alternations)
                if (m, n) == (4096, 4096) and "resident_kernel_4096x4096_f32_per_alternation" in traffic else None,
                "traffic_source": str(TRAFFIC_FILE.relative_to(ROOT)) + " (committed counter run, not measured by this run)",
                "flops_per_launch": round(flops), "launch_us": round(sec * 1e6, 1),
                "us_per_alternation": round(us_alt, 3),
                "issue": {"lane_ops_per_launch": round(lane_ops), "peak_lane_ops_per_s": UNPACKED_LANE_OPS_PER_S,
                          "frac": round(lane_ops / sec / UNPACKED_LANE_OPS_PER_S, 4),
                          "note": "vector instructions issued against what add-only work can issue without packed FP32"},
                "latency_floor": {"exchange_us": round(xchg_s * 1e6, 3), "exchanges_per_alternation": 2,
                                  "frac_of_alternation": round(min(1.0, 2 * xchg_s * 1e6 / us_alt), 4),
                                  "note": "two dependent all-to-all exchanges of partial sums per alternation "
                                          "(16 workgroups each), timed alone by the exchange probe"},
                "hbm_equivalent_gbs": round(algo_bytes / (elapsed / args.steps) / 1e9, 1),
                "note": "the remainder is held in registers: hbm_equivalent_gbs is what a streaming pass per "
                        "alternation would have to move, not traffic, and is no roofline fraction"}
        if headline and not args.no_extra:
            extra["roofline_stream"] = stream_roofline(A, 256, "the headline matrix, first 256 terms")
            big = torch.randn(14336, 4096, device="cuda") * 0.02
            extra["roofline_stream_large"] = stream_roofline(big, 64, "14336x4096 f32 N(0, 0.02^2), 64 terms (224 MiB: "
                                                                      "not cache-resident)")
            del big
    elif eng["engine"] == 3:
        roof = stream_roofline(A, w, f"the {m}x{n} matrix of this run, {w} terms")
    else:
        # one launch of the row pass per alternation: 64 further alternations with an event around every kernel
        with scd.ScdContext(A, w + 64, seed, options=engine_opts) as ctx:
            ctx.run(min(w, 4))
            rp_s, rd_s = ctx.profile_sweeps(64)
        gbs = m * n * esize / rp_s / 1e9
        key = f"rowpass_tiled_{m}x{n}_f32_per_launch"
        roof = {"bound": "hbm", "kernel": "rowpass kernel (one launch per alternation)", "achieved": round(gbs, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4),
                "traffic": round(traffic[key]) if key in traffic else None,
                "traffic_source": str(TRAFFIC_FILE.relative_to(ROOT)), "bytes_per_launch": m * n * esize,
                "launch_us": round(rp_s * 1e6, 2), "reduce_launch_us": round(rd_s * 1e6, 2),
                "measured_stream_read_gbs": round(stream_gbs, 1)}

    # Bytes the paper's own scheme would move for this run (Section 3.1's cached products, Section 3.2's
    # delayed update): dense first alternation of a term (R once for u, once for v), then one row of R per
    # changed row sign and one column per changed column sign, plus the update amortised over 32 terms.
    # The sign changes are counted by the sparse engine on the first terms of the same decomposition.
    sample_terms = min(w, 128)
    with scd.ScdContext(A, sample_terms, seed, options={"resident": 0, "sparse_min_mib": 0}) as ctx:
        useful = None
        if ctx.engine()["engine"] == 2:
            ctx.run(sample_terms)
            fl = ctx.sparse_flips()
            per_term = (2.0 * m * n * esize + esize * (n * fl["rows"] + m * fl["cols"]) / sample_terms
                        + 2.0 * m * n * esize / 32.0)
            useful = {"bytes_per_term": round(per_term), "row_sign_changes_per_term": round(fl["rows"] / sample_terms, 1),
                      "col_sign_changes_per_term": round(fl["cols"] / sample_terms, 1),
                      "gbs": round(per_term * terms_per_s / 1e9, 1),
                      "frac": round(per_term * terms_per_s / 1e9 / HBM_PEAK_GBS, 4),
                      "sample": f"sign changes counted on the first {sample_terms} terms"}
    roof["useful_bytes"] = useful

    def curve_of(tr, every=256):
        return {str(k): round(float(tr[k] / tr[0]), 6) for k in range(0, len(tr), every)}

    out = {
        "metric": f"signed-cut terms/s on {m}x{n} f32 (w={w})",
        "value": round(terms_per_s, 2),
        "unit": "terms/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(1e3 * elapsed / args.steps, 3),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"config 2: {m}x{n} f32 i.i.d. N(0,1) (PCG64 seed {seed}), greedy decomposition to w={w}",
                   "terms": w, "alternations_per_term": round(iters_total / w, 2),
                   "final_relative_error": round(final_rel, 6),
                   "engine": ENGINES[eng["engine"]]},
        "roofline": roof,
    }
    out.update(extra)
    if headline and not args.no_extra:
        # the rest of workload 2: the f64 copy of the same matrix to w = 2048 (sparse engine), and the relative
        # error every 256 terms for both runs, beside the values Figure 7's slope gives
        A64d = torch.from_numpy(A64).cuda()
        with scd.ScdContext(A64d, 2048, seed) as ctx:   # warm-up of the code path on a few terms
            ctx.run(8)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        with scd.ScdContext(A64d, 2048, seed) as ctx:
            ctx.run(2048)
            r64 = ctx.results()
            e64 = ctx.engine()
        torch.cuda.synchronize()
        dt64 = time.perf_counter() - t0
        tr64 = r64["trace"].cpu().numpy()
        it64 = int(r64["iters"].sum())
        sparse_roof = None
        key = "sparse_delay_kernel_4096x4096_f64_per_term"
        if e64["engine"] == 2 and key in traffic:
            gbs = traffic[key] * 2048 / e64["last_launch_seconds"] / 1e9
            sparse_roof = {"bound": "hbm", "kernel": "sparse_delay_kernel<double> (one persistent launch)",
                           "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4),
                           "traffic": round(traffic[key] * 2048), "traffic_source": str(TRAFFIC_FILE.relative_to(ROOT)),
                           "launch_us": round(e64["last_launch_seconds"] * 1e6, 1),
                           "note": "achieved = counter bytes (committed counter run) over this run's launch time: the "
                                   "sparse engine moves what the flipped signs need, and is bound by the latency of its "
                                   "exchanges, not by bandwidth"}
        out["f64"] = {"workload": "the f64 copy of the same matrix to w=2048", "w": 2048, "terms_per_s": round(2048 / dt64, 2),
                      "seconds": round(dt64, 3), "alternations_per_term": round(it64 / 2048, 2),
                      "engine": ENGINES[e64["engine"]],
                      "final_relative_error": round(float(tr64[-1] / tr64[0]), 6)}
        if sparse_roof:
            out["roofline_sparse"] = sparse_roof
        out["curve"] = {"every": 256, "f32": curve_of(trace), "f64": curve_of(tr64),
                        "figure7_slope": {"r(2048)": 0.614, "r(8192)": 0.142,
                                          "note": "exp(-2.3845e-4 k), the decay that both printed points of Figure 7 give"}}
        del A64d
    if args.cpu_seconds > 0:
        out["cpu_baseline"] = cpu_baseline(A64, seed, args.cpu_seconds)
    if not args.no_layer and headline:
        # the metric's second figure: one decoder layer at the 50 % widths (its own timed region)
        del A
        lay = layer_mode(args, scd, workloads, torch, np)
        out["layer"] = {k: lay[k] for k in ("metric", "value", "unit", "terms", "terms_per_s", "concurrency", "extrapolated")}
        out["layer"]["matrix_ended_at"] = {r["matrix"]: r["ended_at"] for r in lay["matrices"]}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
