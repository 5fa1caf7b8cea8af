#!/usr/bin/env python3
"""Benchmark of the IVF-RaBitQ batched search on one MI355X.

A step is one rabitq_search over the whole query batch (all stages of the path) with the
index and the queries resident in HBM.  Prints ONE JSON line: queries/sec at the
operating point (the smallest swept nprobe whose recall@k reaches 0.95, or, when the
code width cannot reach it, the smallest nprobe within 0.005 of the best recall reached),
the roofline of the code-scan kernel, and the CPU oracle's throughput on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# integer vector rate of the chip: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-operations per second
MFMA_I8_PEAK_TOPS = 5000.0   # dense int8 matrix-core peak of MI355X, TOP/s
ALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def exact_knn_gpu(X, Q, k, metric):
    import torch
    xn = (X * X).sum(1)
    out = []
    for s in range(0, Q.shape[0], 1000):
        dot = Q[s:s + 1000] @ X.T
        key = (xn[None, :] - 2.0 * dot) if metric == "l2" else -dot
        out.append(key.topk(k, largest=False).indices)
    return torch.cat(out)


def recall(ids, gt):
    return (ids[:, :, None] == gt[:, None, :]).any(2).float().mean().item()


def scan_algorithmic_bytes(gi, Qd, nprobe, cluster_sizes, dim):
    """Bytes the scan must read by definition: every vector of every probed cluster once per
    probing query, 1-bit code (D/8 bytes) plus three fp32 factors."""
    import torch
    qr = gi.rotate(Qd)
    prep = gi.query_prep(qr)
    probes = gi.coarse_probe(qr, prep["sq_norm"], nprobe)["probe_ids"]
    sizes = torch.from_numpy(cluster_sizes).to(probes.device)
    qv = int(sizes[probes.long()].sum().item())
    return qv * (dim // 8 + 12), qv


def cpu_baseline(w, nprobe, sample_n=100_000, sample_q=1000):
    """The CPU oracle as it stands, timed on this host: it builds its own index over a
    bounded sample of the same workload (same mean list size, same k and nprobe, so the
    work per query matches) and answers `sample_q` queries."""
    from oracle import build as obuild, search as osearch
    from paper_2602_23999_amd import synth
    try:
        from threadpoolctl import threadpool_limits
    except Exception:  # pragma: no cover
        threadpool_limits = None
    frac = sample_n / w.n
    ws = w.scaled(n=sample_n, nq=sample_q, nlist=max(nprobe, int(round(w.nlist * frac))))
    X, Q = synth.make_base(ws), synth.make_queries(ws)
    t0 = time.perf_counter()
    ix = obuild.build_index(X, ws.nlist, ws.total_bits, metric=ws.metric, kmeans_iters=4, center=(ws.metric == "l2"))
    t_build = time.perf_counter() - t0
    s = osearch.Searcher(ix)
    times = []

    def run():
        for _ in range(3):
            t0 = time.perf_counter()
            s.search(Q, ws.k, nprobe)
            times.append(time.perf_counter() - t0)
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            run()
    else:
        run()
    qps = sample_q / float(np.median(times))
    return dict(value=qps, unit="queries/s", cores=1, kind="oracle",
                sample=f"oracle-built index over a {sample_n}-vector sample of the same mixture, nlist={ws.nlist} "
                       f"(same mean list size), {sample_q} queries, k={ws.k}, nprobe={nprobe}, median of 3; "
                       f"numpy fp64, single thread; host cores available: {len(os.sched_getaffinity(0))}; "
                       f"index build {t_build:.1f}s not included")


def stream_scan(args):
    """Streaming regime of the code scan: an index whose 1-bit codes and factors (28 B per
    vector at D = 128) are several times larger than the 256 MB last-level cache, searched
    with nprobe = 1 by one query per inverted list, so every byte the scan needs comes from
    HBM exactly once.  The whole search path runs; the line reports the scan kernel."""
    import torch
    from paper_2602_23999_amd import rabitq
    rabitq.load_library()
    n, dim, nlist, bits, k = args.stream_n, 128, args.stream_n // args.stream_list, args.stream_bits, 10
    gen = torch.Generator(device="cuda").manual_seed(1234)
    centres = torch.randn((nlist, dim), generator=gen, device="cuda") * 4.0
    X = torch.empty((n, dim), dtype=torch.float32, device="cuda")
    own = torch.randint(0, nlist, (n,), generator=gen, device="cuda")
    for s0 in range(0, n, 1 << 20):
        e0 = min(n, s0 + (1 << 20))
        X[s0:e0] = centres[own[s0:e0]] + torch.randn((e0 - s0, dim), generator=gen, device="cuda")
    g = np.random.Generator(np.random.PCG64(7)).standard_normal((dim, dim))
    qm, rm = np.linalg.qr(g)
    P = (qm * np.sign(np.diag(rm))[None, :]).astype(np.float32)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    gi = rabitq.Index.build(X, nlist, bits, P, metric="l2", kmeans_iters=4, train_size=n // 10)
    torch.cuda.synchronize()
    log(f"[bench] stream-scan index N={n} nlist={nlist} B={bits}: {time.perf_counter() - t0:.2f}s")
    offsets = np.empty(nlist + 1, np.int64)
    rabitq._check(rabitq.load_library().rabitq_index_export(gi._h, None, None, offsets.ctypes.data, None, None, None,
                                                           None, None, None))
    cluster_sizes = np.diff(offsets).astype(np.int64)
    # one query per generating centre: a fresh draw around it
    Qd = centres + torch.randn((nlist, dim), generator=gen, device="cuda")
    del X, own
    # keep one query per distinct nearest list, so that no two pairs share a list
    first = gi.coarse_probe(gi.rotate(Qd), gi.query_prep(gi.rotate(Qd))["sq_norm"], 1)["probe_ids"].view(-1).long()
    pick = torch.full((nlist,), Qd.shape[0], dtype=torch.int64, device="cuda")
    pick.scatter_reduce_(0, first, torch.arange(Qd.shape[0], device="cuda"), reduce="amin")
    Qd = Qd[pick[pick < Qd.shape[0]]].contiguous()
    nq = Qd.shape[0]
    out_ids = torch.empty((nq, k), dtype=torch.int64, device="cuda")
    out_d = torch.empty((nq, k), dtype=torch.float32, device="cuda")
    gi.set_option("scan_impl", args.scan_impl)
    for _ in range(args.warmup):
        gi.search(Qd, k, 1, out_ids, out_d)
    gi.set_option("profile", args.steps)
    torch.cuda.synchronize()
    t = time.perf_counter()
    for _ in range(args.steps):
        gi.search(Qd, k, 1, out_ids, out_d)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t) / args.steps
    stage_ms, calls = gi.stage_ms()
    gi.set_option("profile", 0)
    alg_bytes, qv = scan_algorithmic_bytes(gi, Qd, 1, cluster_sizes, dim)
    probes = gi.coarse_probe(gi.rotate(Qd), gi.query_prep(gi.rotate(Qd))["sq_norm"], 1)["probe_ids"]
    distinct = int(torch.unique(probes).numel())
    scan_ms = stage_ms["scan"]
    achieved = alg_bytes / (scan_ms * 1e-3) / 1e9
    # what a plain device-to-device copy of 1 GiB reaches on this device (read + write bytes), for scale
    src = torch.empty(256 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 10 * 2 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst
    res = {
        "metric": "code-scan HBM GB/s vs peak, streaming regime (1 GPU)", "value": achieved, "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": sec * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u32 popcount + f32", "data": "synthetic",
        "config": {"workload": f"stream_scan: N={n} D={dim} nlist={nlist} B={bits} nq={nq} k={k} nprobe=1 "
                               f"(one query per list; {distinct} distinct lists probed)",
                   "index_short_bytes": int(cluster_sizes.sum()) * (dim // 8 + 12),
                   "list_size_median_max": [int(np.median(cluster_sizes)), int(cluster_sizes.max())],
                   "stage_ms": {k_: round(v, 4) for k_, v in stage_ms.items()}, "stage_ms_calls": calls,
                   "query_vector_evaluations": qv},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None, "device_copy_gbs": copy_gbs,
                     "kernel": ("scan_kernel", "scan_mfma_kernel", "scan_kernel (lookup tables)",
                                "scan_kernel")[args.scan_impl],  # D = 128: the default choice is the popcount kernel
                     "algorithmic_bytes_per_launch": alg_bytes, "kernel_ms": scan_ms},
    }
    print(json.dumps(res), flush=True)
    gi.close()


def batch_sweep(args, gi, Qd, w, nprobe):
    """Latency of one synchronised rabitq_search by batch size (the paper's batch-size experiment, Section 4.2.2),
    launched eagerly and as a replay of a HIP graph holding the same search."""
    import torch
    rows = []
    for nq in (1, 10, 100, 1000, 10000):
        if nq > Qd.shape[0]:
            continue
        q = Qd[:nq].contiguous()
        oi = torch.empty((nq, w.k), dtype=torch.int64, device="cuda")
        od = torch.empty((nq, w.k), dtype=torch.float32, device="cuda")
        for _ in range(5):
            gi.search(q, w.k, nprobe, oi, od)
        torch.cuda.synchronize()

        def timed(call, reps=50):
            ts = []
            for _ in range(reps):
                t = time.perf_counter()
                call()
                torch.cuda.synchronize()
                ts.append(time.perf_counter() - t)
            return float(np.median(ts)) * 1e3
        eager_ms = timed(lambda: gi.search(q, w.k, nprobe, oi, od))
        ref = oi.clone()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            gi.search(q, w.k, nprobe, oi, od)
        oi.fill_(-7)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(oi, ref), "graph replay differs from the eager search"
        graph_ms = timed(g.replay)
        rows.append(dict(nq=nq, eager_ms=round(eager_ms, 4), graph_ms=round(graph_ms, 4),
                         qps=round(nq / min(eager_ms, graph_ms) * 1e3)))
        log(f"[bench] batch {nq}: eager {eager_ms:.4f} ms, graph replay {graph_ms:.4f} ms")
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="l2_128")
    ap.add_argument("--nprobe", type=int, default=0, help="fix the operating point instead of choosing it by recall")
    ap.add_argument("--n", type=int, default=0, help="override the number of base vectors (for quick runs)")
    ap.add_argument("--bits", type=int, default=0,
                    help="override the workload's total bits per dimension (1..8): shows where the recall ceiling of "
                         "the code size lies; the default run keeps the size the workload states")
    ap.add_argument("--eps0", type=float, default=1.9,
                    help="multiplier of the 1-bit error bound the index is built with (the filter keeps a vector when "
                         "its estimate minus eps0 standard errors is below the threshold)")
    ap.add_argument("--scan-impl", type=int, default=3,
                    help="0: popcount scan, 1: matrix-core scan, 2: lookup-table scan, 3 (default): the library's choice "
                         "by code width (popcount below D = 960)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one elementwise add over 256 MiB (reads 256 MiB, writes 256 MiB): the known-size "
                         "kernel that scales rocprofv3's FETCH_SIZE / WRITE_SIZE readings")
    ap.add_argument("--batch-sweep", action="store_true",
                    help="also time one synchronised search at batch sizes 1..10^4, eager and as a HIP-graph replay "
                         "(adds config.batch_sweep)")
    ap.add_argument("--stream-scan", action="store_true",
                    help="measure the code scan in the streaming regime instead (index far larger than the caches, "
                         "one query per list); prints its own JSON line")
    ap.add_argument("--stream-n", type=int, default=64 * 1024 * 1024)
    ap.add_argument("--stream-bits", type=int, default=1)
    ap.add_argument("--stream-list", type=int, default=1024, help="mean inverted-list length of the streaming index")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures the one-GPU path only: this build has no multi-GPU sharding (run with --gpus 1)")

    import torch
    from paper_2602_23999_amd import rabitq, synth
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a HIP device")
    rabitq.load_library()
    if args.stream_scan:
        return stream_scan(args)
    w = synth.WORKLOADS[args.workload]
    if args.n:
        w = w.scaled(n=args.n, nlist=max(64, int(round(w.nlist * args.n / w.n))))
    if args.bits:
        w = w.scaled(total_bits=args.bits)
    t0 = time.perf_counter()
    X, Q = synth.make_base(w), synth.make_queries(w)
    Xd, Qd = torch.from_numpy(X).cuda(), torch.from_numpy(Q).cuda()
    log(f"[bench] data {w.name} N={w.n} D={w.dim} nq={w.nq}: {time.perf_counter() - t0:.1f}s")
    # random orthogonal P: QR of a seeded Gaussian matrix (host side; the library takes P as an input)
    g = np.random.Generator(np.random.PCG64(7)).standard_normal((w.dim, w.dim))
    qm, rm = np.linalg.qr(g)
    P = (qm * np.sign(np.diag(rm))[None, :]).astype(np.float32)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    gi = rabitq.Index.build(Xd, w.nlist, w.total_bits, P, metric=w.metric, kmeans_iters=10,
                            train_size=max(w.nlist * 40, w.n // 10), center=(w.metric == "l2"), epsilon0=args.eps0)
    torch.cuda.synchronize()
    build_s = time.perf_counter() - t0
    log(f"[bench] index build on the device: {build_s:.3f}s")
    offsets = np.empty(w.nlist + 1, np.int64)
    rabitq._check(rabitq.load_library().rabitq_index_export(gi._h, None, None, offsets.ctypes.data, None, None, None,
                                                           None, None, None))
    cluster_sizes = np.diff(offsets).astype(np.int64)
    gt = exact_knn_gpu(Xd, Qd, w.k, w.metric)
    del Xd

    out_ids = torch.empty((w.nq, w.k), dtype=torch.int64, device="cuda")
    out_d = torch.empty((w.nq, w.k), dtype=torch.float32, device="cuda")

    def timed(nprobe, steps, warmup, profile=False):
        for _ in range(warmup):
            gi.search(Qd, w.k, nprobe, out_ids, out_d)
        if profile:
            gi.set_option("profile", steps)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(steps):
            gi.search(Qd, w.k, nprobe, out_ids, out_d)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / steps

    gi.set_option("scan_impl", args.scan_impl)
    sweep = []
    nprobes = [args.nprobe] if args.nprobe else [p for p in w.nprobes if p <= w.nlist]
    for p in nprobes:
        sec = timed(p, 5, 2)
        r = recall(out_ids, gt)
        sweep.append(dict(nprobe=p, recall=round(r, 4), qps=round(w.nq / sec)))
        log(f"[bench] nprobe={p}: recall@{w.k}={r:.4f} {w.nq / sec:,.0f} q/s")
    best = max(s["recall"] for s in sweep)
    ok = [s for s in sweep if s["recall"] >= 0.95] or [s for s in sweep if s["recall"] >= best - 0.005]
    op = ok[0]
    nprobe = op["nprobe"]

    # timed region: only the scan kernel's two events are recorded (every recorded stage costs two event records
    # per search); the other stages are timed in a separate short pass afterwards
    gi.set_option("profile_stages", 1 << 7)
    sec = timed(nprobe, args.steps, args.warmup, profile=True)
    scan_ms = gi.stage_ms()[0]["scan"]
    gi.set_option("profile_stages", 0x1ff)
    timed(nprobe, min(args.steps, 20), 0, profile=True)
    stage_ms, calls = gi.stage_ms()
    gi.set_option("profile", 0)
    r_op = recall(out_ids, gt)
    qps = w.nq / sec
    alg_bytes, qv = scan_algorithmic_bytes(gi, Qd, nprobe, cluster_sizes, w.dim)
    achieved = alg_bytes / (scan_ms * 1e-3) / 1e9
    traffic = None
    # measured fabric traffic per launch (bytes), from the rocprofv3 --pmc summaries under profiles/
    tpath = os.path.join(ROOT, "profiles", f"scan_kernel_{w.name}_traffic.txt")
    if os.path.exists(tpath):
        for line in open(tpath):
            f = line.split()
            if len(f) >= 2 and f[0] == f"nprobe_{nprobe}":
                traffic = int(f[1])
    # The scan of this workload is served by the caches (every list is probed by ~160 queries of the batch) and is
    # bound by the vector ALUs: 8W + 6 lane-operations per query-vector evaluation (W AND + W popcount per bit-plane,
    # 4 planes, then combine, estimate, bound and compare).  The HBM view of the same launch is kept beside it.
    impl = args.scan_impl if args.scan_impl != 3 else (1 if w.dim >= 960 else 0)
    alu_ops = qv * (8 * (w.dim // 32) + 6)
    alu_achieved = alu_ops / (scan_ms * 1e-3) / 1e12
    roofline = {"bound": "alu", "achieved": alu_achieved, "peak": ALU_PEAK_TOPS, "unit": "TOP/s (integer lane-operations)",
                "frac": alu_achieved / ALU_PEAK_TOPS, "traffic": traffic if impl == 0 else None,
                "kernel": ("scan_kernel", "scan_mfma_kernel", "scan_kernel (lookup tables)")[impl],
                "algorithmic_ops_per_launch": alu_ops, "kernel_ms": scan_ms,
                "hbm_view": {"algorithmic_bytes_per_launch": alg_bytes, "achieved_gbs": achieved, "peak_gbs": HBM_PEAK_GBS,
                             "frac": achieved / HBM_PEAK_GBS,
                             "note": "above 1 because the launch is cache-served; the HBM-bound regime is measured by "
                                     "bench.py --stream-scan"}}
    if impl == 1:
        # the matrix-core scan contracts sign bytes with the int8 query: 2 D integer operations per evaluation on
        # v_mfma_i32_16x16x64_i8, priced against the dense int8 peak
        mfma_ops = qv * 2 * w.dim
        mfma_achieved = mfma_ops / (scan_ms * 1e-3) / 1e12
        roofline.update({"bound": "mfma", "achieved": mfma_achieved, "peak": MFMA_I8_PEAK_TOPS, "unit": "TOP/s (int8)",
                         "frac": mfma_achieved / MFMA_I8_PEAK_TOPS, "algorithmic_ops_per_launch": mfma_ops,
                         "alu_view": {"lane_ops_per_launch": alu_ops, "achieved_tops": alu_achieved,
                                      "peak_tops": ALU_PEAK_TOPS,
                                      "note": "what the popcount formulation of the same evaluations would need"}})
    res = {
        "metric": "queries/sec at recall@10~0.95 (1 GPU); code-scan HBM GB/s vs peak",
        "value": qps, "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("u32 popcount + f32", "i8 matrix cores + f32", "f16 tables + f32")[impl], "data": "synthetic",
        "config": {"workload": f"{w.name}: N={w.n} D={w.dim} nlist={w.nlist} B={w.total_bits} "
                               f"nq={w.nq} k={w.k} nprobe={nprobe}",
                   "recall_at_k": round(r_op, 4), "recall_target": 0.95, "nprobe_sweep": sweep,
                   "stage_ms": {k_: round(v, 4) for k_, v in stage_ms.items()}, "stage_ms_calls": calls,
                   "stage_ms_note": "separate pass with every stage's events recorded; list_build and scan_setup run on a "
                                    "second stream beside seed, so the stages add up to more than ms_per_step",
                   "query_vector_evaluations": qv, "index_builder": "rabitq_index_build (HIP: k-means + two-phase grid search"
                                    + (", vectors centred on their mean)" if w.metric == "l2" else ")"),
                   "index_build_s": round(build_s, 4)},
        "roofline": roofline,
    }
    if args.batch_sweep:
        res["config"]["batch_sweep"] = batch_sweep(args, gi, Qd, w, nprobe)
    if not args.no_cpu_baseline:
        t0 = time.perf_counter()
        res["cpu_baseline"] = cpu_baseline(w, nprobe)
        log(f"[bench] cpu baseline: {res['cpu_baseline']['value']:.1f} q/s ({time.perf_counter() - t0:.1f}s)")
    if args.pmc_calibration:
        cal = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        cal2 = cal + 1.0
        torch.cuda.synchronize()
        del cal, cal2
    print(json.dumps(res), flush=True)
    gi.close()


if __name__ == "__main__":
    main()
