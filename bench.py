#!/usr/bin/env python3
"""Benchmark of the IVF-RaBitQ batched search on one MI355X.

A step is one rabitq_search over the whole query batch (all stages of the path) with the
index and the queries resident in HBM.  Prints ONE JSON line:

* value: queries/sec of the 128-d 1M workload with the code size the workload states
  (4 bits per dimension), at the smallest swept nprobe whose recall@10 reaches 0.95 or,
  when that code size cannot reach it, the smallest nprobe within 0.005 of the best recall
  reached (config.recall_target_met says which);
* config.point_at_recall_target: the same workload at the smallest code size that does reach
  recall@10 >= 0.95, with its own throughput, scan time and roofline;
* roofline: the code-scan kernel of the headline point (cache-served, bound by the vector
  ALUs) and, under roofline.stream, the same kernel in the streaming regime (an index several
  times the last-level cache, one query per list) against the HBM peak;
* cpu_baseline: the CPU oracle timed on the host cores on the same index and queries.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_I8_PEAK_TOPS = 5000.0   # dense int8 matrix-core peak of MI355X, TOP/s
# integer vector rate of the chip: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-operations per second
ALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
RECALL_TARGET = 0.95


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


def rotation_matrix(dim):
    """Random orthogonal P: QR of a seeded Gaussian matrix (host side; the library takes P as an input)."""
    g = np.random.Generator(np.random.PCG64(7)).standard_normal((dim, dim))
    qm, rm = np.linalg.qr(g)
    return (qm * np.sign(np.diag(rm))[None, :]).astype(np.float32)


def cluster_sizes_of(gi):
    from paper_2602_23999_amd import rabitq
    offsets = np.empty(gi.nlist + 1, np.int64)
    rabitq._check(rabitq.load_library().rabitq_index_export(gi._h, None, None, offsets.ctypes.data, None, None, None,
                                                           None, None, None))
    return np.diff(offsets).astype(np.int64)


def scan_algorithmic_bytes(gi, Qd, nprobe, cluster_sizes, dim):
    """Bytes the scan must read by definition: every vector of every probed cluster once per probing query, 1-bit
    code (D/8 bytes) plus the fp32 factors the estimate needs: three (f_add, f_rescale, f_err) when there is a long
    code to refine with, two when the 1-bit estimate is final and no bound is taken (B = 1)."""
    import torch
    qr = gi.rotate(Qd)
    prep = gi.query_prep(qr)
    probes = gi.coarse_probe(qr, prep["sq_norm"], nprobe)["probe_ids"]
    sizes = torch.from_numpy(cluster_sizes).to(probes.device)
    qv = int(sizes[probes.long()].sum().item())
    return qv * (dim // 8 + (8 if gi.total_bits == 1 else 12)), qv, int(torch.unique(probes).numel())


def kernel_source_hash():
    """Identifies the scan kernel a stored counter reading belongs to."""
    h = hashlib.sha256()
    for fn in ("scan.hip", "estimate_mfma.hip", "rq_device.h", "rq_scan_args.h", "scan_dispatch.hip"):
        h.update(open(os.path.join(ROOT, "paper_2602_23999_amd", "csrc", fn), "rb").read())
    return h.hexdigest()[:16]


def stored_traffic(workload, nprobe, split=False):
    """Fabric traffic per scan launch (bytes) from the rocprofv3 --pmc summary under profiles/, if that summary was
    taken with the kernel sources as they are now; else None."""
    path = os.path.join(ROOT, "profiles", f"scan_kernel_{workload}_traffic.txt")
    if not os.path.exists(path):
        return None, "no counter summary under profiles/"
    val, src = None, None
    for line in open(path):
        f = line.split()
        if len(f) >= 2 and f[0] == "kernel_source_hash":
            src = f[1]
        if len(f) >= 2 and f[0] == f"nprobe_{nprobe}" + ("_split" if split else ""):
            val = int(f[1])
    if val is None:
        return None, "no counter reading for this nprobe"
    if src != kernel_source_hash():
        return None, "the counter summary under profiles/ was taken with other kernel sources"
    return val, f"from profiles/{os.path.basename(path)} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, same kernel sources)"


def stored_stream_traffic():
    """Measured over algorithmic bytes of the streaming scan kernel, from the counter summary under profiles/ (taken on
    smaller indices than the streaming leg's: the counter run does not complete at its size), if that summary was taken
    with the kernel sources as they are now; else None."""
    path = os.path.join(ROOT, "profiles", "scan_stream_kernel_traffic.txt")
    if not os.path.exists(path):
        return None
    src, rows = None, []
    for line in open(path):
        f = line.split()
        if len(f) >= 2 and f[0] == "kernel_source_hash":
            src = f[1]
        if len(f) >= 7 and f[0].startswith("n_"):
            written = 0 if f[6] == "none" else int(f[6])
            rows.append({"n": int(f[0][2:]), "algorithmic_bytes": int(f[2]), "read_bytes": int(f[4]),
                         "written_bytes": None if f[6] == "none" else written,
                         "ratio": round((int(f[4]) + written) / int(f[2]), 4)})
    if src != kernel_source_hash() or not rows:
        return None
    return {"source": "profiles/scan_stream_kernel_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on "
                      "paper_2602_23999_amd/stream_probe, same kernel sources)", "launches": rows}


def cpu_baseline(gi, Q, k, nprobe, budget_q=2000):
    """The CPU oracle as it stands, on the index the GPU leg searched (exported from the device and re-indexed into
    the oracle's arrays) and the first min(nq, 2000) of the same queries (10 to 30 s of CPU work), on all host cores the process may use: the
    queries are dealt to one worker process per core, each running the oracle's search unchanged.  The workers are
    started afresh (spawn), load the index from a file and never touch the GPU."""
    import multiprocessing as mp
    import tempfile
    from oracle import build as obuild, parallel as opar
    t0 = time.perf_counter()
    ix = obuild.unpack_device_layout(gi.export())
    cores = len(os.sched_getaffinity(0))
    nq = min(budget_q, Q.shape[0])
    parts = [p for p in np.array_split(np.arange(nq), cores) if len(p)]
    with tempfile.TemporaryDirectory() as tmp:
        path = os.path.join(tmp, "index.npz")
        opar.save_index(path, ix)
        del ix
        with mp.get_context("spawn").Pool(len(parts), initializer=opar.init, initargs=(path,)) as pool:
            assert all(pool.map(opar.ready, range(4 * len(parts))))   # every worker has loaded the index
            t_prep = time.perf_counter() - t0
            jobs = [(Q[p], k, nprobe) for p in parts]
            times = []
            for _ in range(3):
                t0 = time.perf_counter()
                pool.map(opar.run, jobs, chunksize=1)
                times.append(time.perf_counter() - t0)
    return dict(value=nq / float(np.median(times)), unit="queries/s", cores=len(parts), kind="oracle",
                sample=f"the index of the GPU leg (rabitq_index_export -> oracle arrays -> {len(parts)} worker processes, "
                       f"{t_prep:.1f}s, not timed), the first {nq} of its queries, k={k}, nprobe={nprobe}, median of 3; "
                       f"numpy fp64, deliberately unoptimised, one process per host core ({cores} available)")


def build_index(Xd, w, bits, eps0):
    import torch
    from paper_2602_23999_amd import rabitq
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    gi = rabitq.Index.build(Xd, w.nlist, bits, rotation_matrix(w.dim), metric=w.metric, kmeans_iters=10,
                            train_size=max(w.nlist * 40, w.n // 10), center=(w.metric == "l2"), epsilon0=eps0)
    torch.cuda.synchronize()
    return gi, time.perf_counter() - t0


def measure_point(gi, Qd, gt, w, bits, args, label):
    """Sweep nprobe, choose the operating point, time it; returns the point's record."""
    import torch
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
        log(f"[bench] {label} nprobe={p}: recall@{w.k}={r:.4f} {w.nq / sec:,.0f} q/s")
        if r >= RECALL_TARGET and not args.full_sweep:
            break  # the operating point is found; larger nprobe only costs time
    best = max(s["recall"] for s in sweep)
    ok = [s for s in sweep if s["recall"] >= RECALL_TARGET] or [s for s in sweep if s["recall"] >= best - 0.005]
    nprobe = ok[0]["nprobe"]

    # timed region: only the scan kernel's two events are recorded (every recorded stage costs two event records
    # per search); the other stages are timed in a separate short pass afterwards
    gi.set_option("profile_stages", (1 << 7) | (1 << 9))
    sec = timed(nprobe, args.steps, args.warmup, profile=True)
    timed_ms = gi.stage_ms()[0]
    scan_ms, est_ms = timed_ms["scan"], timed_ms["scan_estimate"]
    split = bool(gi.index_info("last_scan_split"))
    r_op = recall(out_ids, gt)
    gi.set_option("profile_stages", 0x3ff)
    timed(nprobe, min(args.steps, 20), 0, profile=True)
    stage_ms, calls = gi.stage_ms()
    gi.set_option("profile", 0)
    # the same point with the filter off (every vector of every probed list refined): the paper's unpruned definition
    gi.set_option("prune", 0)
    gi.search(Qd, w.k, nprobe, out_ids, out_d)
    torch.cuda.synchronize()
    r_unpruned = recall(out_ids, gt)
    gi.set_option("prune", 1)
    return dict(total_bits=bits, nprobe=nprobe, recall_at_k=round(r_op, 4), recall_at_k_unpruned=round(r_unpruned, 4),
                qps=w.nq / sec, ms_per_step=sec * 1e3, scan_ms=scan_ms, scan_split=split, scan_estimate_ms=est_ms,
                nprobe_sweep=sweep,
                stage_ms={k_: round(v, 4) for k_, v in stage_ms.items()}, stage_ms_calls=calls)


def scan_roofline(gi, Qd, w, pt, cluster_sizes, args):
    """Roofline record of the scan kernel at an operating point.  The scan of this workload is served by the caches
    (every list is probed by ~160 queries of the batch) and is bound by the vector ALUs: 8W + 6 lane-operations per
    query-vector evaluation (W AND + W popcount per bit-plane, 4 planes, then combine, estimate, bound and compare).
    The HBM view of the same launch is kept beside it."""
    alg_bytes, qv, _ = scan_algorithmic_bytes(gi, Qd, pt["nprobe"], cluster_sizes, w.dim)
    scan_ms = pt["scan_ms"]
    achieved = alg_bytes / (scan_ms * 1e-3) / 1e9
    impl = args.scan_impl if args.scan_impl != 3 else (1 if w.dim >= 960 else 0)
    alu_ops = qv * (8 * (w.dim // 32) + 6)
    alu_achieved = alu_ops / (scan_ms * 1e-3) / 1e12
    split = pt.get("scan_split", False)
    traffic, traffic_note = (stored_traffic(w.name, pt["nprobe"], split)
                             if impl == 0 and pt["total_bits"] == w.total_bits
                             else (None, "no counter summary for this variant"))
    roofline = {"bound": "alu", "achieved": alu_achieved, "peak": ALU_PEAK_TOPS, "unit": "TOP/s (integer lane-operations)",
                "frac": alu_achieved / ALU_PEAK_TOPS, "traffic": traffic, "traffic_source": traffic_note,
                "kernel": {0: "scan_kernel", 1: "scan_mfma_kernel", 2: "scan_kernel (lookup tables)", 4: "scan_kernel"}[impl],
                "algorithmic_ops_per_launch": alu_ops, "kernel_ms": scan_ms, "query_vector_evaluations": qv,
                "hbm_view": {"algorithmic_bytes_per_launch": alg_bytes, "achieved_gbs": achieved, "peak_gbs": HBM_PEAK_GBS,
                             "frac": achieved / HBM_PEAK_GBS,
                             "note": "above 1 when the launch is cache-served; the HBM-bound regime is roofline.stream"}}
    if split:
        # Split search: the estimates run as estimate_mfma_kernel (matrix cores), the refinement as scan_kernel in its
        # refinement-only form; kernel_ms is the time of the two together (HIP events around both), and `achieved`
        # prices the stage with the same algorithmic figure as the fused kernel, 8W + 6 lane-operations per evaluation.
        est_ms = pt["scan_estimate_ms"]
        mfma_ops = qv * 2 * w.dim
        roofline.update({
            "kernel": "estimate_mfma_kernel + scan_kernel (refinement only)",
            "kernels_ms": {"estimate_mfma_kernel": est_ms, "scan_kernel (refinement only)": scan_ms - est_ms},
            "note": "the 1-bit inner products of this stage run on the matrix cores, so the vector ALUs execute fewer "
                    "operations than the algorithmic figure counts: frac is the rate of popcount-equivalent work "
                    "against the vector peak, not the share of issue slots used",
            "estimate_kernel_mfma_view": {"int8_ops_per_launch": mfma_ops,
                                          "achieved_tops": mfma_ops / (est_ms * 1e-3) / 1e12 if est_ms > 0 else None,
                                          "peak_tops": MFMA_I8_PEAK_TOPS,
                                          "frac": mfma_ops / (est_ms * 1e-3) / 1e12 / MFMA_I8_PEAK_TOPS if est_ms > 0 else None}})
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
    return roofline


def stream_scan(args, n, bits, steps, warmup):
    """Streaming regime of the code scan: an index whose 1-bit codes and factors (28 B per vector at D = 128) are
    several times larger than the 256 MB last-level cache, searched with nprobe = 1 by one query per inverted list,
    so every byte the scan needs comes from HBM exactly once.  The whole search path runs; the record is about the
    scan kernel.  Returns the roofline record."""
    import torch
    from paper_2602_23999_amd import rabitq
    dim, nlist, k = 128, n // args.stream_list, 10
    gen = torch.Generator(device="cuda").manual_seed(1234)
    # mixture generated on the device: N/1024 centres N(0, 16 I); a point is its centre plus a scatter inside one of 64
    # eight-dimensional subspaces (std 3) plus a little isotropic noise (std 0.3), so that, as in descriptor data, a
    # query has neighbours that are clearly nearer than the bulk of its list and the 1-bit filter has something to do
    centres = torch.randn((nlist, dim), generator=gen, device="cuda") * 4.0
    basis = torch.linalg.qr(torch.randn((64, dim, 8), generator=gen, device="cuda"))[0]   # [64][dim][8] orthonormal
    X = torch.empty((n, dim), dtype=torch.float32, device="cuda")
    own = torch.randint(0, nlist, (n,), generator=gen, device="cuda")

    def draw(c_idx):
        z = torch.randn((c_idx.shape[0], 8), generator=gen, device="cuda") * 3.0
        sub = torch.einsum("nk,ndk->nd", z, basis[c_idx % 64])
        return centres[c_idx] + sub + 0.3 * torch.randn((c_idx.shape[0], dim), generator=gen, device="cuda")
    for s0 in range(0, n, 1 << 20):
        e0 = min(n, s0 + (1 << 20))
        X[s0:e0] = draw(own[s0:e0])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    gi = rabitq.Index.build(X, nlist, bits, rotation_matrix(dim), metric="l2", kmeans_iters=4, train_size=n // 10)
    torch.cuda.synchronize()
    build_s = time.perf_counter() - t0
    log(f"[bench] stream-scan index N={n} nlist={nlist} B={bits}: {build_s:.2f}s")
    cluster_sizes = cluster_sizes_of(gi)
    # one query per generating centre: a fresh draw around it
    Qd = draw(torch.arange(nlist, device="cuda"))
    del X, own
    # keep one query per distinct nearest list, so that no two pairs share a list
    first = gi.coarse_probe(gi.rotate(Qd), gi.query_prep(gi.rotate(Qd))["sq_norm"], 1)["probe_ids"].view(-1).long()
    pick = torch.full((nlist,), Qd.shape[0], dtype=torch.int64, device="cuda")
    pick.scatter_reduce_(0, first, torch.arange(Qd.shape[0], device="cuda"), reduce="amin")
    Qd = Qd[pick[pick < Qd.shape[0]]].contiguous()
    nq = Qd.shape[0]
    out_ids = torch.empty((nq, k), dtype=torch.int64, device="cuda")
    out_d = torch.empty((nq, k), dtype=torch.float32, device="cuda")
    gi.set_option("scan_impl", 0)  # D = 128: the popcount kernel (the library's own choice at this width)
    if args.stream_seg_tiles > 0:
        gi.set_option("scan_segment_tiles", args.stream_seg_tiles)
    if not args.stream_longest_first:
        gi.set_option("longest_first", 0)
    for _ in range(warmup):
        gi.search(Qd, k, 1, out_ids, out_d)
    gi.set_option("profile", steps)
    torch.cuda.synchronize()
    t = time.perf_counter()
    for _ in range(steps):
        gi.search(Qd, k, 1, out_ids, out_d)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t) / steps
    stage_ms, calls = gi.stage_ms()
    gi.set_option("profile", 0)
    alg_bytes, qv, distinct = scan_algorithmic_bytes(gi, Qd, 1, cluster_sizes, dim)
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
    gi.close()
    return {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": None, "traffic_source": "no counter run completes at this size: see profiles/scan_kernel_stream_scan.md",
            "traffic_ratio": stored_stream_traffic(),
            "device_copy_gbs": copy_gbs, "kernel": "scan_stream_kernel" if bits == 1 else "scan_stream_long_kernel",
            "algorithmic_bytes_per_launch": alg_bytes, "kernel_ms": scan_ms, "query_vector_evaluations": qv,
            "workload": f"stream_scan: N={n} D={dim} nlist={nlist} B={bits} nq={nq} k={k} nprobe=1 (one query per list; "
                        f"{distinct} distinct lists probed)",
            "index_short_bytes": int(cluster_sizes.sum()) * (dim // 8 + (8 if bits == 1 else 12)),
            "bytes_per_evaluation": dim // 8 + (8 if bits == 1 else 12),
            "list_size_median_max": [int(np.median(cluster_sizes)), int(cluster_sizes.max())],
            "search_ms": sec * 1e3, "stage_ms": {k_: round(v, 4) for k_, v in stage_ms.items()}, "stage_ms_calls": calls,
            "index_build_s": round(build_s, 2)}


def batch_sweep(gi, Qd, w, nprobe):
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
    ap.add_argument("--full-sweep", action="store_true", help="sweep every nprobe of the workload even past the target")
    ap.add_argument("--n", type=int, default=0, help="override the number of base vectors (for quick runs)")
    ap.add_argument("--bits", type=int, default=0,
                    help="override the workload's total bits per dimension (1..8) for the headline point")
    ap.add_argument("--target-bits", type=int, default=-1,
                    help="code size of the second operating point (config.point_at_recall_target): -1 (default) tries "
                         "B+1, B+2, ... until recall@k >= 0.95; 0 skips it")
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
                    help="force the batch-size sweep on (it is part of the default run of the default workload)")
    ap.add_argument("--no-batch-sweep", action="store_true")
    ap.add_argument("--stream-scan", action="store_true",
                    help="run only the streaming-regime measurement and print its own JSON line")
    ap.add_argument("--no-stream", action="store_true", help="skip the streaming-regime leg (roofline.stream)")
    ap.add_argument("--stream-n", type=int, default=0,
                    help="vectors of the streaming index (default 32 Mi inside the default run, 64 Mi with --stream-scan)")
    ap.add_argument("--stream-bits", type=int, default=1)
    ap.add_argument("--stream-seg-tiles", type=int, default=0,
                    help="segment length (tiles) of the streaming leg's work items; 0 = the library's choice")
    ap.add_argument("--stream-longest-first", type=int, default=1,
                    help="0: the streaming leg's work items in cluster order instead of longest list first")
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
        rec = stream_scan(args, args.stream_n or 64 * 1024 * 1024, args.stream_bits, args.steps, args.warmup)
        print(json.dumps({"metric": "code-scan HBM GB/s vs peak, streaming regime (1 GPU)", "value": rec["achieved"],
                          "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                          "ms_per_step": rec["search_ms"], "higher_is_better": True, "scaling": "weak",
                          "vs_baseline": None, "dtype": "u32 popcount + f32", "data": "synthetic",
                          "config": {"workload": rec["workload"]}, "roofline": rec}), flush=True)
        return
    w = synth.WORKLOADS[args.workload]
    if args.n:
        w = w.scaled(n=args.n, nlist=max(64, int(round(w.nlist * args.n / w.n))))
    if args.bits:
        w = w.scaled(total_bits=args.bits)
    t0 = time.perf_counter()
    X, Q = synth.make_base(w), synth.make_queries(w)
    Xd, Qd = torch.from_numpy(X).cuda(), torch.from_numpy(Q).cuda()
    del X
    log(f"[bench] data {w.name} N={w.n} D={w.dim} nq={w.nq}: {time.perf_counter() - t0:.1f}s")
    gt = exact_knn_gpu(Xd, Qd, w.k, w.metric)

    # ---- headline point: the workload as stated ----
    gi, build_s = build_index(Xd, w, w.total_bits, args.eps0)
    log(f"[bench] index build on the device (B={w.total_bits}): {build_s:.3f}s")
    cluster_sizes = cluster_sizes_of(gi)
    pt = measure_point(gi, Qd, gt, w, w.total_bits, args, f"B={w.total_bits}")
    roofline = scan_roofline(gi, Qd, w, pt, cluster_sizes, args)
    impl = args.scan_impl if args.scan_impl != 3 else (1 if w.dim >= 960 else 0)
    config = {"workload": f"{w.name}: N={w.n} D={w.dim} nlist={w.nlist} B={w.total_bits} nq={w.nq} k={w.k} "
                          f"nprobe={pt['nprobe']}",
              "recall_at_k": pt["recall_at_k"], "recall_at_k_unpruned": pt["recall_at_k_unpruned"],
              "recall_target": RECALL_TARGET, "recall_target_met": pt["recall_at_k"] >= RECALL_TARGET,
              "nprobe_sweep": pt["nprobe_sweep"], "stage_ms": pt["stage_ms"], "stage_ms_calls": pt["stage_ms_calls"],
              "stage_ms_note": "separate pass with every stage's events recorded; list_build and scan_setup run on a "
                               "second stream beside seed, so the stages add up to more than ms_per_step",
              "index_builder": "rabitq_index_build (HIP: k-means + two-phase grid search"
                               + (", vectors centred on their mean)" if w.metric == "l2" else ")"),
              "index_build_s": round(build_s, 4)}
    if (args.batch_sweep or args.workload == "l2_128") and not args.no_batch_sweep:
        config["batch_sweep"] = batch_sweep(gi, Qd, w, pt["nprobe"])
    cpu = None
    if not args.no_cpu_baseline:
        t0 = time.perf_counter()
        cpu = cpu_baseline(gi, Q, w.k, pt["nprobe"])
        log(f"[bench] cpu baseline: {cpu['value']:.1f} q/s on {cpu['cores']} threads ({time.perf_counter() - t0:.1f}s)")
    gi.close()

    # ---- the same workload at the smallest code size that reaches the recall target ----
    if not config["recall_target_met"] and args.target_bits != 0:
        cands = [args.target_bits] if args.target_bits > 0 else list(range(w.total_bits + 1, 9))
        for bits in cands:
            gi2, b2 = build_index(Xd, w, bits, args.eps0)
            pt2 = measure_point(gi2, Qd, gt, w, bits, args, f"B={bits}")
            if pt2["recall_at_k"] >= RECALL_TARGET or bits == cands[-1]:
                pt2["roofline"] = scan_roofline(gi2, Qd, w, pt2, cluster_sizes_of(gi2), args)
                pt2["index_build_s"] = round(b2, 4)
                pt2["queries_per_s"] = pt2.pop("qps")
                pt2["note"] = (f"same data, queries and lists; {bits} bits per dimension instead of {w.total_bits}: the "
                               f"smallest code size whose recall@{w.k} reaches {RECALL_TARGET}")
                config["point_at_recall_target"] = pt2
                gi2.close()
                break
            gi2.close()
    del Xd

    # ---- the scan kernel in the streaming regime (HBM roofline) ----
    if not args.no_stream:
        roofline["stream"] = stream_scan(args, args.stream_n or 32 * 1024 * 1024, args.stream_bits, 20, 3)
        log(f"[bench] streaming scan: {roofline['stream']['achieved']:.0f} GB/s = {roofline['stream']['frac']:.3f} of peak")

    res = {
        "metric": "queries/sec at recall@10~0.95 (1 GPU); code-scan HBM GB/s vs peak",
        "value": pt["qps"], "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": pt["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("i8 matrix cores + f32" if pt.get("scan_split") or impl == 1 else
                  "f16 tables + f32" if impl == 2 else "u32 popcount + f32"), "data": "synthetic",
        "config": config, "roofline": roofline,
    }
    if cpu is not None:
        res["cpu_baseline"] = cpu
    if args.pmc_calibration:
        cal = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        cal2 = cal + 1.0
        torch.cuda.synchronize()
        del cal, cal2
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
