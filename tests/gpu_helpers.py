"""Shared helpers of the GPU parity tests: oracle-side stage outputs and comparison rules."""
from __future__ import annotations

import numpy as np
import torch

from oracle import build, search
from paper_2602_23999_amd import rabitq


def upload(ix: dict) -> rabitq.Index:
    return rabitq.index_from_arrays(ix, build.pack_device_layout(ix))


def oracle_stages(s: search.Searcher, Q: np.ndarray, k: int, nprobe: int) -> dict:
    """Every intermediate of the search as the oracle computes it (numpy)."""
    ix = s.ix
    Qr = search.rotate_queries(Q, ix["P"], ix.get("mean"))
    nq, D = Qr.shape
    W = D // 32
    planes = np.empty((nq, 4, W), np.uint32)
    delta = np.empty(nq, np.float32)
    S = np.empty(nq, np.int32)
    for i in range(nq):
        d, qh, s_ = search.quantize_query(Qr[i])
        planes[i] = search.query_bitplanes(qh)
        delta[i], S[i] = d, s_
    Qr64 = Qr.astype(np.float64)
    probes, G, E = search.coarse_probe(Qr, ix["centroids_rot"], nprobe, s.metric)
    # pairs p = q*nprobe + rank grouped by cluster, stable in p (hence in query id)
    flat = probes.reshape(-1)
    order = np.argsort(flat, kind="stable").astype(np.int32)
    counts = np.bincount(flat, minlength=ix["nlist"])
    pair_off = np.zeros(ix["nlist"] + 1, np.int32)
    pair_off[1:] = np.cumsum(counts)
    tau = np.array([s.seed_threshold(probes[i], G[i], E[i], Qr[i], delta[i], planes[i], int(S[i]), k)
                    for i in range(nq)])
    qhat = np.zeros((nq, (D + 63) // 64 * 64), np.int8)
    for i in range(nq):
        qhat[i, :D] = search.quantize_query(Qr[i])[1]
    F = 0 if ix["total_bits"] == 1 else build.long_field_bits(ix["total_bits"])
    lut = np.stack([search.lut_tables(Qr[i]) for i in range(nq)])
    return dict(lut=lut, Qr=Qr, qhat=qhat, q_stage=stage_order(Qr, F), planes=planes, delta=delta, S=S, sum_q=Qr64.sum(1),
                sq_norm=(Qr64 ** 2).sum(1),
                probes=probes, G=G, E=E, pair_off=pair_off, pair_ids=order, tau=tau)


def stage_order(Qr: np.ndarray, F: int) -> np.ndarray:
    """q' in the order the refinement reads it (include/rabitq.h, q_stage): within each
    long-code word of 32/F dimensions, dimension b*(8/F)+s sits at position 4*s+b."""
    if F == 0:
        return Qr.copy()
    D = Qr.shape[1]
    dpw, spb = 32 // F, 8 // F
    d = np.arange(D)
    w, r = d // dpw, d % dpw
    pos = w * dpw + (r % spb) * 4 + (r // spb)
    out = np.empty_like(Qr)
    out[:, pos] = Qr
    return out


def to_dev(st: dict, dev="cuda") -> dict:
    t = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a.astype(dt))).to(dev)
    prep = dict(planes=t(st["planes"].view(np.int32), np.int32), delta=t(st["delta"], np.float32),
                sum_qhat=t(st["S"], np.int32), sum_q=t(st["sum_q"], np.float32), sq_norm=t(st["sq_norm"], np.float32),
                qhat8=t(st["qhat"], np.int8), q_stage=t(st["q_stage"], np.float32), lut=t(st["lut"], np.float16))
    probes = dict(probe_ids=t(st["probes"], np.int32), probe_G=t(st["G"], np.float32), probe_E=t(st["E"], np.float32))
    return dict(q_rot=t(st["Qr"], np.float32), prep=prep, probes=probes, pair_off=t(st["pair_off"], np.int32),
                pair_ids=t(st["pair_ids"], np.int32),
                tau=t(np.minimum(st["tau"], rabitq.FLT_MAX), np.float32))


def compare_topk(g_ids, g_d, o_ids, o_d, atol_q, rtol=1e-4):
    """Parity rule for final results: distances agree position by position within
    rtol/atol; ids agree as sets except for members whose key ties (within tolerance)
    with the k-th key, where several answers are correct.  Returns the number of queries
    whose id lists are exactly equal."""
    nq, k = o_ids.shape
    exact = 0
    for q in range(nq):
        tol = atol_q[q] + rtol * np.abs(o_d[q])
        fin = np.isfinite(o_d[q])
        assert np.array_equal(np.isfinite(g_d[q]), fin), f"query {q}: padding differs"
        assert np.all(np.abs(g_d[q][fin] - o_d[q][fin]) <= tol[fin]), \
            f"query {q}: dist mismatch {g_d[q]} vs {o_d[q]}"
        if np.array_equal(g_ids[q], o_ids[q]):
            exact += 1
            continue
        # a differing order or member must be explained by keys that tie within tolerance
        for a, b in ((g_ids[q], o_ids[q]), (o_ids[q], g_ids[q])):
            da = g_d[q] if a is g_ids[q] else o_d[q]
            for pos, i in enumerate(a):
                if i < 0:
                    continue
                if i in b:
                    pb = int(np.nonzero(b == i)[0][0])
                    if pb != pos:  # reordered: the keys in between must tie
                        lo, hi = min(pos, pb), max(pos, pb)
                        assert abs(o_d[q][hi] - o_d[q][lo]) <= 2 * tol[lo:hi + 1].max(), f"query {q}: order differs without a tie"
                else:          # dropped from the other list: must tie with the k-th key
                    last = o_d[q][fin][-1]
                    assert abs(da[pos] - last) <= 2 * tol[fin][-1], f"query {q}: id {i} differs without a tie at rank k"
    return exact
