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
    pos = qhat8_positions(D)
    for i in range(nq):
        qhat[i, pos] = search.quantize_query(Qr[i])[1]
    F = 0 if ix["total_bits"] == 1 else build.long_field_bits(ix["total_bits"])
    lut = np.stack([search.lut_tables(Qr[i]) for i in range(nq)])
    return dict(lut=lut, Qr=Qr, qhat=qhat, q_stage=stage_order(Qr, F), planes=planes, delta=delta, S=S, sum_q=Qr64.sum(1),
                sq_norm=(Qr64 ** 2).sum(1),
                probes=probes, G=G, E=E, pair_off=pair_off, pair_ids=order, tau=tau)


def qhat8_positions(D: int) -> np.ndarray:
    """Byte position of every dimension in the library's qhat8 array (include/rabitq.h): within each chunk of 64
    dimensions, dimension 32 w + 8 b + 4 h + i sits at byte 16 (2 w + h) + 4 i + b."""
    d = np.arange(D)
    c, r = d >> 6, d & 63
    w, x = r >> 5, r & 31
    return 64 * c + 16 * (2 * w + ((x >> 2) & 1)) + 4 * (x & 3) + (x >> 3)


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


# --------------------------------------------------------------------------------------
# End-to-end comparison in which every difference has to be accounted for.
#
# The GPU's rotated query differs from the oracle's fp64 one in the last fp32 place.  That
# can move a 4-bit digit that sits on a rounding boundary, swap two clusters whose coarse
# scores tie, swap two seeds whose 1-bit estimates tie, or move a vector whose bound ties
# with the threshold across it.  Nothing else may differ.  The check follows the pipeline:
# each GPU stage output is compared with the oracle's for the same input (differences must
# be one of those ties, shown by the oracle's own numbers), and the final result must equal
# the oracle's search run from the GPU's stage outputs, up to vectors whose filter value
# lies within tolerance of the threshold and keys that tie within tolerance.
# --------------------------------------------------------------------------------------
def key_scale(G, E, metric):
    """Size of the terms an estimate is a difference of, per query: tolerances are relative to it."""
    if metric == "l2":
        return np.abs(G).max(axis=1) + 1e-6
    return np.abs(G).max(axis=1) + (E ** 2).max(axis=1) + 1e-6


def gpu_stage_outputs(gi, Qd, k, nprobe, prune=True):
    q_rot = gi.rotate(Qd)
    prep = gi.query_prep(q_rot)
    probes = gi.coarse_probe(q_rot, prep["sq_norm"], nprobe)
    if prune:
        tau = gi.seed_threshold(prep, probes, k)
    else:
        tau = torch.full((Qd.shape[0],), rabitq.FLT_MAX, dtype=torch.float32, device=Qd.device)
    torch.cuda.synchronize()
    return dict(Qr=q_rot.cpu().numpy(), sq_norm=prep["sq_norm"].cpu().numpy().astype(np.float64),
                probes=probes["probe_ids"].cpu().numpy(), G=probes["probe_G"].cpu().numpy().astype(np.float64),
                E=probes["probe_E"].cpu().numpy().astype(np.float64), tau=tau.cpu().numpy().astype(np.float64))


def explain_stage_differences(s: search.Searcher, Q, g: dict, k: int, nprobe: int, prune=True) -> dict:
    """Asserts that the GPU's stage outputs `g` differ from the oracle's only by the allowed ties; returns counts."""
    ix = s.ix
    nq = Q.shape[0]
    Qr_o = search.rotate_queries(Q, ix["P"], ix.get("mean"))
    norm = np.linalg.norm(Qr_o.astype(np.float64), axis=1)
    assert np.all(np.abs(g["Qr"].astype(np.float64) - Qr_o) <= 1e-6 * norm[:, None]), "rotation"
    caused = np.zeros(nq, bool)  # queries with a recorded reason to differ from the oracle's own run
    # digits: a digit may differ only where q'/delta lies within 1e-4 of a half
    # (the lookup-table variant does not quantise the query; its tables follow from q' bit for bit, so there a
    # query whose q' differs at all is one whose binary16 table entries may differ)
    flips = 0
    if s.ip_method != "bitwise":
        caused |= np.array([not np.array_equal(search.lut_tables(Qr_o[i]).view(np.uint16),
                                               search.lut_tables(g["Qr"][i]).view(np.uint16)) for i in range(nq)])
    for i in range(nq if s.ip_method == "bitwise" else 0):
        d_o, qh_o, _ = search.quantize_query(Qr_o[i])
        d_g, qh_g, _ = search.quantize_query(g["Qr"][i])
        bad = np.nonzero(qh_o != qh_g)[0]
        if len(bad):
            t = Qr_o[i].astype(np.float64)[bad] / float(d_o)
            assert np.all(np.abs((t - np.floor(t)) - 0.5) <= 1e-4), f"query {i}: digit differs away from a rounding boundary"
            assert np.all(np.abs(qh_o[bad].astype(int) - qh_g[bad].astype(int)) == 1)
            flips += len(bad)
            caused[i] = True
    # probes: for the GPU's own rotated queries, a differing probe must tie in score
    p_o, G_o, E_o = search.coarse_probe(g["Qr"], ix["centroids_rot"], nprobe, s.metric)
    scale = g["sq_norm"][:, None] + 1.0
    assert np.all(np.abs(g["G"] - G_o) <= 2e-6 * scale), "coarse scores"
    diff = g["probes"] != p_o
    # (a probe of the oracle's own run that differs although the GPU agrees with the oracle on the GPU's q' is a
    # near-tie too: the two q' differ in the last place)
    p_own = search.coarse_probe(Qr_o, ix["centroids_rot"], nprobe, s.metric)[0]
    caused |= diff.any(axis=1) | (p_own != p_o).any(axis=1)
    # (scores agree rank by rank, so a differing id at a rank means two clusters within tolerance of each other)
    probe_ties = int(diff.sum())
    if probe_ties:
        # the displaced cluster's score must lie within tolerance of the score at that rank
        dot = g["Qr"].astype(np.float64) @ ix["centroids_rot"].astype(np.float64).T
        sc = (-dot if s.metric == "ip" else g["sq_norm"][:, None] + (ix["centroids_rot"].astype(np.float64) ** 2).sum(1)[None, :] - 2 * dot)
        qi, ri = np.nonzero(diff)
        assert np.all(np.abs(sc[qi, g["probes"][qi, ri]] - G_o[qi, ri]) <= 4e-6 * scale[qi, 0]), "probe differs without a tie"
    # threshold: from the GPU's own probes; a difference needs a tie among the seed candidates
    tau_ties = 0
    if prune:
        ks = key_scale(g["G"], g["E"], s.metric)
        for i in range(nq):
            d_g, qh_g, S_g = search.quantize_query(g["Qr"][i])
            planes = search.query_bitplanes(qh_g)
            want = min(s.seed_threshold(g["probes"][i], g["G"][i], g["E"][i], g["Qr"][i], d_g, planes, S_g, k), rabitq.FLT_MAX)
            if abs(g["tau"][i] - want) <= 1e-4 * (abs(want) + ks[i]):
                continue
            # which cluster seeded, and is the choice of its M best 1-bit candidates (or of the k-th) a near-tie?
            m = max(k, s.seed_m)
            for c, G, E in zip(g["probes"][i], g["G"][i], g["E"][i]):
                a, b = int(ix["offsets"][c]), int(ix["offsets"][c + 1])
                if b - a < k:
                    continue
                _, _, _, est1, _ = s.pair(c, G, E, g["Qr"][i], d_g, planes, S_g)
                e = np.sort(est1)
                cut = (k if s.B == 1 else m)
                assert b - a > cut and abs(e[cut] - e[cut - 1]) <= 1e-5 * (abs(e[cut]) + ks[i]), \
                    f"query {i}: threshold {g['tau'][i]} vs {want} without a tie among the seeds"
                break
            tau_ties += 1
            caused[i] = True
    return dict(digit_flips=flips, probe_ties=probe_ties, tau_ties=tau_ties, caused=caused)


def oracle_from_stages(s: search.Searcher, Q, g: dict, k: int, nprobe: int):
    """The oracle's search run from the GPU's own stage outputs (rotated queries, probes, thresholds)."""
    return s.search(Q, k, nprobe, prune=True, Qr=g["Qr"], probes=(g["probes"], g["G"], g["E"]), tau=g["tau"],
                    detail=True)


def check_final(s: search.Searcher, ora, ids, dist, k: int, only=None) -> int:
    """The GPU's final result against `ora` = (ids, dists, info) of an oracle search run with detail=True on the same
    stage outputs.  Every difference must be a key tie within tolerance or a vector whose filter value lies within
    tolerance of the threshold.  `only`: the queries to look at (default all).  Returns the number of them whose
    id lists are exactly equal."""
    o_ids, o_d, info = ora
    ks = key_scale(info["G"], info["E"], s.metric)
    exact = 0
    sign = -1.0 if s.metric == "ip" else 1.0
    for q in (range(o_ids.shape[0]) if only is None else only):
        try:
            exact += compare_topk(ids[q:q + 1], dist[q:q + 1], o_ids[q:q + 1], o_d[q:q + 1], 1e-4 * ks[q:q + 1])
            continue
        except AssertionError:
            pass
        # vectors whose filter value lies within tolerance of the threshold may fall either way in fp32
        d = info["details"][q]
        tol = 1e-5 * (abs(d["tau"]) + ks[q])
        certain = d["filt"] <= d["tau"] - tol
        maybe = np.abs(d["filt"] - d["tau"]) <= tol
        assert maybe.any(), f"query {q}: result differs and no vector sits on the threshold"
        got = ids[q][ids[q] >= 0]
        assert np.all(np.isin(got, d["ids"][certain | maybe])), f"query {q}: a result was filtered out by the oracle"
        allowed = certain | (maybe & np.isin(d["ids"], got))
        rk, ri = search.topk_pairs(d["keys"][allowed], d["ids"][allowed], k)
        w_ids = np.full((1, k), -1, np.int64)
        w_d = np.full((1, k), np.inf)
        w_ids[0, :len(ri)] = ri
        w_d[0, :len(rk)] = rk
        compare_topk(ids[q:q + 1], dist[q:q + 1], w_ids, sign * w_d, 1e-4 * ks[q:q + 1])
    return exact


def search_explained(gi, s: search.Searcher, Q, k: int, nprobe: int, prune=True, cache: dict | None = None,
                     sample=None):
    """rabitq_search on the whole batch, with every difference from the oracle accounted for (see above).
    `gi` must already have the scan_impl under test selected.  `sample` (sorted query indices): the GPU runs the
    whole batch, the oracle-side work is done for these queries only and the returned arrays hold their rows.
    `cache` (a dict) keeps the oracle-side work between calls whose stage outputs are the same.
    Returns (ids, dists, counts)."""
    Qd = torch.from_numpy(Q).cuda()
    gi.set_option("prune", int(prune))
    try:
        ids, dist = gi.search(Qd, k, nprobe)
        g = gpu_stage_outputs(gi, Qd, k, nprobe, prune)
    finally:
        gi.set_option("prune", 1)
    ids, dist = ids.cpu().numpy(), dist.cpu().numpy().astype(np.float64)
    if sample is not None:
        ids, dist, Q = ids[sample], dist[sample], Q[sample]
        g = {n: v[sample] for n, v in g.items()}
    key = (s.ip_method, bool(prune), k, nprobe)
    hit = cache.get(key) if cache is not None else None
    if hit is not None and all(np.array_equal(hit[0][n], g[n]) for n in g):
        _, why, ora = hit
    else:
        why = explain_stage_differences(s, Q, g, k, nprobe, prune)
        ora = oracle_from_stages(s, Q, g, k, nprobe)
        if cache is not None:
            cache[key] = (g, why, ora)
    why = dict(why, exact=check_final(s, ora, ids, dist, k), nq=len(Q))
    return ids, dist, why


def check_against_own_run(s: search.Searcher, own, ids, dist, k: int, why: dict) -> int:
    """`own` = the oracle's search on its own fp64 path (detail=True).  A query whose GPU result differs from it
    must have a recorded cause in the stages (why["caused"]) or differ only by final-key ties / vectors on the
    threshold.  Returns the number of queries with identical id lists."""
    same = np.array([np.array_equal(a, b) for a, b in zip(ids, own[0])])
    need = np.nonzero(~same & ~why["caused"])[0]
    check_final(s, own, ids, dist, k, only=need)
    return int(same.sum())

