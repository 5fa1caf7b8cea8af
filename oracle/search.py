"""Oracle batched search (TEST INFRASTRUCTURE ONLY; see package header).

The steps follow Section 3.3 in the paper's order: rotate the batch (3.3.1),
select clusters (3.3.2), prepare the per-query representation once (3.3.3),
cluster-local two-stage estimation (3.3.4) with the bitwise inner product of
Section 3.4.1(2), and the per-query merge (3.3.5).  Floating point is float64
except where a stored format or an integer decision fixes fp32 (stated below).

Readings taken where the paper is silent
----------------------------------------
* Query quantisation (Section 3.4.1(2) gives neither scale nor rounding):
  ``delta = max|q'| / 7``, ``qhat = clamp(rint(q'/delta), -7, 7)`` (round half to
  even), both evaluated in fp32 because they decide integers; 4 two's-complement
  bit-planes, plane 3 weighted -8.
* Lookup-table variant (Section 3.4.1(1), U = 4; the paper fixes neither the
  stored type nor the summation): ``L_j(b)`` is the fp32 sum, in ascending
  dimension order, of the ``q'[4j+i]`` whose bit ``b_i`` is set (bit i of the
  table index is dimension 4j+i), stored as binary16 (the paper's FP16
  example); ``<x_b, q'>`` is the fp32 sum of the looked-up entries in ascending
  block order.  Both are precision decisions of the variant, so they are part of
  its definition here.  The query is not quantised in this variant.
* Refinement uses the unquantised fp32 ``q'`` (Section 3.4.2 does not say in
  which precision the query enters).
* Threshold (Section 3.3.4: the K-th best distance found so far): the running value is
  order dependent on a parallel machine, so it is fixed per query before the
  scan, as the K-th best distance after a first look at the nearest cluster.  In
  the query's nearest probed cluster holding at least K vectors, the
  ``M = max(K, SEED_M)`` vectors with the smallest 1-bit estimates (all of them if
  the cluster is smaller; ties to the lower position) are refined and ``tau`` is
  the K-th smallest of their refined estimates (for B = 1: the K-th smallest
  1-bit estimate).  Every probed cluster is then filtered with that one ``tau``:
  a vector survives when its 1-bit lower bound (B = 1: its 1-bit estimate) is
  <= tau.  The bound of the bitwise scheme also covers the rounding error of the
  4-bit query (bound_radius below); the lookup-table scheme has no such error.  ``tau`` is always >= the final K-th best key of the unpruned search,
  because K scanned vectors have keys <= tau.
* Result: the K smallest (key, id) among survivors; L2 keys are estimated squared
  distances, IP keys are negated estimated inner products.

Parity status
-------------
rotate_queries, coarse_probe  pinned: direct ||q'-c'||^2 loop, full argsort.
quantize_query, bitplanes     pinned: |delta*qhat - q'| <= delta/2, planes
                              reassemble to qhat, storage size of Section 3.4.1.
ip_bitplane                   pinned: exhaustive identity of Section 3.4.1(2).
lut_tables / ip_lut           pinned: every entry against the fp64 dot product of
                              its block within binary16 rounding, the table
                              size of Section 3.4.1(1), the blockwise sum against
                              the fp64 <x_b, q'> within the rounding bound, and
                              exactness on queries whose partial sums are
                              representable.
estimate_1bit / _refined      pinned via build.vector_factors pins; refined
                              estimate error shrinking with B is a trend only
                              ("parity unpinned" for its exact values).
search                        pinned: brute force on tiny inputs (nprobe = nlist,
                              B = 8 recovers exact kNN), pruned == unpruned
                              whenever the oracle's own predicate holds.
"""
from __future__ import annotations

import numpy as np

from .build import short_words

FLT_MAX = float(np.finfo(np.float32).max)
BQ = 4  # query bits (Section 3.4.1(2) example)
SEED_M = 32  # 1-bit candidates refined to seed the threshold (at least K are taken)


# ---- 3.3.1 -----------------------------------------------------------------
def rotate_queries(Q: np.ndarray, P: np.ndarray, mean: np.ndarray | None = None) -> np.ndarray:
    """``Q' = (Q - mean) P`` evaluated in float64 and stored as fp32 [nq, D]; ``mean`` is the
    translation of a centred index (none or zeros otherwise)."""
    q = np.asarray(Q, np.float64)
    if mean is not None:
        q = q - np.asarray(mean, np.float64)[None, :]
    return (q @ np.asarray(P, np.float64)).astype(np.float32)


# ---- 3.3.2 -----------------------------------------------------------------
def coarse_probe(Qr: np.ndarray, C_rot: np.ndarray, nprobe: int, metric: str):
    """Nearest ``nprobe`` clusters per query by the matrix form
    ``s_q 1^T + 1 s_c^T - 2 Q' C^T`` (Section 3.3.2); ties go to the lower
    cluster id.  Returns (probe ids [nq,nprobe] i32, G [nq,nprobe] f64,
    E [nq,nprobe] f64) where G is the additive term of the estimator
    (L2: ||q'-c'||^2, IP: -<q',c'>) and E = ||q'-c'||."""
    q = np.asarray(Qr, np.float64)
    c = np.asarray(C_rot, np.float64)
    sq = np.einsum("ij,ij->i", q, q)
    sc = np.einsum("ij,ij->i", c, c)
    dot = q @ c.T
    d2 = sq[:, None] + sc[None, :] - 2.0 * dot
    score = d2 if metric == "l2" else -dot
    nlist = c.shape[0]
    # lexicographic (score, cluster id): stable argsort on score
    order = np.argsort(score, axis=1, kind="stable")[:, :nprobe]
    G = np.take_along_axis(score, order, axis=1)
    E = np.sqrt(np.maximum(np.take_along_axis(d2, order, axis=1), 0.0))
    assert nprobe <= nlist
    return order.astype(np.int32), G, E


# ---- 3.3.3 / 3.4.1(2) --------------------------------------------------------
def quantize_query(qr: np.ndarray):
    """4-bit signed quantisation of one rotated query (fp32 arithmetic).
    Returns (delta f32, qhat int8 [D], S = sum(qhat) int)."""
    qr = np.asarray(qr, dtype=np.float32)
    amax = np.float32(np.max(np.abs(qr)))
    if amax == np.float32(0.0):
        return np.float32(1.0), np.zeros(qr.shape[0], np.int8), 0
    delta = np.float32(amax / np.float32(7.0))
    t = (qr / delta).astype(np.float32)
    qhat = np.clip(np.rint(t), -7, 7).astype(np.int8)
    return delta, qhat, int(qhat.astype(np.int64).sum())


def query_bitplanes(qhat: np.ndarray) -> np.ndarray:
    """Two's-complement bit-planes [4, W] uint32; bit i of word w of plane j is
    bit j of qhat[32w+i] (Figure 1's q^(j))."""
    D = qhat.shape[0]
    tc = (qhat.astype(np.int64) & 0xF).astype(np.uint32).reshape(D // 32, 32)
    sh = np.arange(32, dtype=np.uint32)
    planes = np.empty((BQ, D // 32), dtype=np.uint32)
    for j in range(BQ):
        planes[j] = (((tc >> np.uint32(j)) & np.uint32(1)) << sh[None, :]).sum(axis=1, dtype=np.uint64)
    return planes


def ip_bitplane(xb_words: np.ndarray, planes: np.ndarray) -> np.ndarray:
    """``<x_b, qhat>`` for packed 1-bit codes [n, W] by AND + popcount over the
    bit-planes: ``-8 pc(x & q3) + 4 pc(x & q2) + 2 pc(x & q1) + pc(x & q0)``."""
    out = np.zeros(xb_words.shape[0], dtype=np.int64)
    for j in range(BQ):
        pc = np.bitwise_count(xb_words & planes[j][None, :]).sum(axis=1, dtype=np.int64)
        w = -(1 << (BQ - 1)) if j == BQ - 1 else (1 << j)
        out += w * pc
    return out


# ---- 3.4.1(1) ----------------------------------------------------------------
LUT_U = 4  # dimensions per lookup block


def lut_tables(qr: np.ndarray) -> np.ndarray:
    """Lookup tables of one rotated query: ``[D/4, 16]`` binary16 with
    ``L_j(b) = sum_i q'[4j+i] b_i`` (bit i of b is dimension 4j+i), the sum taken in
    fp32 in ascending i and then rounded to binary16."""
    qr = np.asarray(qr, dtype=np.float32)
    m = qr.shape[0] // LUT_U
    t = np.zeros((m, 1 << LUT_U), dtype=np.float32)
    for b in range(1 << LUT_U):
        acc = np.zeros(m, dtype=np.float32)
        for i in range(LUT_U):
            if (b >> i) & 1:
                acc = (acc + qr[i::LUT_U][:m]).astype(np.float32)
        t[:, b] = acc
    return t.astype(np.float16)


def ip_lut(xb_words: np.ndarray, tables: np.ndarray) -> np.ndarray:
    """``<x_b, q'>`` for packed 1-bit codes [n, W] by one table lookup per block of
    4 dimensions, summed in fp32 in ascending block order.  Returns fp32 [n]."""
    n = xb_words.shape[0]
    m = tables.shape[0]
    acc = np.zeros(n, dtype=np.float32)
    per_word = 32 // LUT_U
    for j in range(m):
        nib = (xb_words[:, j // per_word] >> np.uint32(LUT_U * (j % per_word))) & np.uint32(15)
        acc = (acc + tables[j][nib].astype(np.float32)).astype(np.float32)
    return acc


def estimate_1bit_lut(G, E, short_factors, ip, sum_q):
    """1-bit estimate and lower bound from ``ip = <x_b, q'>``:
    ``<x_bar, q'> = ip - sum(q')/2`` with ``x_bar = u_b - 1/2``."""
    f = short_factors.astype(np.float64)
    ipq = ip.astype(np.float64) - 0.5 * float(sum_q)
    est = G + f[:, 0] + f[:, 1] * ipq
    lb = est - f[:, 2] * E
    return est, lb


# The 4-bit query's rounding errors (Section 3.4.1(2)) are a second, independent error of the 1-bit estimate: dimension
# i contributes f_rescale * x_bar_i * e_i with x_bar_i = +-1/2 and e_i = q'_i - delta*qhat_i in [-delta/2, delta/2]
# (no clamping error, since delta = max|q'|/7), variance delta^2/12.  Their sum has standard deviation
# |f_rescale| * delta * sqrt(D/48); in units of the code's own error scale f_err * ||q'-c'|| / eps0 (oracle.build.
# vector_factors) that is sqrt((D-1) delta^2 / (12 (1-a^2))) / ||q'-c'||, a = the code's alignment <x,o'>/||x||.  Both
# errors are zero-mean and independent, so the lower bound of Section 3.3.4 keeps its confidence when ||q'-c'|| is
# replaced by sqrt(||q'-c'||^2 + (D-1) delta^2 / (12 (1-a^2))).  For 1-bit codes a^2 concentrates at 2/pi (pinned in
# tests/test_oracle_encode.py), which makes the widening a per-(query, cluster) scalar.
QUANT_ERR_VAR = 1.0 / 12.0            # variance of one rounding error in units of delta^2 (uniform on [-1/2, 1/2])
ONE_BIT_MISALIGN = 1.0 - 2.0 / np.pi  # 1 - a^2 of a 1-bit code in the large-D limit


def bound_radius(E, delta, D):
    """``||q'-c'||`` widened by the 4-bit query's rounding error (see above); ``E`` may be an array."""
    return np.sqrt(np.asarray(E, np.float64) ** 2 + (D - 1.0) * float(delta) ** 2 * QUANT_ERR_VAR / ONE_BIT_MISALIGN)


def estimate_1bit(G, E, short_factors, delta, I, S):
    """1-bit estimate and its lower bound for one (query, cluster) pair; ``E`` is the radius the error factor
    multiplies (bound_radius for a quantised query).
    ``<x_bar, q'> ~= delta * (I - S/2)`` with ``x_bar = u_b - 1/2``."""
    f = short_factors.astype(np.float64)
    ipq = float(delta) * (2.0 * I.astype(np.float64) - float(S)) / 2.0
    est = G + f[:, 0] + f[:, 1] * ipq
    lb = est - f[:, 2] * E
    return est, lb


def estimate_refined(G, long_factors, u, qr, total_bits):
    """Refined estimate from the full code: ``<x, q'> = <u, q'> - c_B sum(q')``."""
    f = long_factors.astype(np.float64)
    q = qr.astype(np.float64)
    cB = ((1 << total_bits) - 1) / 2.0
    ipq = u.astype(np.float64) @ q - cB * q.sum()
    return G + f[:, 0] + f[:, 1] * ipq


def topk_pairs(keys: np.ndarray, ids: np.ndarray, k: int):
    """The k smallest (key, id) pairs in ascending lexicographic order."""
    order = np.lexsort((ids, keys))[:k]
    return keys[order], ids[order]


class Searcher:
    """Holds an index (oracle.build.build_index output) and answers batches."""

    def __init__(self, index: dict, ip_method: str = "bitwise", seed_m: int = SEED_M):
        """``ip_method``: "bitwise" (Section 3.4.1(2), the default) or "lut"
        (Section 3.4.1(1)) for the 1-bit inner product.  ``seed_m``: number of 1-bit
        candidates refined when the threshold is seeded (see the module header)."""
        assert ip_method in ("bitwise", "lut")
        self.ip_method = ip_method
        self.seed_m = seed_m
        self.ix = index
        self.words = short_words(index)  # [N, W] packed 1-bit codes
        self.B = index["total_bits"]
        self.metric = index["metric"]

    # one (query, cluster) pair: all stage outputs
    def pair(self, c, G, E, qr, delta, planes, S):
        ix = self.ix
        s, e = int(ix["offsets"][c]), int(ix["offsets"][c + 1])
        if self.ip_method == "lut":
            I = ip_lut(self.words[s:e], lut_tables(qr))
            est1, lb1 = estimate_1bit_lut(G, E, ix["short_factors"][s:e], I, np.asarray(qr, np.float64).sum())
            return s, e, I, est1, lb1
        I = ip_bitplane(self.words[s:e], planes)
        est1, lb1 = estimate_1bit(G, bound_radius(E, delta, ix["dim"]), ix["short_factors"][s:e], delta, I, S)
        return s, e, I, est1, lb1

    def refined(self, s, e, G, qr, sel=None):
        ix = self.ix
        rows = np.arange(s, e) if sel is None else s + sel
        return estimate_refined(G, ix["long_factors"][rows], ix["u"][rows], qr, self.B)

    def seed_threshold(self, probes, Gs, Es, qr, delta, planes, S, k):
        """tau for one query (see module header)."""
        ix = self.ix
        for c, G, E in zip(probes, Gs, Es):
            s, e = int(ix["offsets"][c]), int(ix["offsets"][c + 1])
            if e - s < k:
                continue
            _, _, _, est1, _ = self.pair(c, G, E, qr, delta, planes, S)
            order = np.lexsort((np.arange(e - s), est1))  # by (1-bit estimate, position in the cluster)
            if self.B == 1:
                return float(est1[order[k - 1]])
            sel = order[:max(k, self.seed_m)]
            return float(np.sort(self.refined(s, e, G, qr, sel))[k - 1])
        return FLT_MAX

    def search(self, Q, k, nprobe, prune=True, Qr=None, detail=False, tau=None, probes=None):
        """Returns (ids [nq,k] i64, dists [nq,k] f64, info).  ``prune=False`` is
        the unpruned definition (every vector of every probed cluster is ranked by
        its final key).  ``info`` holds per-query tau, survivor counts, the probe
        lists, and the count of unpruned top-k members the filter would drop.
        Stage tests may replace the outcome of an earlier step by given values: ``Qr``
        (rotated queries), ``probes`` = (ids [nq,nprobe], G, E) in place of the cluster
        selection, ``tau`` [nq] in place of the seeded thresholds."""
        ix = self.ix
        if Qr is None:
            Qr = rotate_queries(Q, ix["P"], ix.get("mean"))
        nq = Qr.shape[0]
        if probes is None:
            probes, G, E = coarse_probe(Qr, ix["centroids_rot"], nprobe, self.metric)
        else:
            probes, G, E = (np.asarray(probes[0], np.int32), np.asarray(probes[1], np.float64),
                            np.asarray(probes[2], np.float64))
            assert probes.shape == (nq, nprobe)
        out_ids = np.full((nq, k), -1, dtype=np.int64)
        out_d = np.full((nq, k), np.inf, dtype=np.float64)
        taus = np.full(nq, FLT_MAX)
        n_scanned = np.zeros(nq, np.int64)
        n_surv = np.zeros(nq, np.int64)
        dropped = np.zeros(nq, np.int64)
        details = []
        for qi in range(nq):
            qr = Qr[qi]
            delta, qhat, S = quantize_query(qr)
            planes = query_bitplanes(qhat)
            if tau is None:
                tau_q = self.seed_threshold(probes[qi], G[qi], E[qi], qr, delta, planes, S, k)
            else:
                tau_q = float(tau[qi])
            taus[qi] = tau_q
            keys_all, ids_all, filt_all = [], [], []
            for j in range(nprobe):
                c = int(probes[qi, j])
                s, e, I, est1, lb1 = self.pair(c, G[qi, j], E[qi, j], qr, delta, planes, S)
                if e == s:
                    continue
                key = est1 if self.B == 1 else self.refined(s, e, G[qi, j], qr)
                filt = est1 if self.B == 1 else lb1
                keys_all.append(key)
                ids_all.append(ix["ids"][s:e].astype(np.int64))
                filt_all.append(filt)
            if keys_all:
                keys = np.concatenate(keys_all)
                ids = np.concatenate(ids_all)
                filt = np.concatenate(filt_all)
            else:
                keys = np.zeros(0); ids = np.zeros(0, np.int64); filt = np.zeros(0)
            n_scanned[qi] = keys.shape[0]
            surv = filt <= tau_q
            n_surv[qi] = int(surv.sum())
            fk, fi = topk_pairs(keys, ids, k)            # unpruned definition
            pk, pi = topk_pairs(keys[surv], ids[surv], k)  # with the filter
            dropped[qi] = len(fi) - np.isin(fi, pi).sum()
            rk, ri = (pk, pi) if prune else (fk, fi)
            out_ids[qi, :len(ri)] = ri
            out_d[qi, :len(rk)] = rk
            if detail:
                details.append(dict(keys=keys, ids=ids, filt=filt, tau=tau_q))
        if self.metric == "ip":
            out_d = -out_d
        info = dict(tau=taus, scanned=n_scanned, survivors=n_surv, dropped=dropped,
                    probes=probes, G=G, E=E, Qr=Qr, details=details)
        return out_ids, out_d, info
