"""Pins for the lookup-table inner product of Section 3.4.1(1) (CPU only)."""
import os

import numpy as np
import pytest

from oracle import build, search
from paper_2602_23999_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")
H = 2.0 ** -11  # binary16 unit roundoff


def test_table_entries_are_block_dot_products():
    # L_j(b) = <q'^(j), b> for every block and every 4-bit pattern, within binary16 rounding
    rng = np.random.default_rng(3)
    for D, scale in ((32, 1.0), (96, 40.0), (960, 1e-2)):
        q = (rng.standard_normal(D) * scale).astype(np.float32)
        t = search.lut_tables(q)
        assert t.shape == (D // 4, 16) and t.dtype == np.float16
        for j in range(D // 4):
            for b in range(16):
                pattern = np.array([(b >> i) & 1 for i in range(4)], np.float64)
                want = float(pattern @ q[4 * j:4 * j + 4].astype(np.float64))
                assert abs(float(t[j, b]) - want) <= H * abs(want) * 1.01 + 1e-6 * scale + 6e-8
        assert not t[:, 0].any()


def test_table_footprint_matches_the_papers_example():
    with open(os.path.join(GOLD, "paper_sizes.txt")) as f:
        rows = {l.split()[0]: l.split()[1:] for l in f if l.strip() and not l.startswith("#")}
    D, U, entry, nbytes = map(int, rows["lut_bytes"])
    t = search.lut_tables(np.ones(D, np.float32))
    assert U == search.LUT_U and t.itemsize == entry and t.nbytes == nbytes


def test_lookup_sum_is_exact_on_representable_queries():
    # small-integer queries: every table entry and every partial sum is exact, so the result must
    # equal the integer dot product (catches a wrong block, nibble or bit order)
    rng = np.random.default_rng(4)
    for D in (32, 96, 128, 960):
        q = rng.integers(-8, 9, D).astype(np.float32)
        bits = rng.integers(0, 2, (300, D)).astype(np.uint8)
        got = search.ip_lut(build.pack_bits(bits), search.lut_tables(q))
        assert got.dtype == np.float32
        assert np.array_equal(got.astype(np.int64), bits.astype(np.int64) @ q.astype(np.int64))
    # one set bit: the lookup returns the single query coordinate
    q = np.arange(1, 65, dtype=np.float32)
    for pos in (0, 3, 4, 31, 32, 63):
        bits = np.zeros((1, 64), np.uint8); bits[0, pos] = 1
        assert search.ip_lut(build.pack_bits(bits), search.lut_tables(q))[0] == q[pos]


def test_lookup_sum_within_rounding_bound_of_fp64():
    rng = np.random.default_rng(5)
    for D in (128, 768):
        q = (rng.standard_normal(D) * 30).astype(np.float32)
        bits = rng.integers(0, 2, (500, D)).astype(np.uint8)
        t = search.lut_tables(q)
        got = search.ip_lut(build.pack_bits(bits), t).astype(np.float64)
        want = bits.astype(np.float64) @ q.astype(np.float64)
        m = D // 4
        bound = m * H * float(np.abs(t.astype(np.float64)).max()) + m * 2.0 ** -23 * np.abs(q).sum()
        assert np.abs(got - want).max() <= bound
        # and the error is really of binary16 size, not zero (the tables are stored in binary16)
        assert np.abs(got - want).max() > 1e-4


def _tiny(B):
    w = synth.WORKLOADS["tiny"].scaled(n=3000, nq=25, n_centres=8)
    X, Q = synth.make_base(w), synth.make_queries(w)
    return X, Q, build.build_index(X, 8, B)


@pytest.mark.parametrize("B", [1, 4])
def test_lut_and_bitwise_estimates_agree_within_query_quantisation(B):
    # both approximate <x_bar, q'>: the bitwise one with a 4-bit query (error <= delta/2 per
    # dimension, times |x_bar| = 1/2), the table one with binary16 entries
    X, Q, ix = _tiny(B)
    sb, sl = search.Searcher(ix), search.Searcher(ix, ip_method="lut")
    Qr = search.rotate_queries(Q, ix["P"])
    probes, G, E = search.coarse_probe(Qr, ix["centroids_rot"], 3, "l2")
    D = Qr.shape[1]
    for qi in range(5):
        delta, qhat, S = search.quantize_query(Qr[qi])
        planes = search.query_bitplanes(qhat)
        for j in range(3):
            c = int(probes[qi, j])
            s, e, _, est_b, lb_b = sb.pair(c, G[qi, j], E[qi, j], Qr[qi], delta, planes, S)
            _, _, ip, est_l, lb_l = sl.pair(c, G[qi, j], E[qi, j], Qr[qi], delta, planes, S)
            f = ix["short_factors"][s:e].astype(np.float64)
            t = search.lut_tables(Qr[qi]).astype(np.float64)
            bound = np.abs(f[:, 1]) * (D * float(delta) / 4.0 + (D // 4) * H * np.abs(t).max() + 1e-3)
            assert np.all(np.abs(est_l - est_b) <= bound)
            # the table estimate is the closer one to the exact <x_bar, q'> on average
            xbar = build.unpack_bits(sb.words[s:e], D).astype(np.float64) - 0.5
            exact = G[qi, j] + f[:, 0] + f[:, 1] * (xbar @ Qr[qi].astype(np.float64))
            assert np.abs(est_l - exact).mean() <= np.abs(est_b - exact).mean() + 1e-9
            assert np.allclose(est_l - lb_l, f[:, 2] * E[qi, j])


def test_lut_search_full_probe_eight_bits_recovers_exact_knn():
    from oracle import exact
    w = synth.WORKLOADS["tiny"].scaled(n=1500, nq=30, n_centres=8)
    X, Q = synth.make_base(w), synth.make_queries(w)
    ix = build.build_index(X, 8, 8)
    ids, d, info = search.Searcher(ix, ip_method="lut").search(Q, 10, 8)
    gt, _ = exact.exact_knn(X, Q, 10)
    assert exact.recall_at_k(ids, gt) >= 0.97
    assert np.all(info["survivors"] <= info["scanned"])
