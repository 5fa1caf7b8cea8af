"""Pins for the oracle's search pipeline (CPU only)."""
import numpy as np
import pytest

from oracle import build, exact, search
from paper_2602_23999_amd import synth


def _tiny(n=3000, nq=40, B=1, nlist=16):
    w = synth.WORKLOADS["tiny"].scaled(n=n, nq=nq, n_centres=16)
    X, Q = synth.make_base(w), synth.make_queries(w)
    return X, Q, build.build_index(X, nlist, B)


def test_rotation_orthogonal_and_distance_preserving():
    P = build.random_rotation(128, 7).astype(np.float64)
    assert np.abs(P @ P.T - np.eye(128)).max() < 1e-6
    rng = np.random.default_rng(0)
    a, b = rng.standard_normal((2, 128))
    assert abs(np.linalg.norm(a @ P - b @ P) - np.linalg.norm(a - b)) < 1e-5
    assert np.array_equal(build.random_rotation(64, 3), build.random_rotation(64, 3))


def test_exact_knn_matches_python_loops():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((60, 5)); Q = rng.standard_normal((4, 5))
    X[7] = X[3]  # an exact tie
    for metric in ("l2", "ip"):
        ids, sc = exact.exact_knn(X, Q, 6, metric)
        for qi in range(4):
            key = [(sum((Q[qi, d] - X[i, d]) ** 2 for d in range(5)) if metric == "l2"
                    else -sum(Q[qi, d] * X[i, d] for d in range(5)), i) for i in range(60)]
            key.sort()
            assert [i for _, i in key[:6]] == ids[qi].tolist()
    assert exact.recall_at_k(np.array([[1, 2, 3], [4, 5, -1]]), np.array([[3, 2, 9], [5, 7, 8]])) == pytest.approx(0.5)


def test_kmeans_assignment_is_nearest_centroid():
    X, _, ix = _tiny()
    C = ix["centroids"]
    d = ((X[:200, None, :].astype(np.float64) - C[None]) ** 2).sum(2)
    a = np.empty(X.shape[0], np.int64)
    for c in range(ix["nlist"]):
        a[ix["ids"][ix["offsets"][c]:ix["offsets"][c + 1]]] = c
    assert np.array_equal(a[:200], d.argmin(1))
    assert ix["offsets"][-1] == X.shape[0] and sorted(ix["ids"].tolist()) == list(range(X.shape[0]))


def test_kmeans_update_step_gives_the_cluster_means():
    # Two blobs far apart: whatever the seeded initial points, one Lloyd iteration separates them (or leaves one
    # centroid without points, which then keeps its place), and the centroids are the means of their members.
    rng = np.random.default_rng(3)
    a = rng.standard_normal((300, 8)) + 50.0
    b = rng.standard_normal((200, 8)) - 50.0
    X = np.concatenate([a, b])[rng.permutation(500)]
    for seed in range(6):
        C = build.kmeans_lloyd(X, 2, 3, seed)
        assign = build.assign_clusters(X, C)
        for c in range(2):
            members = X[assign == c].astype(np.float64)
            assert len(members) in (200, 300)
            assert np.abs(C[c] - members.mean(axis=0)).max() < 1e-12
    # a centroid that attracts no point keeps its previous position
    far = np.concatenate([X, np.full((1, 8), 1e4)])
    C = build.kmeans_lloyd(far, 3, 4, 0)
    counts = np.bincount(build.assign_clusters(far, C), minlength=3)
    assert counts.sum() == 501 and np.isfinite(C).all()


def test_coarse_probe_matches_direct_loop():
    X, Q, ix = _tiny()
    Qr = search.rotate_queries(Q, ix["P"])
    for metric in ("l2", "ip"):
        p, G, E = search.coarse_probe(Qr, ix["centroids_rot"], 5, metric)
        c = ix["centroids_rot"].astype(np.float64)
        for qi in range(6):
            d2 = np.array([np.sum((Qr[qi].astype(np.float64) - c[j]) ** 2) for j in range(c.shape[0])])
            sc = d2 if metric == "l2" else -(c @ Qr[qi].astype(np.float64))
            o = np.argsort(sc, kind="stable")[:5]
            assert np.array_equal(o, p[qi])
            assert np.allclose(G[qi], sc[o], rtol=1e-9, atol=1e-9)
            assert np.allclose(E[qi], np.sqrt(d2[o]), rtol=1e-7)


def test_rotation_does_not_change_exact_neighbours():
    X, Q, ix = _tiny(n=800, nq=10)
    P = ix["P"].astype(np.float64)
    a, _ = exact.exact_knn(X, Q, 5)
    b, _ = exact.exact_knn(X.astype(np.float64) @ P, Q.astype(np.float64) @ P, 5)
    assert np.array_equal(a, b)


def test_eight_bit_full_probe_recovers_exact_knn():
    w = synth.WORKLOADS["tiny"].scaled(n=1500, nq=30, n_centres=8)
    X, Q = synth.make_base(w), synth.make_queries(w)
    ix = build.build_index(X, 8, 8)
    s = search.Searcher(ix)
    ids, d, info = s.search(Q, 10, 8, prune=False)
    gt, gd = exact.exact_knn(X, Q, 10)
    assert exact.recall_at_k(ids, gt) >= 0.97
    # estimated squared distances of the found true neighbours are close to exact ones
    rel = np.abs(d[:, 0] - gd[:, 0]) / gd[:, 0]
    assert np.median(rel) < 0.01


def test_topk_order_and_padding():
    X, Q, ix = _tiny(n=300, nq=5, nlist=8)
    s = search.Searcher(ix)
    ids, d, _ = s.search(Q, 10, 2, prune=False, detail=False)
    assert np.all(np.diff(d, axis=1)[np.isfinite(np.diff(d, axis=1))] >= 0)
    # k larger than everything scanned -> padded with -1 / +inf
    ids, d, info = s.search(Q, 128, 1, prune=False)
    for qi in range(5):
        n = info["scanned"][qi]
        assert np.all(ids[qi, n:] == -1) and np.all(np.isinf(d[qi, n:])) and np.all(ids[qi, :n] >= 0)


@pytest.mark.parametrize("B", [1, 3])
def test_pruned_equals_unpruned_when_no_winner_is_dropped(B):
    X, Q, ix = _tiny(n=4000, nq=40, B=B)
    s = search.Searcher(ix)
    a, da, ia = s.search(Q, 10, 6, prune=True)
    b, db, _ = s.search(Q, 10, 6, prune=False)
    ok = ia["dropped"] == 0
    assert ok.mean() > 0.8
    assert np.array_equal(a[ok], b[ok]) and np.array_equal(da[ok], db[ok])
    if B == 1:
        assert ok.all()            # filtering the ranking key itself never drops a winner
    assert np.all(ia["survivors"] <= ia["scanned"])
    # tau is a valid upper bound of the final k-th key
    assert np.all(db[:, -1] <= ia["tau"] * (1 + 1e-12) + 1e-12)


def test_ip_metric_search_orders_by_inner_product():
    w = synth.WORKLOADS["ip_768"].scaled(n=1200, nq=12, n_centres=8)
    X, Q = synth.make_base(w)[:, :128].copy(), synth.make_queries(w)[:, :128].copy()
    X /= np.linalg.norm(X, axis=1, keepdims=True); Q /= np.linalg.norm(Q, axis=1, keepdims=True)
    ix = build.build_index(X, 8, 8, metric="ip")
    s = search.Searcher(ix)
    ids, d, _ = s.search(Q, 10, 8, prune=False)
    gt, gs = exact.exact_knn(X, Q, 10, "ip")
    assert exact.recall_at_k(ids, gt) >= 0.95
    assert np.all(np.diff(d, axis=1) <= 0)
    assert np.abs(d[:, 0] - gs[:, 0]).max() < 0.02


def _seed_inputs(s, Q, nprobe):
    ix = s.ix
    Qr = search.rotate_queries(Q, ix["P"])
    probes, G, E = search.coarse_probe(Qr, ix["centroids_rot"], nprobe, s.metric)
    prep = []
    for qr in Qr:
        delta, qhat, S = search.quantize_query(qr)
        prep.append((delta, search.query_bitplanes(qhat), S))
    return Qr, probes, G, E, prep


@pytest.mark.parametrize("B", [3, 8])
def test_seeded_threshold_definition(B):
    # Section 3.3.4 reading: tau = K-th smallest refined estimate among the M best 1-bit candidates
    # of the nearest cluster.  Pins: M = K is the largest of the K refined seeds; M >= cluster size is
    # the K-th key of the unpruned one-cluster search; tau never grows with M; tau bounds the final
    # K-th key of the full search.
    K = 10
    X, Q, ix = _tiny(n=3000, nq=30, B=B)
    Qr, probes, G, E, prep = _seed_inputs(search.Searcher(ix), Q, 4)
    taus = {}
    for M in (K, 16, search.SEED_M, 10 ** 6):
        s = search.Searcher(ix, seed_m=M)
        taus[M] = np.array([s.seed_threshold(probes[i], G[i], E[i], Qr[i], *prep[i], K) for i in range(len(Q))])
    s = search.Searcher(ix)
    assert s.seed_m == search.SEED_M == 32
    sizes = np.diff(ix["offsets"])
    assert np.all(sizes[probes[:, 0]] >= K)          # so the seeding cluster is the nearest one
    # M = K: the largest refined estimate of the K best 1-bit candidates
    for i in range(len(Q)):
        c = int(probes[i, 0])
        a, b, _, est1, _ = s.pair(c, G[i, 0], E[i, 0], Qr[i], *prep[i])
        sel = np.lexsort((np.arange(b - a), est1))[:K]
        assert taus[K][i] == s.refined(a, b, G[i, 0], Qr[i], sel).max()
    # M >= |cluster|: K-th smallest key of the whole nearest cluster (unpruned search with nprobe = 1)
    _, d1, _ = s.search(Q, K, 1, prune=False)
    assert np.allclose(taus[10 ** 6], d1[:, K - 1], rtol=0, atol=0)
    # monotone in M and valid
    assert np.all(taus[K] >= taus[16]) and np.all(taus[16] >= taus[search.SEED_M])
    assert np.all(taus[search.SEED_M] >= taus[10 ** 6])
    assert (taus[K] > taus[search.SEED_M]).mean() > 0.3   # the wider seed set really tightens it
    _, dfull, info = s.search(Q, K, 4, prune=False)
    assert np.all(dfull[:, K - 1] <= taus[search.SEED_M])
    assert np.array_equal(info["tau"] >= dfull[:, K - 1], np.ones(len(Q), bool))


def test_seeded_threshold_one_bit_and_small_clusters():
    K = 10
    X, Q, ix = _tiny(n=3000, nq=20, B=1)
    s = search.Searcher(ix)
    Qr, probes, G, E, prep = _seed_inputs(s, Q, 3)
    for i in range(len(Q)):
        c = int(probes[i, 0])
        _, _, _, est1, _ = s.pair(c, G[i, 0], E[i, 0], Qr[i], *prep[i])
        assert s.seed_threshold(probes[i], G[i], E[i], Qr[i], *prep[i], K) == np.sort(est1)[K - 1]
    # a cluster smaller than M but not smaller than K: all of it is refined
    w = synth.WORKLOADS["tiny"].scaled(n=400, nq=10, n_centres=20)
    X, Q = synth.make_base(w), synth.make_queries(w)
    ix = build.build_index(X, 20, 4)
    s = search.Searcher(ix)
    Qr, probes, G, E, prep = _seed_inputs(s, Q, 20)
    sizes = np.diff(ix["offsets"])
    hit = 0
    for i in range(len(Q)):
        tau = s.seed_threshold(probes[i], G[i], E[i], Qr[i], *prep[i], K)
        ok = np.nonzero(sizes[probes[i]] >= K)[0]
        if len(ok) == 0:
            assert tau == search.FLT_MAX
            continue
        j = int(ok[0]); c = int(probes[i, j])
        a, b = int(ix["offsets"][c]), int(ix["offsets"][c + 1])
        if b - a <= search.SEED_M:
            hit += 1
            assert tau == np.sort(s.refined(a, b, G[i, j], Qr[i]))[K - 1]
    assert hit > 0


def test_centred_index_is_a_pure_translation():
    # a common translation leaves squared distances alone: the centred index must rank like the
    # plain one up to estimation noise, report distances of the original vectors, and its rotated
    # queries must have lost the shared offset
    w = synth.WORKLOADS["l2_128"].scaled(n=4000, nq=30, n_centres=16)
    X, Q = synth.make_base(w), synth.make_queries(w)
    plain = build.build_index(X, 16, 8)
    cent = build.build_index(X, 16, 8, center=True)
    assert not plain["mean"].any()
    assert np.allclose(cent["mean"], X.mean(0), rtol=1e-6)
    # the stored centroids are those of the translated data
    assert np.abs(cent["centroids"].mean(0)).max() < np.abs(plain["centroids"].mean(0)).max() * 0.2
    gt, gd = exact.exact_knn(X, Q, 10)
    for ix in (plain, cent):
        ids, d, _ = search.Searcher(ix).search(Q, 10, 16, prune=False)
        assert exact.recall_at_k(ids, gt) >= 0.97
        assert np.median(np.abs(d[:, 0] - gd[:, 0]) / gd[:, 0]) < 0.01   # distances to the ORIGINAL vectors
    qp = search.rotate_queries(Q, plain["P"], plain["mean"])
    qc = search.rotate_queries(Q, cent["P"], cent["mean"])
    assert np.allclose(qc, qp - (cent["mean"].astype(np.float64) @ cent["P"].astype(np.float64)), atol=2e-3)
    dp = np.mean([search.quantize_query(q)[0] for q in qp])
    dc = np.mean([search.quantize_query(q)[0] for q in qc])
    assert dc < 0.8 * dp                                                 # finer 4-bit query grid
    with pytest.raises(AssertionError):
        build.build_index(X, 16, 4, metric="ip", center=True)
