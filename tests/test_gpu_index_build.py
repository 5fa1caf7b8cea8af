"""rabitq_index_build (HIP: k-means, assignment, two-phase grid-search quantiser, factors,
layout) against the oracle's exact encoder and factor formulas, and end to end."""
import numpy as np
import pytest
import torch

from oracle import build, exact, search
from paper_2602_23999_amd import rabitq, synth

from gpu_helpers import upload
from index_checks import check_built_index

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("wl,n,nlist,B,metric", [
    ("l2_128", 20_000, 40, 4, "l2"), ("l2_96", 9_000, 24, 3, "l2"), ("tiny", 5_000, 16, 1, "l2"),
    ("tiny", 3_000, 12, 8, "l2"), ("l2_960", 3_000, 8, 5, "l2"), ("ip_768", 3_000, 8, 6, "ip"),
    ("tiny", 700, 40, 2, "l2"),   # ragged: lists smaller than a tile, some possibly empty
])
def test_device_builder_against_oracle_formulas(wl, n, nlist, B, metric):
    w = synth.WORKLOADS[wl].scaled(n=n, n_centres=max(8, nlist // 2))
    X = synth.make_base(w)
    P = build.random_rotation(w.dim, 7)
    gi = rabitq.Index.build(torch.from_numpy(X).cuda(), nlist, B, P, metric=metric, kmeans_iters=4, train_size=n // 2)
    out = gi.export()
    assert np.array_equal(out["rotation"], P)
    stats = check_built_index(out, X, B, metric=metric)
    # building twice gives the same bytes (no order-dependent atomics)
    gi2 = rabitq.Index.build(torch.from_numpy(X).cuda(), nlist, B, P, metric=metric, kmeans_iters=4, train_size=n // 2)
    out2 = gi2.export()
    for k in ("offsets", "short_codes", "short_factors", "ids", "long_codes", "long_factors", "centroids"):
        if out[k] is not None:
            assert np.array_equal(out[k], out2[k], equal_nan=True), k
    gi.close(); gi2.close()


def test_centred_device_build():
    # center = 1: the builder works on the vectors minus their mean and the search subtracts it from
    # the queries; every check of the plain build must hold for the translated vectors
    w = synth.WORKLOADS["l2_128"].scaled(n=20_000, nq=100, n_centres=32)
    X, Q = synth.make_base(w), synth.make_queries(w)
    P = build.random_rotation(w.dim, 7)
    gi = rabitq.Index.build(torch.from_numpy(X).cuda(), 40, 4, P, kmeans_iters=4, train_size=10_000, center=True)
    out = gi.export()
    mean = X.mean(0, dtype=np.float64)
    assert np.allclose(out["mean"], mean, rtol=1e-6, atol=1e-6)
    check_built_index(out, (X.astype(np.float64) - out["mean"].astype(np.float64)).astype(np.float32), 4)
    # rotated queries are (q - mean) P
    qr = gi.rotate(torch.from_numpy(Q).cuda()).cpu().numpy()
    want = search.rotate_queries(Q, P, out["mean"])
    assert np.max(np.abs(qr - want)) < 2e-6 * np.abs(Q).sum(1).max()
    # distances refer to the original vectors; recall is that of an oracle-built centred index
    ids, d = gi.search(torch.from_numpy(Q).cuda(), 10, 8)
    gt, gd = exact.exact_knn(X, Q, 10)
    ix = build.build_index(X, 40, 4, kmeans_iters=4, center=True)
    o_ids, _, _ = search.Searcher(ix).search(Q, 10, 8)
    assert exact.recall_at_k(ids.cpu().numpy(), gt) > exact.recall_at_k(o_ids, gt) - 0.03
    assert np.median(np.abs(d.cpu().numpy()[:, 0] - gd[:, 0]) / gd[:, 0]) < 0.1
    # export -> upload round trip keeps the translation
    gj = rabitq.Index(**out)
    ids2, d2 = gj.search(torch.from_numpy(Q).cuda(), 10, 8)
    # (the upload recomputes the centroid norms on the host; the coarse term is a difference of large squares)
    atol = 2e-6 * float(((Q - out["mean"]).astype(np.float64) ** 2).sum(1).max())
    assert torch.equal(ids, ids2) and torch.allclose(d, d2, rtol=1e-5, atol=atol)
    # save -> load (plain .npz) answers identically too
    import os, tempfile
    with tempfile.TemporaryDirectory() as tmp:
        gi.save(os.path.join(tmp, "ix.npz"))
        gk = rabitq.Index.load(os.path.join(tmp, "ix.npz"))
    ids3, d3 = gk.search(torch.from_numpy(Q).cuda(), 10, 8)
    assert torch.equal(ids, ids3) and torch.allclose(d, d3, rtol=1e-5, atol=atol)
    gk.close()
    # an inner-product index cannot be centred
    with pytest.raises(rabitq.RabitqError):
        rabitq.Index.build(torch.from_numpy(X).cuda(), 40, 4, P, metric="ip", center=True)
    gi.close(); gj.close()


def test_device_built_index_searches_like_an_oracle_built_one():
    w = synth.WORKLOADS["l2_128"].scaled(n=40_000, nq=200, n_centres=64)
    X, Q = synth.make_base(w), synth.make_queries(w)
    P = build.random_rotation(w.dim, 7)
    gi = rabitq.Index.build(torch.from_numpy(X).cuda(), 48, 4, P, kmeans_iters=6)
    ids, _ = gi.search(torch.from_numpy(Q).cuda(), 10, 8)
    gt, _ = exact.exact_knn(X, Q, 10)
    r_dev = exact.recall_at_k(ids.cpu().numpy(), gt)
    ix = build.build_index(X, 48, 4, kmeans_iters=6)
    o_ids, _, _ = search.Searcher(ix).search(Q, 10, 8)
    r_ora = exact.recall_at_k(o_ids, gt)
    assert r_dev > r_ora - 0.03, (r_dev, r_ora)
    # the exported index, uploaded again, answers identically
    out = gi.export()
    gj = rabitq.Index(**out)
    ids2, _ = gj.search(torch.from_numpy(Q).cuda(), 10, 8)
    assert torch.equal(ids, ids2)
    gi.close(); gj.close()
