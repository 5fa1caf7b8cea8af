"""End-to-end parity over the corners of the supported shapes: every code width the kernels are instantiated
for, the smallest and largest code sizes, k and nprobe on both sides of the 64-lane selection limit."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import build, exact, search
from paper_2602_23999_amd import synth

from gpu_helpers import check_against_own_run, search_explained, upload

pytestmark = pytest.mark.gpu

#        D    B  n     nlist k    nprobe nq
SHAPES = [
    (32,   8, 2500, 20,   1,   1,    33),
    (64,   7, 2500, 70,   64,  64,   30),
    (256,  2, 3000, 72,   65,  65,   21),
    (512,  1, 3000, 16,   128, 16,   10),
    (1024, 2, 2000, 8,    10,  8,    7),
    (768,  3, 2000, 9,    5,   3,    9),
    (128,  6, 4000, 130,  17,  128,  13),
]


@pytest.mark.parametrize("impl", [0, 1, 4])
@pytest.mark.parametrize("D,B,n,nlist,k,nprobe,nq", SHAPES)
def test_shape_end_to_end(D, B, n, nlist, k, nprobe, nq, impl):
    w = replace(synth.WORKLOADS["tiny"], dim=D, n=n, nq=nq, n_centres=max(4, nlist // 2))
    X, Q = synth.make_base(w), synth.make_queries(w)
    ix = build.build_index(X, nlist, B, kmeans_iters=3)
    s = search.Searcher(ix)
    gi = upload(ix)
    gi.set_option("scan_impl", impl)
    gi.set_option("split_min_pairs", 1)
    ids, dist, why = search_explained(gi, s, Q, k, nprobe)   # every difference from the oracle accounted for
    own = s.search(Q, k, nprobe, detail=True)
    o_ids = own[0]
    # padding (fewer than k survivors) must agree exactly
    assert np.array_equal(ids < 0, o_ids < 0)
    check_against_own_run(s, own, ids, dist, k, why)
    gt, _ = exact.exact_knn(X, Q, k)
    assert abs(exact.recall_at_k(ids, gt) - exact.recall_at_k(o_ids, gt)) <= 0.03
    gi.close()
