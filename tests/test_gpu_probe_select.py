"""Cluster selection (Section 3.3.2) against the oracle for every top-nprobe kernel the library has, at the list
counts the large configurations run: more than 1024 lists with nprobe <= 64 (the streaming kernel's tail loop),
and nprobe > 64 with nlist in (512, 1024], (1024, 2048] and above 2048.  The stage depends on the centroids only,
so the indices hold few vectors; centroids are given, not learnt."""
import numpy as np
import pytest
import torch

from oracle import build, search
from paper_2602_23999_amd import rabitq

from gpu_helpers import upload

pytestmark = pytest.mark.gpu

#        nlist nprobe variant metric
CASES = [
    (1100, 32, 0, "l2"),      # tail loop of the streaming kernel: one partial block of 512 scores after the first 1024
    (4100, 64, 0, "l2"),      # several full blocks and a ragged last one
    (16384, 48, 0, "ip"),     # the list count of the 10M configuration
    (8192, 64, 0, "l2"),      # the list count of the 5M configuration
    (500, 100, 1, "l2"),      # row in registers, 8 scores per lane
    (1000, 100, 2, "l2"),     # 16 per lane
    (1024, 1024, 2, "l2"),    # every list probed
    (1100, 128, 3, "l2"),     # 32 per lane
    (2048, 300, 3, "ip"),
    (2100, 100, 4, "l2"),     # workgroup-wide radix select
    (4100, 300, 4, "l2"),
    (16384, 512, 4, "l2"),    # the largest sweep point of the 10M configuration
]


@pytest.mark.parametrize("nlist,nprobe,variant,metric", CASES)
def test_probe_selection_kernels(nlist, nprobe, variant, metric):
    lib = rabitq.load_library()
    assert lib.rabitq_probe_select_variant(nlist, nprobe) == variant   # the kernel this case is meant to reach
    D, n, nq = 64, 1500, 40
    rng = np.random.default_rng(nlist * 7 + nprobe)
    C = rng.standard_normal((nlist, D))
    if metric == "ip":
        C /= np.linalg.norm(C, axis=1, keepdims=True)
    X = (C[rng.integers(0, nlist, n)] + 0.2 * rng.standard_normal((n, D))).astype(np.float32)
    Q = (C[rng.integers(0, nlist, nq)] + 0.3 * rng.standard_normal((nq, D))).astype(np.float32)
    if nlist >= 4100:   # exact duplicates among the centroids: ties must go to the lower list id
        C[nlist - 5] = C[3]
        C[nlist // 2] = C[7]
    ix = build.build_index(X, nlist, 1, metric=metric, centroids=C)
    gi = upload(ix)
    Qr = search.rotate_queries(Q, ix["P"])
    want_ids, want_G, want_E = search.coarse_probe(Qr, ix["centroids_rot"], nprobe, metric)
    q_rot = torch.from_numpy(Qr).cuda()
    sq = torch.from_numpy((Qr.astype(np.float64) ** 2).sum(1).astype(np.float32)).cuda()
    out = gi.coarse_probe(q_rot, sq, nprobe)
    ids, G, E = (out[k].cpu().numpy() for k in ("probe_ids", "probe_G", "probe_E"))
    scale = (Qr.astype(np.float64) ** 2).sum(1)[:, None] + 1.0
    assert np.all(np.abs(G - want_G) <= 2e-6 * scale)           # cancellation in s_q + s_c - 2<q,c>
    assert np.all(np.diff(G, axis=1) >= 0)                       # best first
    assert np.all(np.abs(E ** 2 - want_E ** 2) <= 4e-6 * scale)
    assert all(len(set(r.tolist())) == nprobe for r in ids) and ids.min() >= 0 and ids.max() < nlist
    # a probe that differs from the oracle's must tie with it in score: the GPU's choice, scored by the oracle
    diff = ids != want_ids
    if diff.any():
        c64 = ix["centroids_rot"].astype(np.float64)
        dot = Qr.astype(np.float64) @ c64.T
        sc = -dot if metric == "ip" else (Qr.astype(np.float64) ** 2).sum(1)[:, None] + (c64 ** 2).sum(1)[None, :] - 2 * dot
        qi, ri = np.nonzero(diff)
        assert np.all(np.abs(sc[qi, ids[qi, ri]] - want_G[qi, ri]) <= 4e-6 * scale[qi, 0])
    assert diff.mean() < 0.01
    # equal scores: the lower list id comes first (duplicated centroids above)
    eq = G[:, 1:] == G[:, :-1]
    assert np.all(ids[:, 1:][eq] > ids[:, :-1][eq])
    gi.close()


def test_every_selection_kernel_has_a_case():
    lib = rabitq.load_library()
    assert {lib.rabitq_probe_select_variant(nlist, nprobe) for nlist, nprobe, _, _ in CASES} == {0, 1, 2, 3, 4}
