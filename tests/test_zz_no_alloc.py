"""rabitq_search_noalloc (the entry point for callers that cannot allocate device memory) against
rabitq_search, through the C ABI: two calls in a row, the second with a smaller input, so that what
the first call left in the static scratch must not leak into the second."""
import numpy as np
import pytest
import torch

from oracle import build
from paper_2602_23999_amd import rabitq, synth

from gpu_helpers import upload

pytestmark = pytest.mark.gpu


def _index(B, n=20_000, nlist=40, nq=300):
    w = synth.WORKLOADS["l2_128"].scaled(n=n, nq=nq, n_centres=64)
    X, Q = synth.make_base(w), synth.make_queries(w)
    ix = build.build_index(X, nlist, B, kmeans_iters=3)
    return upload(ix), torch.from_numpy(Q).cuda()


@pytest.mark.parametrize("B", [4, 1])
def test_noalloc_matches_search_twice(B):
    gi, Q = _index(B)
    # (nq, k, nprobe): the second call is smaller in every size
    for nq, k, nprobe in ((300, 10, 8), (37, 5, 3)):
        q = Q[:nq].contiguous()
        want_ids, want_d = gi.search(q, k, nprobe)
        torch.cuda.synchronize()
        ids = torch.full((nq, k), -7, dtype=torch.int64, device="cuda")
        d = torch.full((nq, k), float("nan"), dtype=torch.float32, device="cuda")
        free_before = torch.cuda.mem_get_info()[0]
        gi.search_noalloc(q, k, nprobe, ids, d)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before      # the device's free memory did not move
        # the same kernels on the same inputs: integer ids and fp32 distances are identical
        assert torch.equal(ids, want_ids)
        assert torch.equal(d, want_d)
    gi.close()


def test_noalloc_rejects_what_does_not_fit():
    gi, Q = _index(4, n=6000, nlist=16, nq=8)
    lib = rabitq.load_library()
    ids = torch.empty((8, 10), dtype=torch.int64, device="cuda")
    d = torch.empty((8, 10), dtype=torch.float32, device="cuda")
    # 10^6 queries x 16 probes x 128 candidate slots cannot fit 64 MiB: rejected on the host, before any
    # pointer is used (the buffers passed here are far too small for that batch)
    rc = lib.rabitq_search_noalloc(gi._h, Q.data_ptr(), 1_000_000, 10, 16, ids.data_ptr(), d.data_ptr(), None)
    assert rc == -1 and b"bytes of workspace" in lib.rabitq_last_error()
    for k, nprobe in ((0, 4), (129, 4), (10, 0), (10, 17)):
        with pytest.raises(rabitq.RabitqError):
            gi.search_noalloc(Q, k, nprobe, ids, d)
    # still usable afterwards
    want_ids, want_d = gi.search(Q, 10, 4)
    gi.search_noalloc(Q, 10, 4, ids, d)
    torch.cuda.synchronize()
    assert torch.equal(ids, want_ids) and torch.equal(d, want_d)
    gi.close()
