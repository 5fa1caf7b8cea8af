"""rabitq_search recorded into a HIP graph: steady-state calls allocate nothing, synchronise nothing and
clear their counters with kernels, so a caller may capture one search and replay it.  Every replay is
checked against the eager result, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2602_23999_amd import synth

from test_gpu_parity import case

pytestmark = pytest.mark.gpu


def tiled(Q: np.ndarray, nq: int) -> np.ndarray:
    """nq queries: the case's own, repeated as often as needed (batches of 256 queries and more use the handle's
    second stream, batches of 2048 and more also clear their scratch on it ahead of time)."""
    reps = -(-nq // len(Q))
    return np.tile(Q, (reps, 1))[:nq].copy()


@pytest.mark.parametrize("name,nq", [("l2_128_b4", 1), ("l2_128_b4", 96), ("tiny_b1", 100), ("l2_96_b3_k100", 16),
                                     ("l2_128_b4", 300), ("tiny_b1", 2500), ("l2_96_b3_k100", 2100)])
def test_captured_search_replays_like_eager(name, nq):
    c = case(name)
    gi, k, nprobe = c["gi"], c["k"], c["nprobe"]
    Q = torch.from_numpy(tiled(c["Q"], nq)).cuda()
    q_in = Q.clone()
    ids = torch.empty((nq, k), dtype=torch.int64, device="cuda")
    dist = torch.empty((nq, k), dtype=torch.float32, device="cuda")
    gi.search(q_in, k, nprobe, ids, dist)              # warm-up: the workspace grows here, outside the capture
    torch.cuda.synchronize()
    e_ids, e_d = ids.clone(), dist.clone()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        gi.search(q_in, k, nprobe, ids, dist)
    rng = np.random.default_rng(0)
    for rep in range(4):
        # new queries in the captured input buffer: a permutation of the batch, so the answers are known
        perm = torch.from_numpy(rng.permutation(nq)).cuda()
        q_in.copy_(Q[perm])
        ids.fill_(-7); dist.fill_(-1.0)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(ids, e_ids[perm]) and torch.equal(dist, e_d[perm]), rep
        # eager work between the replays: an eager search of other queries through the same handle
        o_ids, o_d = gi.search(Q.flip(0).contiguous(), k, nprobe)
        torch.cuda.synchronize()
        assert torch.equal(o_ids, e_ids.flip(0)) and torch.equal(o_d, e_d.flip(0))


@pytest.mark.parametrize("name", ["l2_128_b4", "l2_96_b3_k100", "ragged_b2"])
def test_second_stream_does_not_change_results(name):
    # "overlap": list building and scan set-up on the handle's second stream beside the seeding
    c = case(name)
    gi, k, nprobe = c["gi"], c["k"], c["nprobe"]
    base = len(c["Q"])
    Q = torch.from_numpy(tiled(c["Q"], 2048 + base)).cuda()   # large enough for the second stream and the early clears
    out = {}
    for mode in (1, 0, 1):
        gi.set_option("overlap", mode)
        for rep in range(3):                       # back-to-back calls reuse the workspace and the events
            ids, d = gi.search(Q, k, nprobe)
        torch.cuda.synchronize()
        out.setdefault(mode, []).append((ids.clone(), d.clone()))
    gi.set_option("overlap", 1)
    ref = out[0][0]
    for ids, d in out[1]:
        assert torch.equal(ids, ref[0]) and torch.equal(d, ref[1])
    # the repeated queries give the answers of the small batch (which stays on one stream)
    s_ids, s_d = gi.search(Q[:base].contiguous(), k, nprobe)
    for r0 in range(0, Q.shape[0] - base + 1, base):
        assert torch.equal(ref[0][r0:r0 + base], s_ids) and torch.equal(ref[1][r0:r0 + base], s_d)
    # per-stage timings are still reported for every stage
    gi.set_option("profile", 2)
    gi.search(Q, k, nprobe); gi.search(Q, k, nprobe)
    ms, calls = gi.stage_ms()
    gi.set_option("profile", 0)
    assert calls == 2 and len(ms) == 10 and all(v > 0 for name, v in ms.items() if name != "scan_estimate")


@pytest.mark.parametrize("name,limit", [("l2_128_b4", 7), ("l2_128_b4", 64), ("l2_96_b3_k100", 33), ("ragged_b2", 1)])
def test_sub_batches_do_not_change_results(name, limit):
    # "max_batch": a large batch goes through the pipeline in consecutive sub-batches of one workspace
    c = case(name)
    gi, k, nprobe = c["gi"], c["k"], c["nprobe"]
    Q = torch.from_numpy(c["Q"]).cuda()
    ref_ids, ref_d = gi.search(Q, k, nprobe)
    torch.cuda.synchronize()
    gi.set_option("max_batch", limit)
    try:
        for rep in range(2):
            ids, d = gi.search(Q, k, nprobe)
            torch.cuda.synchronize()
            assert torch.equal(ids, ref_ids) and torch.equal(d, ref_d)
    finally:
        gi.set_option("max_batch", 0)
    ids, d = gi.search(Q, k, nprobe)
    assert torch.equal(ids, ref_ids) and torch.equal(d, ref_d)
