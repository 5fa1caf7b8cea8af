"""Few pairs per list (at most four on average): the popcount kernel runs in its one-pair-per-work-item form, with a
descriptor per work item, lists handed out longest first and the next tiles requested ahead.  Its results are compared
with the oracle through the stage-level scan (oracle pair lists and threshold injected), for whole lists and for lists
cut into segments, and the search must not depend on the hand-out order or on the small-batch kernels."""
import numpy as np
import pytest
import torch

from paper_2602_23999_amd import rabitq

from gpu_helpers import compare_topk, key_scale, oracle_stages, to_dev
from test_gpu_parity import CASES, case

pytestmark = pytest.mark.gpu

# (case, queries): queries * nprobe <= 4 * nlist, above and below the 64 queries of the small-batch kernels
SHAPES = [("tiny_b1", 32), ("l2_128_b4", 30), ("l2_96_b3_k100", 20), ("ragged_b2", 4), ("ip_768_b8", 10),
          ("many_probes_b2", 6), ("centred_b4", 21)]


def sub_case(name, nq):
    c = case(name)
    key = ("stream", nq)
    if key not in c:
        st = oracle_stages(c["s"], c["Q"][:nq], c["k"], c["nprobe"])
        c[key] = dict(st=st, dev=to_dev(st))
    return c, c[key]


@pytest.mark.parametrize("seg_tiles", [0, 1])
@pytest.mark.parametrize("longest_first", [1, 0])
@pytest.mark.parametrize("prune", [True, False])
@pytest.mark.parametrize("name,nq", SHAPES)
def test_streaming_scan_against_oracle(name, nq, prune, longest_first, seg_tiles):
    c, sub = sub_case(name, nq)
    gi, s, k, nprobe = c["gi"], c["s"], c["k"], c["nprobe"]
    nlist = CASES[name][4]
    assert nq * nprobe <= 4 * nlist
    st, d = sub["st"], sub["dev"]
    scale = key_scale(st["G"], st["E"], s.metric)
    tau_np = np.minimum(st["tau"], rabitq.FLT_MAX)
    tau_np = (tau_np + 1e-5 * (np.abs(tau_np) + scale)).astype(np.float32)
    tau_np[st["tau"] >= rabitq.FLT_MAX] = rabitq.FLT_MAX
    if not prune:
        tau_np[:] = rabitq.FLT_MAX
    gi.set_option("scan_impl", 0)
    gi.set_option("longest_first", longest_first)
    gi.set_option("scan_segment_tiles", seg_tiles)
    try:
        keys, cnt, _ = gi.scan(d["prep"], d["probes"], d["pair_off"], d["pair_ids"], torch.from_numpy(tau_np).cuda(), k)
        assert gi.index_info("last_scan_stream") == 1 and gi.index_info("last_scan_split") == 0
        ids, dist = gi.merge(keys, cnt, nq, k, nprobe)
    finally:
        gi.set_option("longest_first", 1)
        gi.set_option("scan_segment_tiles", 0)
    o_ids, o_d, _ = s.search(c["Q"][:nq], k, nprobe, prune=prune, Qr=st["Qr"], tau=tau_np.astype(np.float64))
    n_exact = compare_topk(ids.cpu().numpy(), dist.cpu().numpy().astype(np.float64), o_ids, o_d, 1e-4 * scale)
    assert n_exact >= 0.9 * nq
    assert int(cnt.max()) <= keys.shape[1]


@pytest.mark.parametrize("name,nq", SHAPES)
def test_streaming_raw_inner_products_bit_exact(name, nq):
    """The integer <x_b, qhat> of every (pair, vector) as the one-pair form computes it (debug output of the scan)."""
    from oracle import search as osearch
    c, sub = sub_case(name, nq)
    gi, s, k, nprobe = c["gi"], c["s"], c["k"], c["nprobe"]
    st, d = sub["st"], sub["dev"]
    ix = s.ix
    sizes = np.diff(ix["offsets"]).astype(np.int64)
    tiles = (sizes + 63) // 64
    # slots of every pair's cluster, in pair-list order
    flat = st["probes"].reshape(-1)
    cl = flat[st["pair_ids"]]
    dbg_off = np.zeros(len(cl) + 1, np.int64)
    dbg_off[1:] = np.cumsum(tiles[cl] * 64)
    tau = torch.full((nq,), rabitq.FLT_MAX, dtype=torch.float32, device="cuda")
    gi.set_option("scan_impl", 0)
    _, _, ip = gi.scan(d["prep"], d["probes"], d["pair_off"], d["pair_ids"], tau, k,
                       dbg_off=torch.from_numpy(dbg_off).cuda())
    assert gi.index_info("last_scan_stream") == 1
    ip = ip.cpu().numpy()
    rng = np.random.Generator(np.random.PCG64(5))
    for pos in rng.choice(len(cl), size=min(100, len(cl)), replace=False):
        p = int(st["pair_ids"][pos])
        q, c_id = p // nprobe, int(cl[pos])
        a, b = int(ix["offsets"][c_id]), int(ix["offsets"][c_id + 1])
        want = osearch.ip_bitplane(s.words[a:b], st["planes"][q])
        got = ip[dbg_off[pos]:dbg_off[pos] + (b - a)]
        assert np.array_equal(got, want), (name, pos, p, c_id)


@pytest.mark.parametrize("name,nq", SHAPES)
def test_search_independent_of_hand_out_order_and_small_batch(name, nq):
    c = case(name)
    gi, k, nprobe = c["gi"], c["k"], c["nprobe"]
    q = torch.from_numpy(c["Q"][:nq]).cuda().contiguous()
    gi.set_option("scan_impl", 0)
    try:
        ref = None
        for small in (0, 1):
            for lf in (1, 0):
                gi.set_option("small_batch", small)
                gi.set_option("longest_first", lf)
                ids, d = gi.search(q, k, nprobe)
                torch.cuda.synchronize()
                assert gi.index_info("last_scan_stream") == 1
                if ref is None:
                    ref = (ids.clone(), d.clone())
                assert torch.equal(ids, ref[0]) and torch.equal(d, ref[1]), (name, small, lf)
    finally:
        gi.set_option("small_batch", 1)
        gi.set_option("longest_first", 1)


@pytest.mark.parametrize("name,nq", [("l2_128_b4", 30), ("tiny_b1", 32)])
def test_call_that_may_not_allocate_falls_back_to_the_general_kernel(name, nq):
    """A handle that has not yet made the descriptors' memory (no allocating call of this shape so far) searches a
    streaming-shaped batch with the general kernel when asked through rabitq_search_noalloc; the allocating entry
    point then takes the one-pair form.  Same results, bit for bit."""
    from gpu_helpers import upload
    c = case(name)
    gi = upload(c["ix"])
    k, nprobe = c["k"], c["nprobe"]
    q = torch.from_numpy(c["Q"][:nq]).cuda().contiguous()
    ids = torch.full((nq, k), -7, dtype=torch.int64, device="cuda")
    d = torch.full((nq, k), float("nan"), dtype=torch.float32, device="cuda")
    try:
        gi.set_option("scan_impl", 0)
        gi.search_noalloc(q, k, nprobe, ids, d)
        torch.cuda.synchronize()
        assert gi.index_info("last_scan_stream") == 0
        want_ids, want_d = gi.search(q, k, nprobe)
        torch.cuda.synchronize()
        assert gi.index_info("last_scan_stream") == 1
        assert torch.equal(ids, want_ids) and torch.equal(d, want_d)
        gi.search_noalloc(q, k, nprobe, ids, d)   # now the memory is there
        torch.cuda.synchronize()
        assert gi.index_info("last_scan_stream") == 1
        assert torch.equal(ids, want_ids) and torch.equal(d, want_d)
    finally:
        gi.close()
