"""Batches of at most 64 queries take fused kernels with fewer launches (option "small_batch"): their results must
be those of the general kernels, bit for bit, which the other tests compare with the oracle stage by stage."""
import numpy as np
import pytest
import torch

from test_gpu_parity import case

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("impl", [0, 1, 4])
@pytest.mark.parametrize("name,nq", [("tiny_b1", 1), ("tiny_b1", 64), ("l2_128_b4", 7), ("l2_128_b4", 64),
                                     ("l2_96_b3_k100", 33), ("l2_960_b5", 24), ("ragged_b2", 40), ("many_probes_b2", 48),
                                     ("ip_768_b8", 24), ("centred_b4", 2)])
def test_small_batch_kernels_equal_the_general_ones(name, nq, impl):
    c = case(name)
    gi, k, nprobe = c["gi"], c["k"], c["nprobe"]
    q = torch.from_numpy(c["Q"][:nq]).cuda().contiguous()
    gi.set_option("scan_impl", impl)
    gi.set_option("split_min_pairs", 1)
    try:
        for prune in (1, 0):
            gi.set_option("prune", prune)
            gi.set_option("small_batch", 0)
            want_ids, want_d = gi.search(q, k, nprobe)
            gi.set_option("small_batch", 1)
            ids, d = gi.search(q, k, nprobe)
            torch.cuda.synchronize()
            assert torch.equal(ids, want_ids), (name, nq, prune)
            assert torch.equal(d, want_d), (name, nq, prune)
    finally:
        gi.set_option("prune", 1)
        gi.set_option("small_batch", 1)
        gi.set_option("scan_impl", 0)
