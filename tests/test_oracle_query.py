"""Pins for query quantisation and the bit-plane inner product (CPU only)."""
import os

import numpy as np

from oracle import build, search

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_bitplane_identity_exhaustive_single_dim():
    # Section 3.4.1(2): x_b[i]*qhat[i] == sum_j w_j x_b[i] qhat^(j)[i] for every 4-bit value.
    for qv in range(-8, 8):
        for xb in (0, 1):
            for pos in (0, 13, 31):
                qhat = np.zeros(32, np.int8); qhat[pos] = qv
                bits = np.zeros((1, 32), np.uint8); bits[0, pos] = xb
                got = search.ip_bitplane(build.pack_bits(bits), search.query_bitplanes(qhat))
                assert got[0] == xb * qv


def test_bitplane_identity_random():
    rng = np.random.default_rng(0)
    for D in (32, 96, 128, 960):
        qhat = rng.integers(-7, 8, D).astype(np.int8)
        bits = rng.integers(0, 2, (200, D)).astype(np.uint8)
        got = search.ip_bitplane(build.pack_bits(bits), search.query_bitplanes(qhat))
        want = bits.astype(np.int64) @ qhat.astype(np.int64)
        assert np.array_equal(got, want)


def test_planes_reassemble_and_storage_size():
    rng = np.random.default_rng(1)
    qhat = rng.integers(-7, 8, 1024).astype(np.int8)
    planes = search.query_bitplanes(qhat)
    bits = np.stack([build.unpack_bits(planes[j][None], 1024)[0] for j in range(4)]).astype(np.int64)
    assert np.array_equal(-8 * bits[3] + 4 * bits[2] + 2 * bits[1] + bits[0], qhat)
    with open(os.path.join(GOLD, "paper_sizes.txt")) as f:
        rows = {l.split()[0]: l.split()[1:] for l in f if l.strip() and not l.startswith("#")}
    D, Bq, nbytes = map(int, rows["query_repr_bytes"])
    assert D == 1024 and Bq == search.BQ and planes.nbytes == nbytes


def test_quantisation_bounds():
    rng = np.random.default_rng(2)
    for scale in (1e-3, 1.0, 300.0):
        q = (rng.standard_normal(128) * scale).astype(np.float32)
        delta, qhat, S = search.quantize_query(q)
        assert np.abs(qhat).max() == 7 and S == int(qhat.sum())
        assert np.all(np.abs(delta * qhat.astype(np.float64) - q) <= delta * 0.5 * (1 + 1e-5))
    delta, qhat, S = search.quantize_query(np.zeros(64, np.float32))
    assert delta == 1.0 and not qhat.any() and S == 0
    # round half to even at exact halves: q'/delta = 0.5, 1.5, 2.5 with max = 7
    q = np.array([7.0, 0.5, 1.5, 2.5, -0.5, -1.5] + [0.0] * 26, np.float32)
    _, qhat, _ = search.quantize_query(q)
    assert qhat[:6].tolist() == [7, 0, 2, 2, 0, -2]
