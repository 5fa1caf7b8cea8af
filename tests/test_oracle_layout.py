"""Pin for the device layout written by the oracle (CPU only)."""
import os

import numpy as np

from oracle import build


def _index(counts, D, B, rng):
    n = int(sum(counts))
    off = np.zeros(len(counts) + 1, np.int64); off[1:] = np.cumsum(counts)
    return dict(dim=D, nlist=len(counts), n=n, total_bits=B, offsets=off,
                u=rng.integers(0, 1 << B, (n, D)).astype(np.uint8),
                ids=rng.permutation(n).astype(np.int32),
                short_factors=rng.standard_normal((n, 3)).astype(np.float32),
                long_factors=rng.standard_normal((n, 2)).astype(np.float32))


def test_layout_small_fixture():
    # tests/golden/layout_small.txt is written by hand from the layout definition.
    path = os.path.join(os.path.dirname(__file__), "golden", "layout_small.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    D, B = 64, 3
    counts = [2, 0, 1]
    u = np.zeros((3, D), np.uint8)
    u[0, 0] = 7; u[0, 33] = 4; u[1, 1] = 5; u[2, 63] = 6; u[2, 15] = 3
    off = np.array([0, 2, 2, 3], np.int64)
    ix = dict(dim=D, nlist=3, n=3, total_bits=B, offsets=off, u=u, ids=np.array([10, 11, 12], np.int32),
              short_factors=np.arange(9, dtype=np.float32).reshape(3, 3),
              long_factors=np.arange(6, dtype=np.float32).reshape(3, 2))
    dev = build.pack_device_layout(ix)
    assert dev["tile_offsets"].tolist() == [0, 1, 1, 2] and dev["n_slots"] == 128
    for name, idx, val in rows:
        arr = dev[name]
        if arr.dtype == np.float32:
            assert float(arr[int(idx)]) == float(val), (name, idx)
        else:
            assert int(arr[int(idx)]) == int(val, 0), (name, idx)
    # everything not listed in the fixture is padding
    assert np.count_nonzero(dev["short_codes"]) == 4 and np.count_nonzero(dev["long_codes"]) == 5
    assert np.isinf(dev["short_factors"].reshape(2, 3, 64)[:, 0, :]).sum() == 128 - 3
    assert (dev["ids"] == -1).sum() == 125


def test_layout_roundtrip_ragged():
    rng = np.random.default_rng(0)
    D, B = 96, 5
    ix = _index([70, 0, 64, 1, 129], D, B, rng)
    dev = build.pack_device_layout(ix)
    W = D // 32
    F = build.long_field_bits(B)
    sc = dev["short_codes"].reshape(-1, W, 64).transpose(0, 2, 1).reshape(-1, W)
    sf = dev["short_factors"].reshape(-1, 3, 64).transpose(0, 2, 1).reshape(-1, 3)
    lc = dev["long_codes"].reshape(dev["n_slots"], -1)
    slot = dev["slot"]
    assert dev["tile_offsets"].tolist() == [0, 2, 2, 3, 4, 7]
    msb = build.unpack_bits(sc[slot], D)
    full = build.unpack_fields(lc[slot], F, D)
    assert F == 8 and lc.shape[1] == D * F // 32
    assert np.array_equal(msb, ix["u"] >> (B - 1))
    assert np.array_equal(full, ix["u"])                      # the long code holds the whole code
    assert np.array_equal(sf[slot], ix["short_factors"])
    assert np.array_equal(dev["long_factors"].reshape(-1, 2)[slot], ix["long_factors"])
    assert np.array_equal(dev["ids"][slot], ix["ids"])
    pad = np.setdiff1d(np.arange(dev["n_slots"]), slot)
    assert not sc[pad].any() and not lc[pad].any() and np.all(dev["ids"][pad] == -1)
    assert np.all(np.isinf(sf[pad, 0])) and not sf[pad, 1:].any()
