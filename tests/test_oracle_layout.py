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


def test_whole_code_fields_and_ex_bit_planes_hold_the_same_code():
    # Section 3.4.3 stores only the B-1 ex-bits in the long code; the library stores the whole code in F-bit
    # fields.  Both decode to the same u, so the choice is one of format (bytes read per refined vector), not of
    # arithmetic.  Bytes per vector of the two formats, at the dimensions of the configurations that use them:
    rng = np.random.default_rng(3)
    want_bytes = {(3, 96): (48, 24 + 12), (4, 128): (64, 48 + 16), (5, 960): (960, 480 + 120), (8, 768): (768, 672 + 96)}
    for (B, D), (field_bytes, ex_bytes) in want_bytes.items():
        u = rng.integers(0, 1 << B, (37, D)).astype(np.uint8)
        F = build.long_field_bits(B)
        fields = build.pack_fields(u, F)
        sw = build.pack_bits(u >> (B - 1))
        ex = build.pack_ex_planes(u, B)
        assert np.array_equal(build.unpack_fields(fields, F, D), u)
        assert np.array_equal(build.unpack_ex_planes(sw, ex, B, D), u)
        assert fields.shape[1] * 4 == field_bytes                   # what a refined vector reads today
        assert (ex.shape[1] + sw.shape[1]) * 4 == ex_bytes          # ex-bit planes plus the sign words they need


def test_unpack_device_layout_inverts_pack():
    rng = np.random.default_rng(1)
    for B, D in ((1, 64), (5, 96)):
        ix = _index([70, 0, 64, 1, 129], D, B, rng)
        ix.update(metric="l2", P=rng.standard_normal((D, D)).astype(np.float32),
                  centroids_rot=rng.standard_normal((5, D)).astype(np.float32))
        if B == 1:
            ix["long_factors"] = ix["short_factors"][:, :2].copy()
        dev = build.pack_device_layout(ix)
        arr = dict(dim=D, nlist=5, n=ix["n"], total_bits=B, metric="l2", rotation=ix["P"].reshape(-1),
                   centroids=ix["centroids_rot"].reshape(-1), offsets=ix["offsets"], short_codes=dev["short_codes"],
                   short_factors=dev["short_factors"], long_codes=dev["long_codes"], long_factors=dev["long_factors"],
                   ids=dev["ids"], mean=None)
        back = build.unpack_device_layout(arr)
        for key in ("u", "ids", "short_factors", "long_factors", "offsets", "P", "centroids_rot"):
            assert np.array_equal(back[key], ix[key]), key
