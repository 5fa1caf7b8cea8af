"""Checks of a built index (arrays in the layout of rabitq_index_desc) against the oracle's
exact encoder and factor formulas, for the device builder's tests."""
import numpy as np

from oracle import build


def check_built_index(out: dict, X: np.ndarray, B: int, metric: str = "l2", eps0: float = 1.9,
                      mean_gap: float = 2e-3, max_gap: float = 2e-2):
    n, D = X.shape
    W = D // 32
    nlist = out["nlist"]
    off = out["offsets"]
    counts = np.diff(off)
    assert off[0] == 0 and off[-1] == n and np.all(counts >= 0)
    n_tiles = int(((counts + 63) // 64).sum())
    ids = out["ids"]
    real = ids >= 0
    assert real.sum() == n and sorted(ids[real].tolist()) == list(range(n))
    # padding slots
    sf_all = out["short_factors"].reshape(n_tiles, 3, 64).transpose(0, 2, 1).reshape(-1, 3)
    sc_all = out["short_codes"].reshape(n_tiles, W, 64).transpose(0, 2, 1).reshape(-1, W)
    assert np.all(np.isinf(sf_all[~real, 0])) and not sf_all[~real, 1:].any() and not sc_all[~real].any()
    # real slots follow the cluster order given by offsets
    tiles = (counts + 63) // 64
    tile_off = np.concatenate([[0], np.cumsum(tiles)])
    slot = np.repeat(tile_off[:-1] * 64, counts) + (np.arange(n) - np.repeat(off[:-1], counts))
    assert np.array_equal(np.nonzero(real)[0], slot)
    msb = build.unpack_bits(sc_all[real], D)
    if B > 1:
        F = build.long_field_bits(B)
        u = build.unpack_fields(out["long_codes"].reshape(n_tiles * 64, -1)[real], F, D)
        assert np.array_equal(u >> (B - 1), msb) and u.max() < (1 << B)
    else:
        u = msb
    P = out["rotation"].astype(np.float64)
    assert np.abs(P @ P.T - np.eye(D)).max() < 1e-5
    C_rot = out["centroids"].astype(np.float64)
    cid = np.repeat(np.arange(nlist), counts)
    rows = ids[real]
    Xr = X[rows].astype(np.float64) @ P
    # every list holds its vectors in ascending id order (the grouping is stable) ...
    for c in range(nlist):
        assert np.all(np.diff(rows[off[c]:off[c + 1]]) > 0), c
    # ... and every vector sits in the list of its nearest centroid (scores are fp32 on the device: a near-tie may
    # fall either way)
    d2 = (Xr * Xr).sum(1)[:, None] + (C_rot * C_rot).sum(1)[None, :] - 2.0 * Xr @ C_rot.T
    best = d2.min(axis=1)
    assert np.all(d2[np.arange(n), cid] <= best + 1e-5 * (np.abs(best) + (Xr * Xr).sum(1))), "assignment"
    res = Xr - C_rot[cid]
    r = np.linalg.norm(res, axis=1)
    o_rot = res / np.maximum(r, 1e-300)[:, None]
    # a vector that (almost) coincides with its centroid has no meaningful direction
    good = r > 1e-3 * np.median(r)
    assert good.mean() > 0.99
    cos_builder = build.code_cosine(u, o_rot, B)
    cos_exact = build.code_cosine(build.encode_unit(o_rot, B), o_rot, B)
    gap = (cos_exact - cos_builder)[good]
    assert np.all(gap >= -1e-5), gap.min()
    assert np.mean(gap) < mean_gap and np.max(gap) < max_gap, (np.mean(gap), np.max(gap))
    odc = np.einsum("ij,ij->i", C_rot[cid], res)
    f1 = build.vector_factors(msb.astype(np.float64) - 0.5, o_rot, C_rot[cid], r, metric, eps0, odc)
    sf = sf_all[real]
    assert np.allclose(sf[good], f1[good], rtol=2e-3, atol=2e-3 * np.abs(f1[good]).max())
    if B > 1:
        lf = out["long_factors"].reshape(-1, 2)[real]
        fB = build.vector_factors(u.astype(np.float64) - ((1 << B) - 1) / 2, o_rot, C_rot[cid], r, metric, eps0, odc)
        assert np.allclose(lf[good], fB[good, :2], rtol=2e-3, atol=2e-3 * np.abs(fB[good, :2]).max())
    # assignment is the nearest centroid (fp32 near-ties aside)
    m = min(300, n)
    d = ((Xr[:m, None, :] - C_rot[None]) ** 2).sum(2)
    assert (d.argmin(1) == cid[:m]).mean() > 0.99
    return dict(mean_gap=float(np.mean(gap)), max_gap=float(np.max(gap)))
