"""Pins for the factor formulas and the estimator (CPU only).

The paper defers the estimator's expressions to an external document, so they
are pinned to what the mathematics fixes: exactness when the code direction
equals the data direction, zero-mean error over random rotations, the
1/sqrt(D) error scale, and the tail mass outside the eps0 bound."""
import numpy as np
import pytest

from oracle import build, search


def _est_one(o_raw, c, q, P, B, metric="l2", eps0=1.9):
    """1-bit and full-code estimates of dist(q, o_raw) with float q' (no query quantisation)."""
    P = P.astype(np.float64)
    res = o_raw - c
    r = np.linalg.norm(res)
    o_rot = (res / r) @ P
    u = build.encode_unit(o_rot[None], B)
    c_rot = (c @ P)[None]
    q_rot = q @ P
    odc = np.array([c @ res])
    out = []
    for x in ((u >> (B - 1)).astype(np.float64) - 0.5, u.astype(np.float64) - ((1 << B) - 1) / 2):
        f = build.vector_factors(x, o_rot[None], c_rot, np.array([r]), metric, eps0, odc)[0]
        if metric == "l2":
            G = np.sum((q_rot - c_rot[0]) ** 2)
        else:
            G = -(q_rot @ c_rot[0])
        E = np.linalg.norm(q_rot - c_rot[0])
        est = G + f[0] + f[1] * (x[0] @ q_rot)
        out.append((est, f[2] * E))
    return out


def test_exact_when_data_direction_is_a_grid_direction():
    rng = np.random.default_rng(0)
    D = 64
    for B in (1, 3, 5):
        P = build.random_rotation(D, 11)
        u = rng.integers(0, 1 << B, D)
        x = u - ((1 << B) - 1) / 2
        c = rng.standard_normal(D)
        o_raw = c + 2.5 * (x / np.linalg.norm(x)) @ P.astype(np.float64).T  # o' is exactly x/||x||
        q = rng.standard_normal(D) * 3
        (e1, _), (eB, errB) = _est_one(o_raw, c, q, P, B)
        assert abs(eB - np.sum((q - o_raw) ** 2)) < 1e-5   # fp32-stored P is orthogonal to ~1e-7
        assert errB < 5e-3          # sqrt(1-a^2) with a = 1 - O(1e-8)
        (_, _), (ipB, _) = _est_one(o_raw, c, q, P, B, metric="ip")
        assert abs(-ipB - q @ o_raw) < 1e-5


@pytest.mark.parametrize("metric", ["l2", "ip"])
def test_unbiased_over_rotations_and_error_scale(metric):
    rng = np.random.default_rng(1)
    T = 600
    for D in (64, 256):
        c = rng.standard_normal(D)
        o_raw = c + rng.standard_normal(D)
        q = c + 1.5 * rng.standard_normal(D)
        truth = np.sum((q - o_raw) ** 2) if metric == "l2" else -(q @ o_raw)
        err1, bound1, errB = [], [], []
        for t in range(T):
            P = build.random_rotation(D, 1000 + t)
            (e1, b1), (eB, _) = _est_one(o_raw, c, q, P, 4, metric)
            err1.append(e1 - truth); bound1.append(b1); errB.append(eB - truth)
        err1, bound1, errB = map(np.array, (err1, bound1, errB))
        # zero mean within 3.5 standard errors
        assert abs(err1.mean()) < 3.5 * err1.std() / np.sqrt(T)
        assert abs(errB.mean()) < 3.5 * errB.std() / np.sqrt(T)
        # predicted std: (bound/eps0) * ||z_perp||/||z||, z = q - c, o = unit(o_raw-c)
        z = q - c; o = (o_raw - c) / np.linalg.norm(o_raw - c)
        frac = np.linalg.norm(z - (z @ o) * o) / np.linalg.norm(z)
        pred = (bound1 / 1.9).mean() * frac
        assert 0.85 < err1.std() / pred < 1.15
        # two-sided tail outside the eps0 = 1.9 bound is a few percent (normal tail 5.7 %)
        assert 0.01 < np.mean(np.abs(err1) > bound1) < 0.10
        # 4-bit code is far more accurate than the 1-bit code
        assert errB.std() < 0.25 * err1.std()


def test_error_scales_as_inverse_sqrt_dim():
    rng = np.random.default_rng(2)
    stds = {}
    for D in (64, 1024):
        errs = []
        for t in range(300):
            c = np.zeros(D)
            o_raw = rng.standard_normal(D); o_raw /= np.linalg.norm(o_raw)
            q = rng.standard_normal(D); q /= np.linalg.norm(q)
            P = build.random_rotation(D, 5000 + t) if D == 64 else np.eye(D, dtype=np.float32)
            # for D=1024 a random o_raw with identity P is already a uniformly random direction
            (e1, _), _ = _est_one(o_raw, c, q, P, 1)
            errs.append(e1 - np.sum((q - o_raw) ** 2))
        stds[D] = np.std(errs)
    assert 3.2 < stds[64] / stds[1024] < 5.0   # sqrt(1024/64) = 4


def test_degenerate_vector_equal_to_centroid():
    X = np.zeros((70, 32), np.float32)
    X[:35] = 1.0
    X[35:] = -1.0
    ix = build.build_index(X, 2, 4, centroids=np.stack([X[0], X[40]]).astype(np.float64))
    assert np.all(ix["short_factors"] == 0) and np.all(ix["long_factors"] == 0)
    assert np.all(ix["u"] == 8)
    s = search.Searcher(ix)
    q = np.full((1, 32), 0.5, np.float32)
    ids, d, _ = s.search(q, 3, 2)
    assert np.allclose(d[0], 32 * 0.25, atol=1e-4) and ids[0].tolist() == [0, 1, 2]


def test_bound_covers_the_query_rounding_error():
    """The 1-bit estimate from the 4-bit query has two independent errors: the code's and the query's rounding.
    In a regime where the two are of the same size (a query far from the origin but close to the centroid), the
    error's spread matches the combined prediction, search.bound_radius reproduces it from the expected alignment
    of 1-bit codes, and the lower bound built on it fails as often as a 1.9-sigma bound should, which the bound on
    ||q'-c'|| alone does not."""
    rng = np.random.default_rng(5)
    D, T, eps0 = 256, 800, 1.9
    c = 2.5 * rng.standard_normal(D)
    o_raw = c + rng.standard_normal(D)
    q = c + 0.5 * rng.standard_normal(D)
    true = np.sum((q - o_raw) ** 2)
    z_exact, z_radius, over_new, over_old, ratio = [], [], 0, 0, []
    for t in range(T):
        P = build.random_rotation(D, 1000 + t).astype(np.float64)
        res = o_raw - c
        r = np.linalg.norm(res)
        o_rot = (res / r) @ P
        xb = (o_rot >= 0).astype(np.float64)[None] - 0.5
        c_rot, q_rot = (c @ P)[None], (q @ P).astype(np.float32)
        f = build.vector_factors(xb, o_rot[None], c_rot, np.array([r]), "l2", eps0)[0]
        delta, qhat, S = search.quantize_query(q_rot)
        I = int(((xb[0] + 0.5) * qhat).sum())
        G = np.sum((q_rot.astype(np.float64) - c_rot[0]) ** 2)
        E = np.sqrt(G)
        est1, lb = search.estimate_1bit(G, search.bound_radius(E, delta, D), f[None].astype(np.float32), delta,
                                        np.array([I]), S)
        err = est1[0] - true
        s_code = f[2] * E / eps0
        s_query = abs(f[1]) * float(delta) * np.sqrt(D / 48.0)
        ratio.append(s_query / s_code)
        z_exact.append(err / np.hypot(s_code, s_query))
        z_radius.append(err / (f[2] * search.bound_radius(E, delta, D) / eps0))
        over_new += lb[0] > true
        over_old += est1[0] - f[2] * E > true
    assert 0.7 < np.median(ratio) < 1.5                      # the regime: both errors matter
    assert abs(np.std(z_exact) - 1.0) < 0.12 and abs(np.mean(z_exact)) < 0.12
    assert abs(np.std(z_radius) - 1.0) < 0.12               # the expected alignment stands in for the code's own
    tail = 0.0287                                            # 1 - Phi(1.9)
    assert abs(over_new / T - tail) < 3.5 * np.sqrt(tail / T)
    assert over_old / T > tail + 5 * np.sqrt(tail / T)       # the bound on the code's error alone is not one


def test_bound_radius_is_negligible_where_the_query_grid_is_fine():
    # benchmark-like sizes: delta ~ 10, ||q'-c'|| ~ 250, D = 128
    assert search.bound_radius(250.0, 10.0, 128) / 250.0 < 1.03
    assert search.bound_radius(0.0, 0.0, 128) == 0.0
