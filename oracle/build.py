"""Oracle index construction (TEST INFRASTRUCTURE ONLY; see package header).

Everything is float64 numpy unless a stored array is fp32 by format.  Each
function cites the passage of the paper it restates.

Conventions
-----------
* Row vectors; the rotated form of ``x`` is ``x' = x @ P`` with ``P`` orthogonal
  (Section 2.2, Eq. (2): the codebook is rotated by a random orthogonal matrix;
  the paper writes column vectors and ``o' = P^-1 o``, which is the same map for
  ``P -> P^T``).
* ``B`` = total bits per dimension, code ``u in {0..2^B-1}^D``, grid point
  ``x = u - c_B`` with ``c_B = (2^B-1)/2`` (Eq. (1)).
* 1-bit code ``u_b`` = most significant bit of ``u``; ex-code = remaining bits
  (Section 3.1, paragraph on the index build).

Parity status
-------------
random_rotation      pinned: orthogonality, norm / distance preservation.
kmeans_lloyd         pinned: assignment = brute-force nearest centroid; update step =
                     the members' mean to 1e-12 on separated blobs; an empty cluster
                     keeps its centroid.
encode_unit          pinned: brute force over the whole grid for tiny D, B;
                     B = 1 closed form (sign bits, cosine = ||o'||_1/sqrt(D)).
vector_factors       pinned: exactness when o' is itself a grid direction;
                     zero-mean error over random rotations; 1/sqrt(D) error
                     scale (tests/test_oracle_estimator.py).
pack_device_layout   pinned: hand-written fixture tests/golden/layout_small.txt
                     and unpack(pack(x)) == x; unpack_device_layout is its inverse.
pack_ex_planes       pinned: decodes, with the short code, to the same u as the
                     whole-code fields (the long code of Section 3.4.3 vs the stored one).
"""
from __future__ import annotations

import numpy as np

TILE = 64  # vectors per tile of the device layout


# --------------------------------------------------------------------------
# Rotation (Section 2.2, Eq. (2); Section 3.2.1)
# --------------------------------------------------------------------------
def random_rotation(D: int, seed: int) -> np.ndarray:
    """Haar-distributed orthogonal ``P`` [D, D]: QR of a Gaussian matrix with the
    sign of R's diagonal folded into Q (which makes the factorisation unique).
    Returned as the fp32 matrix that is stored in the index."""
    rng = np.random.Generator(np.random.PCG64(seed))
    g = rng.standard_normal((D, D))
    q, r = np.linalg.qr(g)
    q = q * np.sign(np.diag(r))[None, :]
    return q.astype(np.float32)


# --------------------------------------------------------------------------
# IVF clustering (Section 2.1; Section 3.2.1)
# --------------------------------------------------------------------------
def _sqdist_argmin(X: np.ndarray, C: np.ndarray, chunk: int = 8192) -> np.ndarray:
    """Index of the nearest row of C for every row of X (squared L2, ties to the
    lower index), computed in float64 in chunks."""
    cn = np.einsum("ij,ij->i", C, C)
    out = np.empty(X.shape[0], dtype=np.int64)
    for s in range(0, X.shape[0], chunk):
        x = X[s:s + chunk].astype(np.float64)
        d = cn[None, :] - 2.0 * (x @ C.T)  # ||x||^2 is constant per row
        out[s:s + chunk] = np.argmin(d, axis=1)
    return out


def kmeans_lloyd(X: np.ndarray, nlist: int, iters: int, seed: int,
                 train_size: int | None = None) -> np.ndarray:
    """Plain Lloyd k-means: ``nlist`` centroids [nlist, D] float64.

    Initial centroids are distinct training points chosen with the seed; an
    empty cluster keeps its previous centroid.  The paper uses a balanced
    k-means whose algorithm it does not give and trains on one tenth of the
    data (Section 4.2.3); ``train_size`` selects the seeded training subset."""
    rng = np.random.Generator(np.random.PCG64(seed))
    n = X.shape[0]
    if train_size is not None and train_size < n:
        tr = X[np.sort(rng.choice(n, size=train_size, replace=False))]
    else:
        tr = X
    tr = np.asarray(tr, dtype=np.float64)
    C = tr[np.sort(rng.choice(tr.shape[0], size=nlist, replace=False))].copy()
    for _ in range(iters):
        a = _sqdist_argmin(tr, C)
        cnt = np.bincount(a, minlength=nlist)
        sums = np.zeros_like(C)
        np.add.at(sums, a, tr)
        nz = cnt > 0
        C[nz] = sums[nz] / cnt[nz, None]
    return C


def assign_clusters(X: np.ndarray, C: np.ndarray) -> np.ndarray:
    """Nearest centroid of each vector (Section 3.2.1)."""
    return _sqdist_argmin(X, C)


# --------------------------------------------------------------------------
# Exact RaBitQ B-bit code of a rotated unit vector (Section 2.2, Eq. (3))
# --------------------------------------------------------------------------
def encode_unit(o_rot: np.ndarray, B: int, chunk: int | None = None) -> np.ndarray:
    """Codes ``u`` [n, D] uint8 maximising ``<u - c_B, o'> / ||u - c_B||``.

    Follows the critical-rescaling-factor enumeration the paper recalls in
    Section 2.2: with ``y_i = |o'_i|`` the grid point closest to ``t*o'`` has
    magnitudes ``m_i + 1/2``, ``m_i = min(floor(t*y_i), 2^(B-1)-1)``; it changes
    only at the critical ``t = k/y_i`` (k = 1..2^(B-1)-1).  Sweeping them in
    ascending order, the numerator grows by ``y_i`` and the squared norm by
    ``(k+1/2)^2 - (k-1/2)^2 = 2k`` per event; the best prefix (first maximum,
    the start state included) gives the code.  ``o'_i >= 0`` takes the upper
    half of the grid, so for B = 1 the code is the sign bit."""
    o_rot = np.asarray(o_rot, dtype=np.float64)
    n, D = o_rot.shape
    half = 1 << (B - 1)
    L = half - 1
    m = np.zeros((n, D), dtype=np.int64)
    if L > 0:
        if chunk is None:
            chunk = max(16, int(4_000_000 // (D * L)))  # bounds the [chunk, D*L] work arrays
        k = np.arange(1, L + 1, dtype=np.float64)
        dden = np.tile(2.0 * k, D)  # event e = i*L + (k-1)
        for s in range(0, n, chunk):
            y = np.abs(o_rot[s:s + chunk])
            nn = y.shape[0]
            with np.errstate(divide="ignore"):
                t = (k[None, None, :] / y[:, :, None]).reshape(nn, D * L)
            order = np.argsort(t, axis=1, kind="stable")
            t_sorted = np.take_along_axis(t, order, axis=1)
            dnum = np.repeat(y, L, axis=1)
            num0 = 0.5 * y.sum(axis=1)
            num = num0[:, None] + np.cumsum(np.take_along_axis(dnum, order, axis=1), axis=1)
            den2 = D / 4.0 + np.cumsum(dden[order], axis=1)
            obj = num / np.sqrt(den2)
            obj[~np.isfinite(t_sorted)] = -np.inf  # a zero coordinate never moves
            obj = np.concatenate([(num0 / np.sqrt(D / 4.0))[:, None], obj], axis=1)
            best = np.argmax(obj, axis=1)  # number of events applied
            rank = np.empty_like(order)
            np.put_along_axis(rank, order, np.arange(D * L)[None, :].repeat(nn, 0), axis=1)
            m[s:s + chunk] = (rank < best[:, None]).reshape(nn, D, L).sum(axis=2)
    u = np.where(o_rot >= 0.0, half + m, half - 1 - m)
    return u.astype(np.uint8)


def code_cosine(u: np.ndarray, o_rot: np.ndarray, B: int) -> np.ndarray:
    """``<x, o'> / ||x||`` for ``x = u - c_B`` (the objective of Eq. (3))."""
    x = u.astype(np.float64) - ((1 << B) - 1) / 2.0
    return np.einsum("ij,ij->i", x, o_rot) / np.linalg.norm(x, axis=1)


# --------------------------------------------------------------------------
# Per-vector factors (the last paragraph of Section 2.2 says that the estimate
# needs the code's inner product with q' and a few stored factors, without
# giving them; Section 3.4.3 splits them into short and long factors.  The
# formulas below are derived from Eq. (1)-(3).)
# --------------------------------------------------------------------------
def vector_factors(x: np.ndarray, o_rot: np.ndarray, c_rot: np.ndarray,
                   r: np.ndarray, metric: str, eps0: float,
                   o_dot_c: np.ndarray | None = None) -> np.ndarray:
    """Factors [n, 3] float64 = (f_add, f_rescale, f_err) for grid points ``x``.

    For a unit vector ``o`` with code direction ``x``, any ``z`` satisfies
    ``<o, z> ~= <x, z'> / <x, o'>`` (the code's component orthogonal to ``o'`` is
    uniformly oriented under the random rotation, so the error has zero mean and
    standard deviation ``||z_perp|| * sqrt(1-a^2) / (a*sqrt(D-1))`` with
    ``a = <x, o'>/||x||``).  With ``z = q - c``:

    L2:  ``||q - o_r||^2 = ||q-c||^2 + r^2 - 2r<o, q-c>``
         est = G + f_add + f_rescale * <x, q'>,   G = ||q' - c'||^2
         f_add = r^2 + 2r<x,c'>/<x,o'>,  f_rescale = -2r/<x,o'>
         f_err = 2r * eps0 * sqrt(1-a^2) / (a*sqrt(D-1));  bound: est - f_err*||q'-c'||
    IP:  key = -<q, o_r>,  ``<q,o_r> = <q,c> + <c, o_r-c> + r<o, q-c>``
         G = -<q',c'>,  f_add = -<c, o_r-c> + r<x,c'>/<x,o'>,  f_rescale = -r/<x,o'>
         f_err = r * eps0 * sqrt(1-a^2) / (a*sqrt(D-1))   (``o_dot_c`` = <c, o_r-c>)

    ``r == 0`` (vector equals its centroid): all factors 0, so est = G exactly."""
    n, D = x.shape
    xo = np.einsum("ij,ij->i", x, o_rot)
    xc = np.einsum("ij,ij->i", x, c_rot)
    xn = np.linalg.norm(x, axis=1)
    ok = r > 0.0
    xo_s = np.where(ok, xo, 1.0)
    a = np.clip(xo_s / xn, 0.0, 1.0)
    a_s = np.where(ok, a, 1.0)
    # a code at right angles to (or pointing away from) its vector carries no information about it: the error
    # scale is unbounded there, stated as +inf rather than obtained from a division by zero
    pos = a_s > 0.0
    spread = np.full(n, np.inf)
    spread[pos] = np.sqrt(np.maximum(1.0 - a_s[pos] * a_s[pos], 0.0)) / (a_s[pos] * np.sqrt(D - 1.0))
    f = np.zeros((n, 3), dtype=np.float64)
    if metric == "l2":
        f[:, 0] = r * r + 2.0 * r * xc / xo_s
        f[:, 1] = -2.0 * r / xo_s
        f[:, 2] = 2.0 * r * eps0 * spread
    elif metric == "ip":
        f[:, 0] = -o_dot_c + r * xc / xo_s
        f[:, 1] = -r / xo_s
        f[:, 2] = r * eps0 * spread
    else:
        raise ValueError(metric)
    f[~ok] = 0.0  # o_r == c: every term vanishes (for IP, <c, o_r - c> = 0 too)
    return f


# --------------------------------------------------------------------------
# Whole index (Section 3.1 on the index build, Section 3.4.3 layout)
# --------------------------------------------------------------------------
def build_index(X: np.ndarray, nlist: int, total_bits: int, metric: str = "l2",
                seed_rotation: int = 7, seed_kmeans: int = 99, kmeans_iters: int = 10,
                train_size: int | None = None, eps0: float = 1.9,
                centroids: np.ndarray | None = None, workers: int = 1, center: bool = False) -> dict:
    """Build the flat IVF-RaBitQ index over raw vectors ``X`` [N, D].

    ``center`` (L2 only): the mean of the data (fp64 column mean, stored as fp32) is
    subtracted from every vector before anything else and the search subtracts it from
    every query; squared distances are unchanged by a common translation, while the
    rotated query, which Section 3.4.1(2) quantises to 4 bits, loses the offset all
    vectors share and with it most of its quantisation error.

    Steps in the paper's order (Section 3.1): learn centroids and assign; per
    cluster normalise with respect to the centroid, rotate by P, quantise; split
    each code into the 1-bit code and the ex-code; compute factors; store all
    arrays flattened in cluster order with one CSR offset array (Section 3.4.3).

    Returns a dict of canonical (unpadded, cluster-ordered) arrays:
      P [D,D] f32, centroids_rot [nlist,D] f32, offsets [nlist+1] i64,
      ids [N] i32 (original row of each stored vector), u [N,D] u8 (full codes),
      short_factors [N,3] f32, long_factors [N,2] f32, r [N] f64, and scalars.
    """
    X = np.asarray(X)
    N, D = X.shape
    assert D % 32 == 0 and 1 <= total_bits <= 8
    mean = np.zeros(D, dtype=np.float32)
    if center:
        assert metric == "l2", "a translation changes inner products"
        mean = X.mean(axis=0, dtype=np.float64).astype(np.float32)
        X = (X.astype(np.float64) - mean.astype(np.float64)).astype(np.float32)
    B = total_bits
    P = random_rotation(D, seed_rotation)
    P64 = P.astype(np.float64)
    if centroids is None:
        C = kmeans_lloyd(X, nlist, kmeans_iters, seed_kmeans, train_size)
    else:
        C = np.asarray(centroids, dtype=np.float64)
    assign = assign_clusters(X, C)
    order = np.argsort(assign, kind="stable")  # cluster order, ascending id inside
    counts = np.bincount(assign, minlength=nlist)
    offsets = np.zeros(nlist + 1, dtype=np.int64)
    np.cumsum(counts, out=offsets[1:])
    C_rot = (C @ P64).astype(np.float32)  # stored rotated centroids c'
    C_rot64 = C_rot.astype(np.float64)

    u = np.empty((N, D), dtype=np.uint8)
    sf = np.empty((N, 3), dtype=np.float32)
    lf = np.zeros((N, 2), dtype=np.float32)
    rr = np.empty(N, dtype=np.float64)
    cB = ((1 << B) - 1) / 2.0
    chunk = 16384

    def do_chunk(s):
        rows = order[s:s + chunk]
        cid = assign[rows]
        c = C[cid]
        res = X[rows].astype(np.float64) - c
        r = np.linalg.norm(res, axis=1)
        ok = r > 0.0
        o = np.where(ok[:, None], res / np.where(ok, r, 1.0)[:, None], 0.0)
        o_rot = o @ P64
        uu = encode_unit(o_rot, B)
        uu[~ok] = 1 << (B - 1)  # degenerate: MSB set, ex-code 0 (factors are 0)
        c_rot = C_rot64[cid]
        o_dot_c = np.einsum("ij,ij->i", c, res)
        xb = (uu >> (B - 1)).astype(np.float64) - 0.5
        f1 = vector_factors(xb, o_rot, c_rot, r, metric, eps0, o_dot_c)
        sf[s:s + chunk] = f1.astype(np.float32)
        if B > 1:
            xf = uu.astype(np.float64) - cB
            fB = vector_factors(xf, o_rot, c_rot, r, metric, eps0, o_dot_c)
            lf[s:s + chunk] = fB[:, :2].astype(np.float32)
        else:
            lf[s:s + chunk] = f1[:, :2].astype(np.float32)
        u[s:s + chunk] = uu
        rr[s:s + chunk] = r

    starts = range(0, N, chunk)
    if workers > 1:
        # chunks are independent and numpy releases the GIL in its heavy loops; threads only
        # spread the same arithmetic over the host cores
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(do_chunk, starts))
    else:
        for s in starts:
            do_chunk(s)
    return dict(dim=D, nlist=nlist, n=N, total_bits=B, metric=metric, eps0=eps0, mean=mean,
                P=P, centroids=C, centroids_rot=C_rot, offsets=offsets,
                ids=order.astype(np.int32), u=u, short_factors=sf, long_factors=lf, r=rr)


# --------------------------------------------------------------------------
# Bit packing and the device layout (Section 3.4.3)
# --------------------------------------------------------------------------
def pack_bits(bits: np.ndarray) -> np.ndarray:
    """[n, D] 0/1 -> [n, D/32] uint32; bit i (LSB = 0) of word w is dim 32w+i."""
    n, D = bits.shape
    b = bits.astype(np.uint32).reshape(n, D // 32, 32)
    sh = np.arange(32, dtype=np.uint32)
    return (b << sh[None, None, :]).sum(axis=2, dtype=np.uint64).astype(np.uint32)


def unpack_bits(words: np.ndarray, D: int) -> np.ndarray:
    n = words.shape[0]
    sh = np.arange(32, dtype=np.uint32)
    return ((words[:, :, None] >> sh[None, None, :]) & 1).reshape(n, D).astype(np.uint8)


def long_field_bits(total_bits: int) -> int:
    """Width F of one long-code field: B rounded up to 2, 4 or 8 (the field holds the
    whole code, sign bit included, so refinement reads one array)."""
    for f in (2, 4, 8):
        if total_bits <= f:
            return f
    raise ValueError(total_bits)


def pack_fields(vals: np.ndarray, F: int) -> np.ndarray:
    """[n, D] small ints -> [n, D*F/32] uint32; dim i sits in word i // (32/F) at
    bit offset F * (i mod (32/F)), little-endian."""
    n, D = vals.shape
    per = 32 // F
    v = vals.astype(np.uint64).reshape(n, D // per, per)
    sh = (np.arange(per, dtype=np.uint64) * np.uint64(F))
    return (v << sh[None, None, :]).sum(axis=2, dtype=np.uint64).astype(np.uint32)


def unpack_fields(words: np.ndarray, F: int, D: int) -> np.ndarray:
    n = words.shape[0]
    per = 32 // F
    sh = (np.arange(per, dtype=np.uint32) * np.uint32(F))
    mask = np.uint32((1 << F) - 1)
    return ((words[:, :, None] >> sh[None, None, :]) & mask).reshape(n, D).astype(np.uint8)


def short_words(index: dict) -> np.ndarray:
    """1-bit codes of all vectors as packed words [N, W]."""
    B = index["total_bits"]
    return pack_bits(index["u"] >> (B - 1))


def pack_device_layout(index: dict) -> dict:
    """The byte-exact arrays the search library uploads.

    The paper stores, per cluster, the packed words of all vectors for one
    32-dimension group contiguously (Section 3.4.3, interleaved layout).  The
    interleave granularity used here is a tile of 64 vectors (one wavefront):

      cluster c owns ceil(n_c/64) tiles; tile_offsets[c] is its first tile.
      short_codes   u32 [n_tiles][W][64]   word w of lane l of tile t at (t*W+w)*64+l
      short_factors f32 [n_tiles][3][64]   (f_add, f_rescale, f_err) planes
      long_codes    u32 [n_slots][D*F/32]  the full B-bit code per dim in F-bit fields
                                           (F = B rounded up to 2,4,8; absent if B=1)
      long_factors  f32 [n_slots][2]       (f_add, f_rescale) of the full code
      ids           i32 [n_slots]
    Padding slots: codes 0, f_add = +inf, other factors 0, id = -1."""
    D, B, nlist = index["dim"], index["total_bits"], index["nlist"]
    W = D // 32
    off = index["offsets"]
    counts = np.diff(off)
    tiles = (counts + TILE - 1) // TILE
    tile_off = np.zeros(nlist + 1, dtype=np.int64)
    np.cumsum(tiles, out=tile_off[1:])
    n_tiles = int(tile_off[-1])
    n_slots = n_tiles * TILE
    # slot of each stored vector
    within = np.arange(index["n"], dtype=np.int64) - np.repeat(off[:-1], counts)
    slot = np.repeat(tile_off[:-1] * TILE, counts) + within
    sw = short_words(index)
    sc = np.zeros((n_slots, W), dtype=np.uint32)
    sc[slot] = sw
    short_codes = sc.reshape(n_tiles, TILE, W).transpose(0, 2, 1).copy()
    sf = np.zeros((n_slots, 3), dtype=np.float32)
    sf[:, 0] = np.inf
    sf[slot] = index["short_factors"]
    short_factors = sf.reshape(n_tiles, TILE, 3).transpose(0, 2, 1).copy()
    ids = np.full(n_slots, -1, dtype=np.int32)
    ids[slot] = index["ids"]
    out = dict(tile_offsets=tile_off, n_tiles=n_tiles, n_slots=n_slots,
               short_codes=short_codes.reshape(-1), short_factors=short_factors.reshape(-1),
               ids=ids, long_codes=None, long_factors=None, slot=slot)
    if B > 1:
        F = long_field_bits(B)
        lw = pack_fields(index["u"], F)
        lc = np.zeros((n_slots, lw.shape[1]), dtype=np.uint32)
        lc[slot] = lw
        lfa = np.zeros((n_slots, 2), dtype=np.float32)
        lfa[slot] = index["long_factors"]
        out["long_codes"] = lc.reshape(-1)
        out["long_factors"] = lfa.reshape(-1)
    return out


def pack_ex_planes(u: np.ndarray, B: int) -> np.ndarray:
    """The long code exactly as Section 3.4.3 describes it: only the B-1 ex-bits of each dimension (the sign bit
    lives in the short code), stored as B-1 bit-planes of W words, plane j = bit j of ``u mod 2^(B-1)``:
    [n, (B-1)*W] uint32.  The library stores the whole code in F-bit fields instead (pack_fields); both are
    encodings of the same ``u`` and this function exists so that a test can show it and count the bytes."""
    n, D = u.shape
    ex = u.astype(np.uint32) & np.uint32((1 << (B - 1)) - 1)
    return np.concatenate([pack_bits((ex >> np.uint32(j)) & np.uint32(1)) for j in range(B - 1)], axis=1) \
        if B > 1 else np.zeros((n, 0), np.uint32)


def unpack_ex_planes(short_words_: np.ndarray, planes: np.ndarray, B: int, D: int) -> np.ndarray:
    """``u = 2^(B-1) u_b + u_ex`` from the short code [n, W] and the ex-bit planes [n, (B-1)*W]."""
    W = D // 32
    u = unpack_bits(short_words_, D).astype(np.uint32) << np.uint32(B - 1)
    for j in range(B - 1):
        u |= unpack_bits(planes[:, j * W:(j + 1) * W], D).astype(np.uint32) << np.uint32(j)
    return u.astype(np.uint8)


def unpack_device_layout(arr: dict) -> dict:
    """Inverse of pack_device_layout: the canonical (unpadded, cluster-ordered) index from arrays in the layout the
    search library uploads and exports (keys: dim, nlist, n, total_bits, metric, rotation, centroids, offsets,
    short_codes, short_factors, long_codes, long_factors, ids, mean).  Lets the oracle search an index that was
    built elsewhere; nothing is recomputed, every array is only re-indexed."""
    D, B, nlist, n = int(arr["dim"]), int(arr["total_bits"]), int(arr["nlist"]), int(arr["n"])
    W = D // 32
    off = np.asarray(arr["offsets"], np.int64)
    counts = np.diff(off)
    tiles = (counts + TILE - 1) // TILE
    tile_off = np.zeros(nlist + 1, dtype=np.int64)
    np.cumsum(tiles, out=tile_off[1:])
    n_tiles = int(tile_off[-1])
    within = np.arange(n, dtype=np.int64) - np.repeat(off[:-1], counts)
    slot = np.repeat(tile_off[:-1] * TILE, counts) + within
    sc = np.asarray(arr["short_codes"], np.uint32).reshape(n_tiles, W, TILE).transpose(0, 2, 1).reshape(-1, W)[slot]
    sf = np.asarray(arr["short_factors"], np.float32).reshape(n_tiles, 3, TILE).transpose(0, 2, 1).reshape(-1, 3)[slot]
    ids = np.asarray(arr["ids"], np.int32)[slot]
    if B > 1:
        F = long_field_bits(B)
        u = unpack_fields(np.asarray(arr["long_codes"], np.uint32).reshape(n_tiles * TILE, -1)[slot], F, D)
        lf = np.asarray(arr["long_factors"], np.float32).reshape(-1, 2)[slot]
        assert np.array_equal(u >> (B - 1), unpack_bits(sc, D)), "sign bit of the long code differs from the short code"
    else:
        u = unpack_bits(sc, D)
        lf = sf[:, :2].copy()
    mean = arr.get("mean")
    mean = np.zeros(D, np.float32) if mean is None else np.asarray(mean, np.float32)
    return dict(dim=D, nlist=nlist, n=n, total_bits=B, metric=arr["metric"], mean=mean,
                P=np.asarray(arr["rotation"], np.float32).reshape(D, D),
                centroids_rot=np.asarray(arr["centroids"], np.float32).reshape(nlist, D), offsets=off,
                ids=ids, u=u, short_factors=sf, long_factors=lf)
