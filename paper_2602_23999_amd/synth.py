"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random numbers: it holds none of the method's
arithmetic and is the one module that the tests hand to both the CPU oracle
and the HIP path.  The public datasets the paper measures on (Section 4.1,
Table 1) are not available here; each recipe below takes the shape, value
range and cluster structure of one of them and stands in for it.

Every generator is chunked so that the largest configuration never holds more
than one fp32 copy of the base matrix plus one chunk.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    n: int            # base vectors
    dim: int
    n_centres: int    # mixture components
    nlist: int        # IVF lists
    total_bits: int   # B
    nq: int
    k: int
    nprobes: tuple
    metric: str = "l2"
    seed_data: int = 1234
    seed_query: int = 4321

    def scaled(self, n=None, nq=None, nlist=None, n_centres=None, total_bits=None):
        kw = {}
        if n is not None: kw["n"] = n
        if nq is not None: kw["nq"] = nq
        if nlist is not None: kw["nlist"] = nlist
        if n_centres is not None: kw["n_centres"] = n_centres
        if total_bits is not None: kw["total_bits"] = total_bits
        return replace(self, **kw)


WORKLOADS = {
    # Tiny L2 case: 64 isotropic clusters, sigma 0.3, 1-bit codes.
    "tiny": Workload("tiny", 10_000, 128, 64, 64, 1, 100, 10, (8,)),
    # 128-d image-descriptor shape: non-negative integer-valued features in [0,255].
    "l2_128": Workload("l2_128", 1_000_000, 128, 1024, 1024, 4, 10_000, 10, (8, 16, 32, 64, 128)),
    # 960-d dense descriptors, anisotropic clusters.
    "l2_960": Workload("l2_960", 1_000_000, 960, 2048, 1024, 5, 1_000, 10, (16, 32, 64, 128, 256)),
    # 96-d unit-normalised deep features.
    "l2_96": Workload("l2_96", 10_000_000, 96, 16384, 16384, 3, 10_000, 100, (32, 64, 128, 256, 512)),
    # 768-d unit-norm text embeddings, maximum inner product.
    "ip_768": Workload("ip_768", 5_000_000, 768, 4096, 8192, 8, 10_000, 10, (64,), metric="ip"),
    # The same with concentrated clusters (noise norm 0.15, cos(x, centre) ~ 0.99): the literal recipe above is so
    # diffuse (cos ~ 0.25) that no list structure helps; this variant is the one with a meaningful recall.
    "ip_768_tight": Workload("ip_768_tight", 5_000_000, 768, 4096, 8192, 8, 10_000, 10, (64,), metric="ip"),
}


def _rng(seed, stream):
    return np.random.Generator(np.random.PCG64([seed, stream]))


def _centres(w: Workload) -> np.ndarray:
    r = _rng(w.seed_data, 0)
    D = w.dim
    if w.name == "tiny":
        return r.standard_normal((w.n_centres, D))
    if w.name == "l2_128":
        # Two-level mixture with low intrinsic dimension: 32 coarse modes, each with
        # its own 12-d subspace; components are scattered inside their mode's
        # subspace, so neighbouring components overlap the way descriptor clusters do
        # and a query's neighbours spread over several inverted lists.
        modes, basis, which = _l2_128_modes(w)
        z = r.standard_normal((w.n_centres, L2_128_SUBDIM)) * L2_128_CENTRE_STD
        return modes[which] + np.einsum("nk,nkd->nd", z, basis[which])
    if w.name == "l2_960":
        return r.standard_normal((w.n_centres, D))
    if w.name in ("l2_96", "ip_768", "ip_768_tight"):
        c = r.standard_normal((w.n_centres, D))
        return c / np.linalg.norm(c, axis=1, keepdims=True)
    raise KeyError(w.name)


# l2_128 recipe: std of the in-subspace component scatter, of the in-subspace point
# scatter, and of the isotropic noise added in all 128 dimensions.
L2_128_CENTRE_STD = 12.0
L2_128_LOCAL_STD = 23.0
L2_128_ISO_STD = 1.5
L2_128_SUBDIM = 12


def _l2_128_modes(w: Workload):
    r = _rng(w.seed_data, 7)
    D = w.dim
    modes = np.clip(r.normal(36.0, 26.0, (32, D)), 0.0, None)
    basis = np.stack([np.linalg.qr(r.standard_normal((D, L2_128_SUBDIM)))[0].T for _ in range(32)])
    which = r.integers(0, 32, w.n_centres)
    return modes, basis, which


def _draw(w: Workload, centres: np.ndarray, n: int, seed: int, stream: int, chunk: int = 65536) -> np.ndarray:
    D = w.dim
    out = np.empty((n, D), dtype=np.float32)
    aux = _rng(w.seed_data, 1)
    if w.name == "l2_960":
        scales = np.sqrt(aux.uniform(0.1, 1.0, (w.n_centres, D)))  # per-cluster diagonal std
    if w.name == "l2_128":
        _, basis, which = _l2_128_modes(w)
    r = _rng(seed, stream)
    for s in range(0, n, chunk):
        m = min(chunk, n - s)
        comp = r.integers(0, w.n_centres, m)
        g = r.standard_normal((m, D))
        if w.name == "tiny":
            x = centres[comp] + 0.3 * g
        elif w.name == "l2_128":
            z = r.standard_normal((m, L2_128_SUBDIM)) * L2_128_LOCAL_STD
            x = centres[comp] + np.einsum("nk,nkd->nd", z, basis[which[comp]]) + L2_128_ISO_STD * g
            x = np.rint(np.clip(x, 0.0, 255.0))
        elif w.name == "l2_960":
            x = centres[comp] + scales[comp] * g
        elif w.name == "l2_96":
            x = centres[comp] + (0.5 / np.sqrt(D)) * g
            x /= np.linalg.norm(x, axis=1, keepdims=True)
        elif w.name == "ip_768":
            x = centres[comp] + g / np.sqrt(50.0)  # tangent variance 1/kappa, kappa = 50
            x /= np.linalg.norm(x, axis=1, keepdims=True)
        elif w.name == "ip_768_tight":
            x = centres[comp] + (0.15 / np.sqrt(D)) * g
            x /= np.linalg.norm(x, axis=1, keepdims=True)
        else:
            raise KeyError(w.name)
        out[s:s + m] = x.astype(np.float32)
    return out


def make_base(w: Workload) -> np.ndarray:
    """Base vectors [n, dim] fp32."""
    return _draw(w, _centres(w), w.n, w.seed_data, 2)


def make_queries(w: Workload, nq: int | None = None) -> np.ndarray:
    """Fresh draws from the same mixture [nq, dim] fp32."""
    return _draw(w, _centres(w), w.nq if nq is None else nq, w.seed_query, 3)
