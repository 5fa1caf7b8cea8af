"""Device-side index construction used by the benchmark and by library users.

Builds the flat IVF-RaBitQ arrays in the layout of ``rabitq_index_desc`` from raw
vectors that live on the GPU.  The pipeline follows the paper's index build
(Section 3.2): k-means on a training subset, assignment, normalisation with respect to
the centroid, rotation by P, quantisation by the two-phase grid search over the
rescaling factor (Section 3.2.2: N_coarse uniform samples, then N_fine samples around
the best one), split into 1-bit code and long code, factors.

This module is plumbing around the search path (it is not on it): it is written with
torch tensor operations on the device, one cluster-ordered chunk at a time, and shares
no code with the CPU oracle, which has its own exact encoder.
"""
from __future__ import annotations

import numpy as np
import torch

TILE = 64
N_COARSE = 64   # Section 4.1: defaults of the two-phase grid search
N_FINE = 32


def _field_bits(total_bits: int) -> int:
    """Long-code field width: B rounded up to 2, 4 or 8 (0 when there is no long code)."""
    return 0 if total_bits <= 1 else next(f for f in (2, 4, 8) if total_bits <= f)


def random_rotation(dim: int, seed: int, device) -> torch.Tensor:
    g = torch.Generator(device="cpu").manual_seed(seed)
    a = torch.randn((dim, dim), generator=g, dtype=torch.float64)
    q, r = torch.linalg.qr(a)
    q = q * torch.sign(torch.diagonal(r))[None, :]
    return q.to(torch.float32).to(device)


def _nearest(x: torch.Tensor, c: torch.Tensor, chunk: int = 65536) -> torch.Tensor:
    cn = (c * c).sum(1)
    out = torch.empty(x.shape[0], dtype=torch.int64, device=x.device)
    for s in range(0, x.shape[0], chunk):
        d = cn[None, :] - 2.0 * (x[s:s + chunk] @ c.T)
        out[s:s + chunk] = d.argmin(1)
    return out


def kmeans(x: torch.Tensor, nlist: int, iters: int, seed: int, train_size: int | None) -> torch.Tensor:
    g = torch.Generator(device="cpu").manual_seed(seed)
    n = x.shape[0]
    tr = x if (train_size is None or train_size >= n) else x[torch.randperm(n, generator=g)[:train_size].to(x.device)]
    c = tr[torch.randperm(tr.shape[0], generator=g)[:nlist].to(x.device)].clone()
    for _ in range(iters):
        a = _nearest(tr, c)
        cnt = torch.bincount(a, minlength=nlist).to(tr.dtype)
        s = torch.zeros_like(c).index_add_(0, a, tr)
        nz = cnt > 0
        c[nz] = s[nz] / cnt[nz, None]
    return c


def grid_search_codes(o_rot: torch.Tensor, total_bits: int) -> torch.Tensor:
    """Two-phase grid search over the rescaling factor t (Section 3.2.2).  For a sample t
    the closest grid point has magnitudes m+1/2 with m = min(floor(t|o'|), 2^(B-1)-1); the
    objective is <x, o'>/||x||.  The range [0, 1.5 * 2^(B-1) / max|o'|] covers every
    factor that still changes the code of the largest coordinate."""
    n, D = o_rot.shape
    half = 1 << (total_bits - 1)
    L = half - 1
    y = o_rot.abs()
    if L == 0:
        m = torch.zeros_like(y, dtype=torch.int64)
    else:
        t_end = 1.5 * half / y.max(dim=1).values.clamp_min(1e-30)          # [n]

        def best_of(ts):                                                    # ts [n, S]
            m_ = torch.clamp((ts[:, :, None] * y[:, None, :]).floor(), max=L) + 0.5
            obj = (m_ * y[:, None, :]).sum(2) / m_.square().sum(2).sqrt()
            return ts.gather(1, obj.argmax(1, keepdim=True))[:, 0]
        steps = torch.arange(1, N_COARSE + 1, device=y.device, dtype=y.dtype) / N_COARSE
        t_c = best_of(t_end[:, None] * steps[None, :])
        width = t_end / N_COARSE
        fine = torch.linspace(-1.0, 1.0, N_FINE, device=y.device, dtype=y.dtype)
        t_f = best_of((t_c[:, None] + width[:, None] * fine[None, :]).clamp_min(0.0))
        m = torch.clamp((t_f[:, None] * y).floor(), max=L).to(torch.int64)
    return torch.where(o_rot >= 0, half + m, half - 1 - m).to(torch.uint8)


def _factors(x, o_rot, c_rot, r, metric, eps0, o_dot_c):
    D = x.shape[1]
    xo = (x * o_rot).sum(1)
    xc = (x * c_rot).sum(1)
    ok = r > 0
    xo = torch.where(ok, xo, torch.ones_like(xo))
    a = (xo / x.norm(dim=1)).clamp(0.0, 1.0)
    a = torch.where(ok, a, torch.ones_like(a))
    spread = (1.0 - a * a).clamp_min(0.0).sqrt() / (a * (D - 1.0) ** 0.5)
    if metric == "l2":
        f = torch.stack([r * r + 2.0 * r * xc / xo, -2.0 * r / xo, 2.0 * r * eps0 * spread], 1)
    else:
        f = torch.stack([-o_dot_c + r * xc / xo, -r / xo, r * eps0 * spread], 1)
    f[~ok] = 0.0
    return f


def _pack_bits(bits: torch.Tensor) -> torch.Tensor:
    n, D = bits.shape
    sh = torch.arange(32, device=bits.device, dtype=torch.int64)
    w = (bits.to(torch.int64).reshape(n, D // 32, 32) << sh).sum(2)
    return w.to(torch.int64)


def _pack_fields(vals: torch.Tensor, F: int) -> torch.Tensor:
    n, D = vals.shape
    per = 32 // F
    sh = torch.arange(per, device=vals.device, dtype=torch.int64) * F
    return (vals.to(torch.int64).reshape(n, D // per, per) << sh).sum(2)


def build_index(x: torch.Tensor, nlist: int, total_bits: int, metric: str = "l2", seed_rotation: int = 7,
                seed_kmeans: int = 99, kmeans_iters: int = 10, train_size: int | None = None, eps0: float = 1.9,
                chunk: int = 8192) -> dict:
    """Returns a dict with the scalar description and HOST numpy arrays ready for
    ``rabitq.Index(**...)`` (see include/rabitq.h for the layout)."""
    assert x.dtype == torch.float32
    N, D = x.shape
    B = total_bits
    W = D // 32
    F = _field_bits(B)
    dev = x.device
    P = random_rotation(D, seed_rotation, dev)
    P64 = P.double()
    C = kmeans(x, nlist, kmeans_iters, seed_kmeans, train_size)
    assign = _nearest(x, C)
    order = torch.sort(assign, stable=True).indices
    counts = torch.bincount(assign, minlength=nlist)
    offsets = torch.zeros(nlist + 1, dtype=torch.int64, device=dev)
    offsets[1:] = counts.cumsum(0)
    tiles = (counts + TILE - 1) // TILE
    tile_off = torch.zeros(nlist + 1, dtype=torch.int64, device=dev)
    tile_off[1:] = tiles.cumsum(0)
    n_tiles = int(tile_off[-1].item())
    n_slots = n_tiles * TILE
    C64 = C.double()
    C_rot = (C64 @ P64).float()
    C_rot64 = C_rot.double()
    sorted_cid = assign[order]
    within = torch.arange(N, device=dev) - offsets[:-1][sorted_cid]
    slot = tile_off[:-1][sorted_cid] * TILE + within

    sc = torch.zeros((n_slots, W), dtype=torch.int64, device=dev)
    sf = torch.zeros((n_slots, 3), dtype=torch.float32, device=dev)
    sf[:, 0] = float("inf")
    ids = torch.full((n_slots,), -1, dtype=torch.int32, device=dev)
    ids[slot] = order.to(torch.int32)
    lc = lf = None
    if B > 1:
        lc = torch.zeros((n_slots, D * F // 32), dtype=torch.int64, device=dev)
        lf = torch.zeros((n_slots, 2), dtype=torch.float32, device=dev)
    cB = ((1 << B) - 1) / 2.0
    for s in range(0, N, chunk):
        rows = order[s:s + chunk]
        sl = slot[s:s + chunk]
        cid = sorted_cid[s:s + chunk]
        c = C64[cid]
        res = x[rows].double() - c
        r = res.norm(dim=1)
        ok = r > 0
        o = torch.where(ok[:, None], res / r.clamp_min(1e-300)[:, None], torch.zeros_like(res))
        o_rot = o @ P64
        u = grid_search_codes(o_rot, B)
        u[~ok] = 1 << (B - 1)
        c_rot = C_rot64[cid]
        odc = (c * res).sum(1)
        msb = (u >> (B - 1))
        f1 = _factors(msb.double() - 0.5, o_rot, c_rot, r, metric, eps0, odc)
        sc[sl] = _pack_bits(msb)
        sf[sl] = f1.float()
        if B > 1:
            fB = _factors(u.double() - cB, o_rot, c_rot, r, metric, eps0, odc)
            lc[sl] = _pack_fields(u, F)
            lf[sl] = fB[:, :2].float()

    def u32(t):
        return t.cpu().numpy().astype(np.uint32)
    short_codes = u32(sc.reshape(n_tiles, TILE, W).permute(0, 2, 1).contiguous()).reshape(-1)
    short_factors = sf.reshape(n_tiles, TILE, 3).permute(0, 2, 1).contiguous().cpu().numpy().reshape(-1)
    return dict(dim=D, nlist=nlist, n=N, total_bits=B, metric=metric,
                rotation=P.cpu().numpy(), centroids=C_rot.cpu().numpy(), offsets=offsets.cpu().numpy(),
                short_codes=short_codes, short_factors=short_factors, ids=ids.cpu().numpy(),
                long_codes=None if lc is None else u32(lc).reshape(-1),
                long_factors=None if lf is None else lf.cpu().numpy().reshape(-1))
