"""Runs the oracle's search, unchanged, in several worker processes (TEST INFRASTRUCTURE ONLY).

Queries are independent, so a batch is dealt to one process per host core; every worker loads the same index
arrays from a file and answers its share with oracle.search.Searcher.search.  Nothing of the method lives here."""
from __future__ import annotations

import numpy as np

_searcher = None
_SCALARS = ("dim", "nlist", "n", "total_bits")


def save_index(path: str, ix: dict) -> None:
    """Writes the arrays of an index dict (oracle.build.build_index / unpack_device_layout) to an .npz file."""
    np.savez(path, **{k: np.asarray(v) for k, v in ix.items() if v is not None})


def init(path: str) -> None:
    """Worker initialiser: loads the index written by save_index and keeps a Searcher for it."""
    global _searcher
    from .search import Searcher
    with np.load(path, allow_pickle=False) as z:
        ix = {k: z[k] for k in z.files}
    for k in _SCALARS:
        ix[k] = int(ix[k])
    ix["metric"] = str(ix["metric"])
    _searcher = Searcher(ix)


def run(job):
    """job = (queries [m, D], k, nprobe): returns the ids of the worker's share."""
    Q, k, nprobe = job
    return _searcher.search(Q, k, nprobe)[0]


def ready(_):
    return _searcher is not None
