"""oracle.parallel runs the unchanged oracle search in worker processes: same answers as the serial run, on an index
that went through the device layout and back (CPU only)."""
import multiprocessing as mp
import os
import tempfile

import numpy as np

from oracle import build, parallel, search
from paper_2602_23999_amd import synth


def test_worker_processes_give_the_serial_answers():
    w = synth.WORKLOADS["l2_128"].scaled(n=6000, nq=24, n_centres=32)
    X, Q = synth.make_base(w), synth.make_queries(w)
    ix = build.build_index(X, 16, 4, kmeans_iters=3, center=True)
    dev = build.pack_device_layout(ix)
    arr = dict(dim=128, nlist=16, n=ix["n"], total_bits=4, metric="l2", rotation=ix["P"].reshape(-1),
               centroids=ix["centroids_rot"].reshape(-1), offsets=ix["offsets"], short_codes=dev["short_codes"],
               short_factors=dev["short_factors"], long_codes=dev["long_codes"], long_factors=dev["long_factors"],
               ids=dev["ids"], mean=ix["mean"])
    back = build.unpack_device_layout(arr)
    want = search.Searcher(ix).search(Q, 10, 4)[0]
    with tempfile.TemporaryDirectory() as tmp:
        path = os.path.join(tmp, "index.npz")
        parallel.save_index(path, back)
        with mp.get_context("spawn").Pool(2, initializer=parallel.init, initargs=(path,)) as pool:
            parts = np.array_split(np.arange(len(Q)), 2)
            got = pool.map(parallel.run, [(Q[p], 10, 4) for p in parts])
    assert np.array_equal(np.concatenate(got), want)
