"""CPU oracle for the IVF-RaBitQ batched-search path.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, double-precision
restatement of what the search path computes (index construction included,
because the index defines the codes both sides read).  Only the test-suite,
the smoke check and the benchmark's CPU-baseline leg may import it; the HIP
library and its Python binding never do, and share no code with it.

Modules
-------
build   k-means IVF, random rotation, exact RaBitQ B-bit encoding, per-vector
        factors, and the packing of the flat index arrays.
search  query rotation, coarse probing, 4-bit query quantisation, bit-plane
        inner products, 1-bit / refined estimators, threshold seeding and top-k.
exact   brute-force k-nearest neighbours and recall.

Parity status of every function is listed in the header of its module.
"""
