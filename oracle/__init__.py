"""CPU oracle for the Product Quantization Tree (PQT) query path.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, float64 statement of
what the query path computes, written from the paper's text.  It shares no
code with the HIP library or its Python binding and imports neither.  Only
the test-suite, the smoke check and the benchmark's CPU-baseline leg may use
it; the product never routes through it.

Modules
  pqt_query     the online phase, steps O1..O9 (Sec. 3.2, 3.3 "Online computation")
  pqt_build     a plain offline builder (Sec. 3.1, 3.3 "Offline computation", Sec. 4)
  pqt_index_io  reader/writer of the index file both sides load

Parity pins (tests marked "not gpu"): brute force (Eq. 1) under exhaustive
settings, bins are a partition of the database, the triangulation identity of
Eq. 9 against explicit reconstruction, closed forms of Eq. 9 at lambda in
{0, 1/2, 1}, full-sort vs priority-queue bin order, counts of Sec. 3.1/3.2, and
library sorts/cdist for the elementary steps.  Every function here has at
least one such pin; none is "parity unpinned".  The paper's printed tables
depend on SIFT1M/GIST1M/SIFT1B, which are not available: unpinned.
"""
