"""CPU oracle for the GossipGraD data-parallel hot path (arXiv 1803.05880).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, obviously-correct
restatement of what the hot path computes, written from the paper's
definitions.  It shares no code with the HIP library and imports nothing from
it.  Only the test-suite, the smoke check and the benchmark's cpu-baseline leg
may import it; the product path never does.

Modules
  philox    counter-based generator used for every random draw of the method
  schedule  shuffled communicators, hypercube / dissemination partner maps,
            partner rotation                      (Sec. 4.3, 4.4, 4.5.1)
  gossip    momentum-SGD update, pairwise model averaging, the staleness-1
            and gradient-averaging variants, the recursive-doubling
            all-reduce comparator                 (Eq. 1-2, Sec. 3.1, Sec. 6)
  shuffle   sample-index rotation: ring of used batches and the
            partner-swap variant                  (Sec. 4.5.2, Lemma 1)

Pin status (see tests/test_oracle_*.py): every function is pinned by closed
forms, invariants, brute force or a library routine, except the raw Philox
word stream, which is pinned only structurally (Weyl constants by closed form,
round invertibility, two independently written implementations, statistical
uniformity): "parity unpinned" for the literal word values.  Nothing else
depends on the literal values -- the method needs *a* deterministic stream.
"""
