"""CPU oracle for the RetrievalAttention decode hot path and its index build.

TEST INFRASTRUCTURE ONLY. This package is a plain, slow, obviously-correct CPU
statement of what the HIP library computes, written from the paper
(arXiv 2409.10516). It shares no code with the HIP path and imports nothing from
the product package; only tests, the smoke check and the benchmark's CPU-baseline
leg may import it. The product never falls back to it.

Modules, each function citing the passage it follows:
  attention.py   Eq. 1 (softmax attention), Eq. 2 (sparse attention over a subset),
                 Appendix A Eq. 4-5 (two-set combination), static pattern of Sec. 3.3.
  mips.py        inner-product order, brute-force top-k ("Flat", Sec. 4.1), exact KNN
                 of Sec. 3.2 / Fig. 2b, recall as defined in Sec. 2.4.
  projection.py  KNN-to-key-graph projection of Sec. 3.2. The paper gives this step
                 one sentence; the reading implemented here is documented in the
                 module header. PARITY UNPINNED by the paper (no worked example): it
                 is pinned by brute-force recounts, invariants and a hand-worked case.
  search.py      greedy best-first graph search (Sec. 2.4 describes it in a clause;
                 beam width, expansion width and tie-breaking are this build's).
  decode.py      Algorithm 1 for the fixed static pattern: search, sparse attention
                 over the retrieved set, dense attention over the static set, combine.
"""
