"""CPU oracle for the per-batch graph-embedding training step.

TEST INFRASTRUCTURE ONLY.  Everything under ``oracle/`` is a plain, slow,
fp64 numpy restatement of what the training step computes (contrastive
softmax loss of Eq. 1 with sampled negatives, DistMult / ComplEx / TransE
scores of Sec. 2.1, Adagrad as named in Sec. 5.1).  It shares no code with
the HIP library and must never be imported by it.  Only the tests, the smoke
check and the benchmark's ``cpu_baseline`` leg may call into it.

Every function is pinned by the ``-m "not gpu"`` tests against closed forms,
finite differences, brute-force loops, published known-answer vectors or
library routines; none is "parity unpinned" except the whole-step composition,
for which the paper prints no worked numeric example (it is pinned by the
composition of the pinned parts plus a brute-force loop on tiny inputs).
"""
