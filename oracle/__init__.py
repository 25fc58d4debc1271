"""TEST INFRASTRUCTURE: fp64 CPU oracle for Recurrent Hybrid Attention (ReHyAt).

Two independent evaluations of the paper's operator:

* ``oracle.brute``  -- numpy, the defining double sum of section 3.2 (Eq. 5-9
  with the token sets of Eq. 10-13) written out per query token; O(N^2), tiny
  inputs only.
* ``oracle.cref``   -- plain C (``rehyat_oracle.c``), the chunk-wise RNN of
  section 3.3 (Eq. 14-18); usable at the full video shapes.

Neither imports, links or shares code with the GPU library.  Only tests, the
smoke check and the benchmark's ``cpu_baseline`` leg may use this package; the
product path never does.

Readings the paper does not fix (stabiliser per row, per-head 1/sqrt(d), ReLU
in phi, layer widths) are marked "parity unpinned" in ``rehyat_oracle.c``.
"""
