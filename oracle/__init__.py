"""CPU oracle for the matmul sumcheck prover -- TEST INFRASTRUCTURE ONLY.

This package is the slow, obviously-correct definition of what the GPU path
must compute.  It is imported only by the test-suite, by the smoke check and
by the CPU-baseline leg of the benchmark; the product library never calls it
and shares no code, tables or helpers with it.

Two tiers, both written from the definitions (not from the GPU code):

* ``oracle.reference`` -- tier 0, pure Python integers.  Every quantity is the
  textbook formula written out: multilinear extension by explicit summation,
  round polynomials by summation over the boolean cube, SHA-256 through
  ``hashlib``.
* ``oracle.fast`` + ``oracle/native/imm_oracle.c`` -- tier 1, plain C using
  ``unsigned __int128`` and ``%`` for every field operation, row loops spread
  over host threads.  Validated bit-for-bit against tier 0 before it is used
  for the larger workloads.

The paper (sections 2.1, 2.2, 5.2 and the VC algorithm in the appendix) only
requires *that* the reference model's continuous transformations are proven
with a (Prove, Vrfy) pair over hash commitments; it prints no proof system.
The protocol implemented here is the standard sumcheck for matrix products
over the Goldilocks field; the concrete conventions (variable order,
transcript bytes, padding) are listed at the top of ``oracle/reference.py``.

Parity pins: every function here is pinned by tests that do not re-type its
formula (hand-computed worked examples over the integers, boolean-point
identities, affine-in-each-variable checks, brute force on 4x4x4, hashlib).
No function is "parity unpinned".
"""
