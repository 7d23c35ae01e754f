"""CPU oracle for the VarDrop training hot path (test infrastructure only).

A plain, slow, fp64 NumPy statement of what the hot path computes, written from
the paper's method section (Alg. 1, Def. 1, Eq. 1-3; the token embedding of the kept
variates after the backbone of Sec. 4.1) and from the published
definition of Philox4x32-10 (Salmon et al., SC'11).  It exists so that the GPU
library can be checked against something that shares no code with it.

Rules of use:
  * only the test-suite, the smoke check and the CPU-baseline leg of the
    benchmark may import this package; the product never does;
  * nothing here imports the GPU package, and no expected value in here or in
    the tests was produced by the GPU path.

Every function is pinned by CPU-only tests against closed forms, printed facts
of the paper, library routines and brute force; none is "parity unpinned".
The choices the paper leaves open (hash encoding, group numbering, random
generator, tie-breaks) are conventions of this repository; they are stated in
each docstring.
"""
