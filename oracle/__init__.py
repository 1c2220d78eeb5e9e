"""CPU oracle for the CodedReduce hot path.  TEST INFRASTRUCTURE ONLY.

Everything under this package is a slow, plain, fp64 (or exact-rational)
restatement of what the method computes, written from the paper.  It shares no
code with the HIP library and must never be imported by the product path:
only the tests, the smoke check and the benchmark's CPU-baseline leg use it.

Modules
-------
gc_code   gradient-coding matrices B (encoding) and A (decoding), Section II-C
cr_tree   (n,L)-regular tree, CompAlloc (Algorithm 1), CR.Allocate and
          CR.Execute (Algorithm 2), the computation load of Theorem 1, and the
          plain definition of the full gradient, eq. (3)
native    ctypes wrapper around cr_native.c: the same per-segment gradient
          loops in plain C with OpenMP, for inputs too large for numpy temporaries
"""
